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

#include <hip/hip_cooperative_groups.h>

#include <algorithm>
#include <cfloat>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <type_traits>

// Scratch block of lqsgd_step_static (see static_scratch() below): device memory that is part of
// the code object, one copy per GPU.  In host code this name is a handle for hipGetSymbolAddress,
// never an address.
static __device__ __align__(256) unsigned char scratch[LQSGD_STATIC_SCRATCH_BYTES];

namespace lqsgd {
namespace {

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
typedef float v4f __attribute__((ext_vector_type(4)));
// Loads through a pointer in the constant address space are assumed not to
// change while the kernel runs; with a wave-uniform address they become
// scalar loads (one fetch per wavefront, no vector register traffic).  Used
// for factor rows that an earlier kernel wrote.
typedef const float __attribute__((address_space(4)))* const_fp;

// Streaming hints: data that is read once (gradients, residual) is loaded
// with the non-temporal hint so that it does not displace the factor panels.
#ifndef LQSGD_NT_G
#define LQSGD_NT_G 1
#endif
#ifndef LQSGD_NT_E          // residual sweeps (eager schedule); sweep 0 follows its store policy, see add_project_kernel
#define LQSGD_NT_E 1
#endif
#ifndef LQSGD_NT_M
#define LQSGD_NT_M 1
#endif
#ifndef LQSGD_RT           // rows a wavefront carries through one column pass of sweep 0 (rank <= 8)
#define LQSGD_RT 8
#endif
#ifndef LQSGD_BM_U2
#define LQSGD_BM_U2 4  // the same for the form with two blocks of 32 ranks (rank pad 64)
#endif
#ifndef LQSGD_BM_U
#define LQSGD_BM_U 8   // pairs of rows per step of the matrix-core sweep 1 (4: 829 us, 8: 750 us, 16: 833 us at 8192^2 x 16)
#endif
#ifndef LQSGD_BQ_LATE      // matrix-core sweep 0, fused mode: fetch the P product's Q slice after the G-hat part
#define LQSGD_BQ_LATE 1
#endif
#ifndef LQSGD_B_U          // rows a wavefront of sweep 1 has in flight
#define LQSGD_B_U 8
#endif
#ifndef LQSGD_B_INTERLEAVE  // sweep 1: row blocks of at least this many rows are split between the wavefronts in groups of LQSGD_B_U rows
#define LQSGD_B_INTERLEAVE 512
#endif
#ifndef LQSGD_A_WAVES      // occupancy target of sweep 0 (waves per SIMD)
#define LQSGD_A_WAVES 1
#endif

template <int V>
struct Pk {
  float v[V];
};

// Every tensor the kernels touch lives in device memory, but a pointer fetched from a pointer table
// (the caller's gradient and output tensors) is a generic one as far as the compiler knows, and it
// would use flat-address instructions for it, which complete out of order with the global ones and
// force every wait to be a wait for everything.  The streaming loads and stores say "global" outright.
template <typename T>
__device__ __forceinline__ const T __attribute__((address_space(1)))* gptr(const void* p) {
  return (const T __attribute__((address_space(1)))*)p;
}
template <typename T>
__device__ __forceinline__ T __attribute__((address_space(1)))* gptr(void* p) {
  return (T __attribute__((address_space(1)))*)p;
}

// VEC floats at (wave-uniform row base) + (per-lane byte offset).
template <int V, bool NT>
__device__ __forceinline__ Pk<V> ldrow(const char* rowbase, unsigned boff);
template <>
__device__ __forceinline__ Pk<4> ldrow<4, false>(const char* rowbase, unsigned boff) {
  const v4f t = *gptr<v4f>(rowbase + boff);
  return Pk<4>{{t.x, t.y, t.z, t.w}};
}
template <>
__device__ __forceinline__ Pk<4> ldrow<4, true>(const char* rowbase, unsigned boff) {
  const v4f t = __builtin_nontemporal_load(gptr<v4f>(rowbase + boff));
  return Pk<4>{{t.x, t.y, t.z, t.w}};
}
template <>
__device__ __forceinline__ Pk<1> ldrow<1, false>(const char* rowbase, unsigned boff) {
  return Pk<1>{{*gptr<float>(rowbase + boff)}};
}
template <>
__device__ __forceinline__ Pk<1> ldrow<1, true>(const char* rowbase, unsigned boff) {
  return Pk<1>{{__builtin_nontemporal_load(gptr<float>(rowbase + boff))}};
}
// The same for a row of bfloat16 values (gradients handed over in bfloat16): boff is the byte
// offset the fp32 loaders would use; a bfloat16 is the upper half of the float it stands for.
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
template <int V, bool NT>
__device__ __forceinline__ Pk<V> ldrow_bf16(const char* rowbase, unsigned boff) {
  Pk<V> r;
  if constexpr (V == 4) {
    const auto* p = gptr<v2u>(rowbase + (boff >> 1));
    const v2u t = NT ? __builtin_nontemporal_load(p) : *p;
    r.v[0] = __uint_as_float(t.x << 16); r.v[1] = __uint_as_float(t.x & 0xffff0000u);
    r.v[2] = __uint_as_float(t.y << 16); r.v[3] = __uint_as_float(t.y & 0xffff0000u);
  } else {
    const unsigned short t = *gptr<unsigned short>(rowbase + (boff >> 1));
    r.v[0] = __uint_as_float((unsigned)t << 16);
  }
  return r;
}
// Gradient row in either format.
template <int V, bool NT, bool GB16>
__device__ __forceinline__ Pk<V> ldgrad(const char* rowbase, unsigned boff) {
  if constexpr (GB16) return ldrow_bf16<V, NT>(rowbase, boff);
  else return ldrow<V, NT>(rowbase, boff);
}
// Start of gradient row `off / cols` given its element offset.
template <bool GB16>
__device__ __forceinline__ const char* grad_row(const float* G, size_t off) {
  return reinterpret_cast<const char*>(G) + off * (GB16 ? 2 : 4);
}
template <bool GB16>
__device__ __forceinline__ float grad_elem(const float* G, size_t idx) {
  if constexpr (GB16) return __uint_as_float((unsigned)gptr<unsigned short>(G)[idx] << 16);
  else return gptr<float>(G)[idx];
}

template <int V, bool NT>
__device__ __forceinline__ void strow(char* rowbase, unsigned boff, const Pk<V>& x);
template <>
__device__ __forceinline__ void strow<4, false>(char* rowbase, unsigned boff, const Pk<4>& x) {
  const v4f t = {x.v[0], x.v[1], x.v[2], x.v[3]};
  *gptr<v4f>(rowbase + boff) = t;
}
template <>
__device__ __forceinline__ void strow<4, true>(char* rowbase, unsigned boff, const Pk<4>& x) {
  const v4f t = {x.v[0], x.v[1], x.v[2], x.v[3]};
  __builtin_nontemporal_store(t, gptr<v4f>(rowbase + boff));
}
template <>
__device__ __forceinline__ void strow<1, false>(char* rowbase, unsigned boff, const Pk<1>& x) {
  *gptr<float>(rowbase + boff) = x.v[0];
}
template <>
__device__ __forceinline__ void strow<1, true>(char* rowbase, unsigned boff, const Pk<1>& x) {
  __builtin_nontemporal_store(x.v[0], gptr<float>(rowbase + boff));
}

// Factor slice of VEC consecutive columns starting at column c of a cols x r
// row-major factor F, as s[v*RP + k].  EXACT (r == RP) is the fast path.
// Output of the reconstruction G-hat = P-bar Q-bar^T (Eq. (7)): either stored as it is, or applied
// to the caller's parameters, w <- w - eta G-hat (Algorithm 1, "Model update"; Eq. (2)).
template <int V>
__device__ __forceinline__ void emit_ghat(float* __restrict__ rowbase, unsigned boff, Pk<V> gh, int update, float eta) {
  if (update) {
    const Pk<V> w = ldrow<V, false>(reinterpret_cast<const char*>(rowbase), boff);
#pragma unroll
    for (int v = 0; v < V; ++v) gh.v[v] = fmaf(-eta, gh.v[v], w.v[v]);
    strow<V, false>(reinterpret_cast<char*>(rowbase), boff, gh);
  } else {
    strow<V, true>(reinterpret_cast<char*>(rowbase), boff, gh);
  }
}

// x where `on`, else +0: a bit mask instead of a select, so that the compiler cannot turn the
// unconditional load that produced x back into a branch around a conditional one
__device__ __forceinline__ float keep_if(float x, bool on) {
  return __uint_as_float(__float_as_uint(x) & (on ? 0xffffffffu : 0u));
}

// Ranks that do not fill their pad (r < RP): the loaders below still fetch RP values per factor
// row, unconditionally, running up to RP - 1 elements into what follows the row (the next row, or
// the slack the host leaves after every factor buffer), and zero the surplus afterwards.
template <int RP, int VEC, bool EXACT>
__device__ __forceinline__ void load_slice(const float* __restrict__ F, int c, int r, float (&s)[VEC * RP]) {
  if constexpr (EXACT) {
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
      for (int k = 0; k < RP; ++k) s[v * RP + k] = keep_if(F[(size_t)(c + v) * r + k], k < r);
  }
}

template <int RP, int VEC, bool EXACT>
__device__ __forceinline__ void store_slice(float* __restrict__ F, int c, int r, const float (&s)[VEC * RP]) {
  if constexpr (EXACT) {
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

// Row of a rows x r factor into p[k] (zero beyond r), plain loads.
template <int RP>
__device__ __forceinline__ void load_row(const float* __restrict__ F, int row, int r, bool exact, float (&p)[RP]) {
  if (exact) {
    const float* b = F + (size_t)row * RP;
#pragma unroll
    for (int k = 0; k < RP; ++k) p[k] = b[k];
  } else {
    const float* b = F + (size_t)row * r;
#pragma unroll
    for (int k = 0; k < RP; ++k) p[k] = keep_if(b[k], k < r);
  }
}

// Wave-uniform row of a factor written by an earlier kernel: scalar loads.
template <int RP, bool EXACT>
__device__ __forceinline__ void load_row_uniform(const float* F, int row, int r, float (&p)[RP]) {
  if constexpr (EXACT) {
    const_fp b = (const_fp)(F + (size_t)row * RP);
#pragma unroll
    for (int k = 0; k < RP; ++k) p[k] = b[k];
  } else {
    const_fp b = (const_fp)(F + (size_t)row * r);
    float t[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) t[k] = b[k];
#pragma unroll
    for (int k = 0; k < RP; ++k) p[k] = keep_if(t[k], k < r);
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
constexpr int pow2ceil(int n) { return n <= 1 ? 1 : 2 * pow2ceil((n + 1) / 2); }

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order.
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// The absmax cells that later kernels of the iteration raise with atomic maxima start from zero:
// absmax(Q_w) always (sweep 1 or the reduce that follows it), absmax of the raw P_w in the
// aggregate-first order.  Called by the first workgroup of sweep 0, which nothing of this iteration
// that touches those cells can overtake.
__device__ __forceinline__ void zero_absmax_cells(const DevArgs& a, int nthreads) {
  for (int i = threadIdx.x; i < a.W * a.L; i += nthreads) {
    a.scaleQ[i] = 0.0f;
    if (a.agg_first) a.scaleP[i] = 0.0f;
  }
}

// ---------------------------------------------------------------------------
// sweep 0: M = G + E (Eq. (9)),  P_w partial = M_w Q  (Algorithm 1, "P <- G'Q")
// One wavefront per work item: rows [row0, row0+nrows) x columns [col0, col1),
// RT rows at a time; a lane accumulates RT x r partial dot products over its
// columns, one butterfly per row group adds them over the lanes.
// ---------------------------------------------------------------------------
template <int RP, int VEC, int RT, bool EXACT, bool FULL, bool FUSE, bool GB16, bool NTS>
__device__ __forceinline__ void add_project_cols(const char* const (&gr)[RT], char* const (&mr)[RT],
                                                 const float* __restrict__ Q, const float (&pb)[RT * RP], int r, int nr,
                                                 int cbeg, int cend, float (&acc)[RT * RP]) {
  for (int c = cbeg; c < cend; c += kWave * VEC) {
    float q[VEC * RP];
    load_slice<RP, VEC, EXACT>(Q, c, r, q);
    const unsigned boff = (unsigned)c * 4u;
    Pk<VEC> g[RT], e[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      if (FULL || t < nr) {
        g[t] = ldgrad<VEC, LQSGD_NT_G != 0, GB16>(gr[t], boff);
        e[t] = ldrow<VEC, NTS>(mr[t], boff);
      } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v) { g[t].v[v] = 0.0f; e[t].v[v] = 0.0f; }
      }
    }
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      Pk<VEC> m;
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        float ev = e[t].v[v];
        if constexpr (FUSE) {
          // the buffer still holds last iteration's M: E = M - P-bar Q-bar^T (Eq. (8)),
          // with the same operation order as the stand-alone residual sweep
          float gh = 0.0f;
#pragma unroll
          for (int k = 0; k < RP; ++k) gh = fmaf(pb[t * RP + k], q[v * RP + k], gh);
          ev = ev - gh;
        }
        m.v[v] = g[t].v[v] + ev;
      }
      if (FULL || t < nr) strow<VEC, NTS>(mr[t], boff, m);
#pragma unroll
      for (int v = 0; v < VEC; ++v)
#pragma unroll
        for (int k = 0; k < RP; ++k) acc[t * RP + k] = fmaf(m.v[v], q[v * RP + k], acc[t * RP + k]);
    }
  }
}

template <int RP, int VEC, int RT, bool EXACT, bool FUSE, bool GB16 = false, bool NTS = false>
__device__ __forceinline__ void add_project_tile(const float* __restrict__ G, float* __restrict__ M,
                                                 const float* __restrict__ Q, const float* Pb,
                                                 float* __restrict__ Pp, int cols, int r, int row0, int nrows,
                                                 int col0, int col1, int lane) {
  constexpr int N = RT * RP;
  for (int rg = 0; rg < nrows; rg += RT) {
    const int nr = min(RT, nrows - rg);
    float acc[N];
    float pb[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.0f;
    const char* gr[RT];
    char* mr[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      const int row = row0 + rg + min(t, nr - 1);
      const size_t off = (size_t)row * cols;
      gr[t] = grad_row<GB16>(G, off);
      mr[t] = reinterpret_cast<char*>(M + off);
      if constexpr (FUSE) {
        float p[RP];
        load_row_uniform<RP, EXACT>(Pb, row, r, p);
#pragma unroll
        for (int k = 0; k < RP; ++k) pb[t * RP + k] = p[k];
      } else {
#pragma unroll
        for (int k = 0; k < RP; ++k) pb[t * RP + k] = 0.0f;
      }
    }
    if (nr == RT)
      add_project_cols<RP, VEC, RT, EXACT, true, FUSE, GB16, NTS>(gr, mr, Q, pb, r, nr, col0 + lane * VEC, col1, acc);
    else
      add_project_cols<RP, VEC, RT, EXACT, false, FUSE, GB16, NTS>(gr, mr, Q, pb, r, nr, col0 + lane * VEC, col1, acc);
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

// FUSE: the residual update of the previous iteration has been deferred; the
// buffer holds M_{t-1} and this sweep forms E_{t-1} = M_{t-1} - P-bar Q-bar^T on
// the fly (Q-bar is the warm-start Q this sweep multiplies by anyway).
// NTS: the residual slabs are streamed -- E (or last iteration's M) is read with the non-temporal
// hint and M is written with non-temporal stores; chosen by the host from the size of the working set.
template <int RP, bool FUSE, bool GB16, bool NTS>
__global__ __launch_bounds__(256, LQSGD_A_WAVES) void add_project_kernel(DevArgs a, const Tile* __restrict__ tiles, int ntiles, int reverse) {
  constexpr int RT = (RP <= 8) ? LQSGD_RT : 4;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  if (blockIdx.x == 0) zero_absmax_cells(a, 256);
  const int t = blockIdx.x * 4 + wave;
  if (t >= ntiles) return;
  const Tile tl = tiles[reverse ? ntiles - 1 - t : t];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const float* G = a.grads[(size_t)worker * a.n_all + ld.gidx];
  float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  const float* Q = a.Qbar + ld.q_off;
  const float* Pb = a.Pbar + ld.p_off;
  float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + ld.ppart_off + (size_t)tl.aux * ld.np_pad;
  const int col0 = tl.aux * ld.segw;
  const int col1 = min(ld.cols, col0 + ld.segw);
  if (ld.vec == 4) {
    if (ld.r == RP)
      add_project_tile<RP, 4, RT, true, FUSE, GB16, NTS>(G, M, Q, Pb, Pp, ld.cols, ld.r, tl.row0, tl.nrows, col0, col1, lane);
    else
      add_project_tile<RP, 4, RT, false, FUSE, GB16, NTS>(G, M, Q, Pb, Pp, ld.cols, ld.r, tl.row0, tl.nrows, col0, col1, lane);
  } else {
    // rows that are not 16-byte aligned (cols % 4 != 0): tiny layers, one generic path
    add_project_tile<RP, 1, RT, false, FUSE, GB16, NTS>(G, M, Q, Pb, Pp, ld.cols, ld.r, tl.row0, tl.nrows, col0, col1, lane);
  }
}

// ---------------------------------------------------------------------------
// LogQuantize of Section 4.1 for one value and for a packed group of 8 (used by
// the exchange kernels, by the Gram-Schmidt kernels that quantise their own
// output, and by the sweeps that dequantise packets themselves).
// The code of u = |x|/s is the number of decision thresholds <= u, i.e.
// nearest-level rounding in the q-domain of Eq. (5): a hardware log2 gives the
// level to within one, the two loops move it to the exact count.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int quantise_one(float u, float alpha, float qscale, int lv, const float* s_thr) {
  const float t = __log2f(fmaf(alpha, u, 1.0f)) * qscale;
  int k = (int)(t + 0.5f);
  k = max(0, min(lv, k));
  while (k < lv && s_thr[k] <= u) ++k;
  while (k > 0 && s_thr[k - 1] > u) --k;
  return k;
}

// One group of kXGroup consecutive factor elements of one worker: LogQuantize against the worker's
// absmax s (codes: number of thresholds <= |x| / s; sign bit only on a non-zero code), the packed
// group (`bits` magnitude bytes, one sign byte) stored if STORE, and the dequantised values
// (Eq. (6): +-s level_k) in val.
template <bool STORE>
__device__ __forceinline__ void quantise_group(const float (&x)[kXGroup], float s, int bits, int lv, float alpha, float qscale,
                                               const float* s_thr, const float* s_lev, uint8_t* mp, uint8_t* sp,
                                               float (&val)[kXGroup]) {
  unsigned long long magbits = 0;
  unsigned sgnbits = 0;
#pragma unroll
  for (int i = 0; i < kXGroup; ++i) {
    const int k = (s > 0.0f) ? quantise_one(fabsf(x[i]) / s, alpha, qscale, lv, s_thr) : 0;
    magbits |= (unsigned long long)k << (i * bits);
    if (x[i] < 0.0f && k > 0) sgnbits |= 1u << i;
  }
  if constexpr (STORE) {
    if (bits == 8) {
      *reinterpret_cast<unsigned long long*>(mp) = magbits;
    } else if (bits == 4) {
      *reinterpret_cast<unsigned*>(mp) = (unsigned)magbits;
    } else if (bits == 2) {
      *reinterpret_cast<unsigned short*>(mp) = (unsigned short)magbits;
    } else {
      for (int bb = 0; bb < bits; ++bb) mp[bb] = (uint8_t)(magbits >> (8 * bb));
    }
    *sp = (uint8_t)sgnbits;
  }
#pragma unroll
  for (int i = 0; i < kXGroup; ++i) {
    const int k = (int)((magbits >> (i * bits)) & (unsigned long long)lv);
    const float v = s * s_lev[k];
    val[i] = ((sgnbits >> i) & 1u) ? -v : v;
  }
}

// ---------------------------------------------------------------------------
// orth: P_w = sum of the column-segment partials; modified Gram-Schmidt
// (Algorithm 1, "Orthonormalize"), right-looking: column j is normalised, then
// removed from every later column, which applies the projections to a column
// in the same order as the left-looking form.  One workgroup per (layer,
// worker); a lane owns rows tid, tid+256, ... through all passes, so the only
// communication is the block-wide sums.  Ends with absmax(P_w) -> scaleP.
// In the aggregate-first order (orth_shared) the same kernels run once per layer
// on the aggregated factor: input = one plane at P-bar, output in place, the
// un-orthonormalised aggregate kept where `Ppre` points, no absmax.
// ---------------------------------------------------------------------------
template <int RP>
__global__ __launch_bounds__(256) void orth_kernel(DevArgs a) {
  __shared__ float red[2][4][RP];
  __shared__ float redmax[4];
  const int lw = blockIdx.x;
  const int layer = lw / a.W, worker = lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const int rows = ld.rows, r = ld.r, nseg = a.orth_shared ? 1 : ld.nseg;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + (a.orth_shared ? ld.p_off : ld.ppart_off);
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
  if (tid == 0 && !a.orth_shared)
    a.scaleP[(size_t)worker * a.L + layer] = fmaxf(fmaxf(redmax[0], redmax[1]), fmaxf(redmax[2], redmax[3]));
}

// ---------------------------------------------------------------------------
// orth, register-resident: the same computation for layers of at most
// BS * RPT rows; a lane keeps its RPT rows in registers through all passes and
// only the block-wide sums go through LDS (one barrier per column).
// ---------------------------------------------------------------------------
template <int RP, int RPT, int BS>
__global__ __launch_bounds__(BS) void orth_reg_kernel(DevArgs a) {
  constexpr int NW = BS / kWave;
  constexpr int LG = log2c(RP);
  __shared__ float red[2][NW][RP];
  __shared__ float redmax[NW];
  const int lw = blockIdx.x;
  const int layer = lw / a.W, worker = lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const int rows = ld.rows, r = ld.r, nseg = a.orth_shared ? 1 : ld.nseg;
  const bool exact = (r == RP);
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + (a.orth_shared ? ld.p_off : ld.ppart_off);
  float* pre = a.Ppre + (size_t)worker * a.p_stride + ld.p_off;
  float* orth = a.Porth + (size_t)worker * a.p_stride + ld.p_off;

  float v[RPT][RP];
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int row = tid + i * BS;
#pragma unroll
    for (int k = 0; k < RP; ++k) v[i][k] = 0.0f;
    if (row < rows) {
      for (int s = 0; s < nseg; ++s) {
        float t[RP];
        load_row<RP>(Pp + (size_t)s * ld.np_pad, row, r, exact, t);
#pragma unroll
        for (int k = 0; k < RP; ++k) v[i][k] += t[k];
      }
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k < r) pre[(size_t)row * r + k] = v[i][k];
    }
  }

  // The column index must reach every use as a constant, so that the rows stay in registers (a
  // run-time index would move v to scratch memory).  Up to rank pad 16 unrolling does that; at rank
  // pad 32 the loop is too large to be unrolled on request, and each column is an instantiation.
  if constexpr (RP >= 32) {
    static_for<RP>([&](auto jc) __attribute__((always_inline)) {
      constexpr int j = decltype(jc)::value;
      // only the products with columns j .. RP - 1 are needed: they lie in the last N columns,
      // N the next power of two (the width the butterfly below needs)
      constexpr int N = pow2ceil(RP - j), K0 = RP - N, LGN = log2c(N);
      if (j < r) {
        float s[N];
#pragma unroll
        for (int k = 0; k < N; ++k) s[k] = 0.0f;
#pragma unroll
        for (int i = 0; i < RPT; ++i)
#pragma unroll
          for (int k = 0; k < N; ++k) s[k] = fmaf(v[i][j], v[i][K0 + k], s[k]);
        transpose_reduce<N, N, 32>(s, lane);
        const int b = j & 1;
        if ((lane & (kWave / N - 1)) == 0) red[b][wave][K0 + (lane >> (6 - LGN))] = s[0];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < N; ++k) {
          float t = 0.0f;
#pragma unroll
          for (int wv = 0; wv < NW; ++wv) t += red[b][wv][K0 + k];
          s[k] = t;
        }
        const float nrm2 = s[j - K0];
        const float inv = (nrm2 > FLT_MIN) ? 1.0f / sqrtf(nrm2) : 0.0f;
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
          const float qv = v[i][j] * inv;
          v[i][j] = qv;
#pragma unroll
          for (int k = j + 1; k < RP; ++k) v[i][k] = fmaf(-(s[k - K0] * inv), qv, v[i][k]);
        }
      }
    });
  } else {
#pragma unroll
    for (int j = 0; j < RP; ++j) {
      if (j < r) {
        float s[RP];
  #pragma unroll
        for (int k = 0; k < RP; ++k) s[k] = 0.0f;
  #pragma unroll
        for (int i = 0; i < RPT; ++i)
  #pragma unroll
          for (int k = 0; k < RP; ++k) s[k] = fmaf(v[i][j], v[i][k], s[k]);
        transpose_reduce<RP, RP, 32>(s, lane);
        const int b = j & 1;
        if ((lane & (kWave / RP - 1)) == 0) red[b][wave][lane >> (6 - LG)] = s[0];
        __syncthreads();
  #pragma unroll
        for (int k = 0; k < RP; ++k) {
          float t = 0.0f;
  #pragma unroll
          for (int wv = 0; wv < NW; ++wv) t += red[b][wv][k];
          s[k] = t;
        }
        const float nrm2 = s[j];
        const float inv = (nrm2 > FLT_MIN) ? 1.0f / sqrtf(nrm2) : 0.0f;
  #pragma unroll
        for (int i = 0; i < RPT; ++i) {
          const float qv = v[i][j] * inv;
          v[i][j] = qv;
  #pragma unroll
          for (int k = j + 1; k < RP; ++k) v[i][k] = fmaf(-(s[k] * inv), qv, v[i][k]);
        }
      }
    }
  }

  float mx = 0.0f;
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int row = tid + i * BS;
    if (row < rows) {
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k < r) {
          orth[(size_t)row * r + k] = v[i][k];
          mx = fmaxf(mx, fabsf(v[i][k]));
        }
    }
  }
  mx = wave_max(mx);
  if (lane == 0) redmax[wave] = mx;
  __syncthreads();
  if (tid == 0 && !a.orth_shared) {
    float m = redmax[0];
#pragma unroll
    for (int wv = 1; wv < NW; ++wv) m = fmaxf(m, redmax[wv]);
    a.scaleP[(size_t)worker * a.L + layer] = m;
  }
}

// ---------------------------------------------------------------------------
// orth, many workgroups per (layer, worker): for tall factors with few
// (layer, worker) pairs, where one workgroup each would leave the chip idle.
// The rows are cut into slices of 256; launch j (j = 0 .. r) applies the update
// of column j-1 to its slice (using the block-wide totals of launch j-1, added
// up over the slices in slice order) and then forms its slice's partial dot
// products of column j with the columns after it.  The grid-wide dependency
// between columns is the kernel boundary.  Launch 0 sums the sweep-0 partials,
// launch r finishes with absmax(P_w) through an integer atomic max.
// only_if (optional): one word per (layer, worker) pair, written by an earlier
// kernel; the launches skip the pairs whose word is zero.
// ---------------------------------------------------------------------------
template <int RP>
__global__ __launch_bounds__(256) void orth_wide_kernel(DevArgs a, int j, int nslice_max, const int* only_if) {
  __shared__ float red[4][RP];
  __shared__ float redmax[4];
  const int lw = blockIdx.x / nslice_max, slice = blockIdx.x - lw * nslice_max;
  if (only_if && only_if[lw] == 0) return;       // this pair was finished by the Cholesky-QR kernels
  const int layer = lw / a.W, worker = lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const int rows = ld.rows, r = ld.r;
  const int nslice = (rows + 255) >> 8;
  if (slice >= nslice || j > r) return;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int row = slice * 256 + tid;
  const bool live = row < rows;
  float* pre = a.Ppre + (size_t)worker * a.p_stride + ld.p_off;
  float* orth = a.Porth + (size_t)worker * a.p_stride + ld.p_off;
  float* part = a.orth_part;    // [2][L*W][nslice_max][RP]
  const size_t pstride = (size_t)a.L * a.W * nslice_max * RP;
  float v[RP];
#pragma unroll
  for (int k = 0; k < RP; ++k) v[k] = 0.0f;
  if (j == 0) {
    if (slice == 0 && tid == 0 && !a.orth_shared) a.scaleP[(size_t)worker * a.L + layer] = 0.0f;
    if (live) {
      if (only_if) {
        // The Cholesky-QR kernels have left the sum of the planes in `pre`, and where Gram-Schmidt
        // runs in place (the plane is the output) they have overwritten the plane itself.
#pragma unroll
        for (int k = 0; k < RP; ++k)
          if (k < r) v[k] = pre[(size_t)row * r + k];
      } else {
        const float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + (a.orth_shared ? ld.p_off : ld.ppart_off);
        const int nseg = a.orth_shared ? 1 : ld.nseg;
        for (int s = 0; s < nseg; ++s) {
          const float* src = Pp + (size_t)s * ld.np_pad + (size_t)row * r;
#pragma unroll
          for (int k = 0; k < RP; ++k)
            if (k < r) v[k] += src[k];
        }
      }
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k < r) {
          pre[(size_t)row * r + k] = v[k];
          orth[(size_t)row * r + k] = v[k];
        }
    }
  } else {
    const int c = j - 1;                         // the column this launch finishes
    const float* pin = part + (size_t)(c & 1) * pstride + (size_t)lw * nslice_max * RP;
    float tot[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) tot[k] = 0.0f;
    for (int s = 0; s < nslice; ++s) {
#pragma unroll
      for (int k = 0; k < RP; ++k) tot[k] += pin[(size_t)s * RP + k];
    }
    float nrm2 = 0.0f;
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k == c) nrm2 = tot[k];
    const float inv = (nrm2 > FLT_MIN) ? 1.0f / sqrtf(nrm2) : 0.0f;
    if (live) {
      float* dst = orth + (size_t)row * r;
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k < r) v[k] = dst[k];
      float qv = 0.0f;
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k == c) qv = v[k] * inv;
#pragma unroll
      for (int k = 0; k < RP; ++k) {
        if (k == c) v[k] = qv;
        else if (k > c && k < r) v[k] = fmaf(-(tot[k] * inv), qv, v[k]);
      }
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k >= c && k < r) dst[k] = v[k];
    }
  }
  if (j < r) {
    // partial <column j, column k> over this slice, every k (entries k < j are not used)
    float vj = 0.0f;
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k == j) vj = v[k];
    float s[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) s[k] = vj * v[k];
    transpose_reduce<RP, RP, 32>(s, lane);
    if ((lane & (kWave / RP - 1)) == 0) red[wave][lane >> (6 - log2c(RP))] = s[0];
    __syncthreads();
    if (tid < RP)
      part[(size_t)(j & 1) * pstride + ((size_t)lw * nslice_max + slice) * RP + tid] =
          (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
  } else {
    float mx = 0.0f;
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k < r) mx = fmaxf(mx, fabsf(v[k]));
    mx = wave_max(mx);
    if (lane == 0) redmax[wave] = mx;
    __syncthreads();
    if (tid == 0 && !a.orth_shared) {
      const float m = fmaxf(fmaxf(redmax[0], redmax[1]), fmaxf(redmax[2], redmax[3]));
      atomicMax(reinterpret_cast<unsigned int*>(a.scaleP + (size_t)worker * a.L + layer), __float_as_uint(m));
    }
  }
}

// ---------------------------------------------------------------------------
// orth, many workgroups per (layer, worker), one launch: the same slicing as
// orth_wide_kernel, but every workgroup keeps its 256 rows in registers through
// all columns, and the slices of a (layer, worker) pair exchange their partial
// dot products through a table in memory while the kernel runs.  The kernel is
// launched cooperatively, so all workgroups are resident and no slice waits
// for one that cannot start.
// A table entry is 64 bits: the partial <column j, column k> of one slice and a
// tag naming the launch and the column, written with ONE device-scope atomic
// store.  A reader polls an entry until it carries the tag it expects: value
// and "ready" arrive together, there is no counter and no fence (a device-
// scope fence writes back and invalidates a die's whole L2: ~100 us per column
// measured; the runtime's grid barrier ~65 us).  All entries of a pair are
// polled in parallel (one or a few per thread), collected in LDS and added up
// in slice order.  The table is double-buffered by column parity: a slice can
// only write column j + 2 after it has read every slice's column j + 1, which
// they write only after they have finished reading column j.
// Every wait is bounded; if one ever expires the workgroup raises the status
// word and carries on, so the kernel always ends.
// ---------------------------------------------------------------------------
constexpr unsigned kTablePolls = 1u << 20;      // default bound of a wait (about a second)
constexpr int kCoopMaxSlices = 64;               // rows <= 16384 per factor in this form

__device__ __forceinline__ unsigned long long table_load(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The columns of one slice, all r of them: v holds the slice's rows (one per thread) and leaves
// orthonormalised.  red [4 RP], tot_s [RP] and gather_s [kCoopMaxSlices RP] are LDS.
template <int RP>
__device__ __forceinline__ void coop_columns(float (&v)[RP], int r, int lw, int slice, int nslice, int nslice_max, int max_rank,
                                             unsigned long long* table, unsigned long long epoch, int* status,
                                             unsigned max_polls, size_t pstride, float* red, float* tot_s, float* gather_s) {
  constexpr int EPT = (kCoopMaxSlices * RP + 255) / 256;     // table entries a thread collects per column
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int nent = nslice * RP;
  for (int j = 0; j < r; ++j) {                  // r is the same for every slice of the pair
    const unsigned tag = (unsigned)(epoch * (unsigned long long)max_rank + (unsigned long long)(j + 1));
    unsigned long long* tab = table + (size_t)(j & 1) * pstride + (size_t)lw * nslice_max * RP;
    float vj = 0.0f;
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k == j) vj = v[k];
    float s[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) s[k] = vj * v[k];
    transpose_reduce<RP, RP, 32>(s, lane);
    if ((lane & (kWave / RP - 1)) == 0) red[wave * RP + (lane >> (6 - log2c(RP)))] = s[0];
    __syncthreads();
    if (tid < RP) {
      const float val = (red[tid] + red[RP + tid]) + (red[2 * RP + tid] + red[3 * RP + tid]);
      __hip_atomic_store(tab + (size_t)slice * RP + tid, ((unsigned long long)tag << 32) | __float_as_uint(val),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // collect every slice's entry for this column
    unsigned long long x[EPT];
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      const int e = tid + i * 256;
      x[i] = (e < nent) ? table_load(tab + e) : ((unsigned long long)tag << 32);
    }
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      const int e = tid + i * 256;
      unsigned polls = 0;
      while ((unsigned)(x[i] >> 32) != tag) {
        if (++polls >= max_polls) {
          __hip_atomic_store(status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
          break;
        }
        __builtin_amdgcn_s_sleep(1);
        x[i] = table_load(tab + e);
      }
      if (e < nent) gather_s[e] = __uint_as_float((unsigned)x[i]);
    }
    __syncthreads();
    if (tid < RP) {
      float t = 0.0f;
      for (int sl = 0; sl < nslice; ++sl) t += gather_s[sl * RP + tid];
      tot_s[tid] = t;
    }
    __syncthreads();
    const float nrm2 = tot_s[j];
    const float inv = (nrm2 > FLT_MIN) ? 1.0f / sqrtf(nrm2) : 0.0f;
    float qv = 0.0f;
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k == j) qv = v[k] * inv;
#pragma unroll
    for (int k = 0; k < RP; ++k) {
      if (k == j) v[k] = qv;
      else if (k > j && k < r) v[k] = fmaf(-(tot_s[k] * inv), qv, v[k]);
    }
    __syncthreads();                             // red, gather_s and tot_s are reused by the next column
  }
}

template <int RP>
__global__ __launch_bounds__(256) void orth_coop_kernel(DevArgs a, int nslice_max, int max_rank,
                                                        unsigned long long* table, unsigned long long epoch,
                                                        int* status, unsigned max_polls) {
  __shared__ float red[4 * RP];
  __shared__ float tot_s[RP];
  __shared__ float gather_s[kCoopMaxSlices * RP];
  __shared__ float redmax[4];
  const int lw = blockIdx.x / nslice_max, slice = blockIdx.x - lw * nslice_max;
  const int layer = lw / a.W, worker = lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const int rows = ld.rows, r = ld.r;
  const int nslice = (rows + 255) >> 8;
  if (slice >= nslice) return;                   // workgroup-uniform
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int row = slice * 256 + tid;
  const bool live = row < rows;
  float* pre = a.Ppre + (size_t)worker * a.p_stride + ld.p_off;
  float* orth = a.Porth + (size_t)worker * a.p_stride + ld.p_off;
  const size_t pstride = (size_t)a.L * a.W * nslice_max * RP;   // [2][L*W][nslice_max][RP] entries
  float v[RP];
#pragma unroll
  for (int k = 0; k < RP; ++k) v[k] = 0.0f;
  // The absmax cell is shared by all slices: zeroed here with a device-scope store, raised with
  // atomics at the end.  Every slice reads slice 0's first table entry before it gets there.
  if (slice == 0 && tid == 0 && !a.orth_shared) {
    __hip_atomic_store(a.scaleP + (size_t)worker * a.L + layer, 0.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): acknowledged before this slice publishes anything
  }
  if (live) {
    const float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + (a.orth_shared ? ld.p_off : ld.ppart_off);
    const int nseg = a.orth_shared ? 1 : ld.nseg;
    for (int s = 0; s < nseg; ++s) {
      const float* src = Pp + (size_t)s * ld.np_pad + (size_t)row * r;
#pragma unroll
      for (int k = 0; k < RP; ++k)
        if (k < r) v[k] += src[k];
    }
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k < r) pre[(size_t)row * r + k] = v[k];
  }
  coop_columns<RP>(v, r, lw, slice, nslice, nslice_max, max_rank, table, epoch, status, max_polls, pstride, red, tot_s,
                   gather_s);
  float mx = 0.0f;
  if (live) {
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k < r) {
        orth[(size_t)row * r + k] = v[k];
        mx = fmaxf(mx, fabsf(v[k]));
      }
  }
  mx = wave_max(mx);
  if (lane == 0) redmax[wave] = mx;
  __syncthreads();
  if (tid == 0 && !a.orth_shared) {
    const float m = fmaxf(fmaxf(redmax[0], redmax[1]), fmaxf(redmax[2], redmax[3]));
    atomicMax(reinterpret_cast<unsigned int*>(a.scaleP + (size_t)worker * a.L + layer), __float_as_uint(m));
  }
}

// ---------------------------------------------------------------------------
// exchange: LogQuantize (Eq. (5) discretised to 2^b levels, Section 4.1),
// pack, LogDequantize (Eq. (6)) and the mean over workers that stands in for
// the All-Reduce.
//   kQuantOnly: factors -> packets      kMeanOnly: packets -> mean
//   kFused:     factors -> packets and mean in one pass
// A workgroup takes kXBlockGroups groups of 8 consecutive factor elements; a
// lane handles one (group, worker) pair -- b magnitude bytes + 1 sign byte --
// eight workers at a time; the dequantised values meet in LDS, where lane
// (group, j) adds up element j over the workers in worker order.
// The code of u = |x|/s is the number of decision thresholds <= u, i.e.
// nearest-level rounding in the q-domain of Eq. (5): a hardware log2 gives the
// level to within one, the two loops move it to the exact count.
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void exchange_kernel(DevArgs a, const XTile* __restrict__ tiles, int phase) {
  __shared__ float s_thr[256];
  __shared__ float s_lev[256];
  __shared__ float s_val[8][kXGroup][kXBlockGroups];   // [worker slot][element][group]
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
  const int gl = tid & (kXBlockGroups - 1);
  const int slot = tid / kXBlockGroups;            // worker slot, and the element this lane sums
  const int g = tl.grp0 + gl;
  const int e0 = g * kXGroup;
  const bool gvalid = e0 < n_el;
  const int nvalid = gvalid ? min(kXGroup, n_el - e0) : 0;
  const size_t fstride = phase ? a.q_stride : a.p_stride;
  const float* fac = (phase ? a.Qw + ld.q_off : a.Porth + ld.p_off) + e0;
  uint8_t* mag = (phase ? a.magQ + ld.magq_off : a.magP + ld.magp_off) + (size_t)g * bits;
  uint8_t* sgn = (phase ? a.sgnQ + ld.sgnq_off : a.sgnP + ld.sgnp_off) + g;
  const size_t mstride = phase ? a.magq_stride : a.magp_stride;
  const size_t sstride = phase ? a.sgnq_stride : a.sgnp_stride;
  const float* scale = phase ? a.scaleQ : a.scaleP;
  const float qscale = phase ? a.qscale_q : a.qscale_p;

  float acc = 0.0f;
  for (int wbase = 0; wbase < a.W; wbase += 8) {
    const int w = wbase + slot;
    float val[kXGroup];
#pragma unroll
    for (int i = 0; i < kXGroup; ++i) val[i] = 0.0f;
    if (gvalid && w < a.W) {
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
#pragma unroll
        for (int i = 0; i < kXGroup; ++i) val[i] = x[i];
      } else {
        const float s = scale[(size_t)w * a.L + tl.layer];
        if (MODE != kMeanOnly) {
          quantise_group<true>(x, s, bits, lv, a.alpha, qscale, s_thr, s_lev, mag + (size_t)w * mstride,
                               sgn + (size_t)w * sstride, val);
        } else {
          unsigned long long magbits = 0;
          const uint8_t* mp = mag + (size_t)w * mstride;
          for (int bb = 0; bb < bits; ++bb) magbits |= (unsigned long long)mp[bb] << (8 * bb);
          const unsigned sgnbits = sgn[(size_t)w * sstride];
#pragma unroll
          for (int i = 0; i < kXGroup; ++i) {
            const int k = (int)((magbits >> (i * bits)) & (unsigned long long)lv);
            const float v = s * s_lev[k];
            val[i] = ((sgnbits >> i) & 1u) ? -v : v;
          }
        }
      }
    }
    if (MODE != kQuantOnly) {
#pragma unroll
      for (int i = 0; i < kXGroup; ++i) s_val[slot][i][gl] = val[i];
      __syncthreads();
      const int nw = min(8, a.W - wbase);
      for (int sidx = 0; sidx < nw; ++sidx) acc += s_val[sidx][slot][gl];
      __syncthreads();
    }
  }
  if (MODE != kQuantOnly) {
    if (gvalid && slot < nvalid) {
      float* out = (phase ? a.Qbar + ld.q_off : a.Pbar + ld.p_off) + e0;
      out[slot] = acc / (float)a.W;
    }
  }
}

// ---------------------------------------------------------------------------
// sweep 1: Q_w partial = M_w^T P-bar over a row block (Algorithm 1,
// "Q <- G'^T P").  One workgroup per (row block, 64*VEC-column chunk); its four
// wavefronts split the rows and their partial sums meet in LDS, where they are
// added in wavefront order.
// ---------------------------------------------------------------------------
template <int RP, int VEC, bool EXACT>
__device__ __forceinline__ void back_project_rows(const float* __restrict__ M, const float* Pb, int cols, int r,
                                                  int ra, int rb, unsigned boff, float (&acc)[VEC * RP]) {
  constexpr int U = LQSGD_B_U;
  int i = ra;
  for (; i + U <= rb; i += U) {
    Pk<VEC> m[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      m[u] = ldrow<VEC, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(M + (size_t)(i + u) * cols), boff);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float p[RP];
      load_row_uniform<RP, EXACT>(Pb, i + u, r, p);
#pragma unroll
      for (int v = 0; v < VEC; ++v)
#pragma unroll
        for (int k = 0; k < RP; ++k) acc[v * RP + k] = fmaf(m[u].v[v], p[k], acc[v * RP + k]);
    }
  }
  for (; i < rb; ++i) {
    const Pk<VEC> m = ldrow<VEC, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(M + (size_t)i * cols), boff);
    float p[RP];
    load_row_uniform<RP, EXACT>(Pb, i, r, p);
#pragma unroll
    for (int v = 0; v < VEC; ++v)
#pragma unroll
      for (int k = 0; k < RP; ++k) acc[v * RP + k] = fmaf(m.v[v], p[k], acc[v * RP + k]);
  }
}

template <int RP, int VEC, bool EXACT>
__device__ __forceinline__ void back_project_tile(const DevArgs& a, const LayerDesc& ld, const Tile& tl, int layer, int worker,
                                                  float* comb, float* redmax, int wave, int lane) {
  constexpr int NV = VEC * RP;
  const int cols = ld.cols, r = ld.r;
  const float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  const float* Pb = a.Pbar + ld.p_off;
  const int c0 = tl.aux * (kWave * VEC);
  const int c = c0 + lane * VEC;
  const bool active = c < cols;
  const int per = (tl.nrows + 3) >> 2;
  const int ra = min(tl.row0 + wave * per, tl.row0 + tl.nrows);
  const int rb = min(ra + per, tl.row0 + tl.nrows);
  float acc[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) acc[i] = 0.0f;
  if (active) {
    if (tl.nrows >= LQSGD_B_INTERLEAVE) {
      // Tall row blocks: the four wavefronts take groups of 8 rows in turn instead of a quarter of
      // the block each, so that they read rows close to each other at any time (four streams
      // hundreds of rows apart read the 8192^2 set at 6.0 TB/s, interleaved at 6.6 TB/s).
      const int rend = tl.row0 + tl.nrows;
      for (int g0 = tl.row0 + wave * LQSGD_B_U; g0 < rend; g0 += 4 * LQSGD_B_U)
        back_project_rows<RP, VEC, EXACT>(M, Pb, cols, r, g0, min(g0 + LQSGD_B_U, rend), (unsigned)c * 4u, acc);
    } else {
      back_project_rows<RP, VEC, EXACT>(M, Pb, cols, r, ra, rb, (unsigned)c * 4u, acc);
    }
  }
  // A layer whose rows fit one row block: this item holds the whole sum, Q_w is stored directly
  // and its absmax raised here (the cell was zeroed by sweep 0); otherwise a partial plane per
  // row block, added up by reduce_q_kernel.
  const bool direct = ld.direct_q != 0;
  float* Qp = direct ? a.Qw + (size_t)worker * a.q_stride + ld.q_off
                     : a.Qpart + (size_t)worker * a.qpart_stride + ld.qpart_off + (size_t)(tl.row0 / ld.rbb) * ld.nq_pad;
  float mx = 0.0f;
  if constexpr (EXACT && NV % 4 == 0 && NV <= 64) {
    // comb[wave][lane * NV + i]; afterwards every lane of the workgroup adds the four
    // partials of NV/4 consecutive outputs (wave order) and stores them: the chunk's
    // slice of the factor is contiguous, 64 * NV floats from column c0.
#pragma unroll
    for (int i = 0; i < NV / 4; ++i)
      reinterpret_cast<float4*>(comb + (size_t)wave * (kWave * NV) + lane * NV)[i] =
          make_float4(acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]);
    __syncthreads();
    const int tid = wave * kWave + lane;
    const int nout = min(kWave * VEC, cols - c0) * RP;     // floats this chunk owns
#pragma unroll
    for (int j = 0; j < (NV + 15) / 16; ++j) {   // 64 * NV / 4 float4 outputs over 256 lanes
      const int o = (j * 256 + tid) * 4;
      if (o < nout) {
        float4 s = reinterpret_cast<const float4*>(comb + o)[0];
#pragma unroll
        for (int wv = 1; wv < 4; ++wv) {
          const float4 t = reinterpret_cast<const float4*>(comb + (size_t)wv * (kWave * NV) + o)[0];
          s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        reinterpret_cast<float4*>(Qp + (size_t)c0 * RP + o)[0] = s;
        mx = fmaxf(fmaxf(mx, fmaxf(fabsf(s.x), fabsf(s.y))), fmaxf(fabsf(s.z), fabsf(s.w)));
      }
    }
  } else {
    // generic path: (wave 0 + wave 2) + (wave 1 + wave 3) through two LDS planes
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
      store_slice<RP, VEC, EXACT>(Qp, c, r, acc);
#pragma unroll
      for (int v = 0; v < VEC; ++v)
#pragma unroll
        for (int k = 0; k < RP; ++k)
          if (c + v < cols && k < r) mx = fmaxf(mx, fabsf(acc[v * RP + k]));
    }
  }
  if (direct) {     // workgroup-uniform
    mx = wave_max(mx);
    if (lane == 0) redmax[wave] = mx;
    __syncthreads();
    if (wave == 0 && lane == 0) {
      const float m = fmaxf(fmaxf(redmax[0], redmax[1]), fmaxf(redmax[2], redmax[3]));
      atomicMax(reinterpret_cast<unsigned int*>(a.scaleQ + (size_t)worker * a.L + layer), __float_as_uint(m));
    }
  }
}

// ---------------------------------------------------------------------------
// 1-D tensors: plain mean over the workers (Eq. (1)).  Runs as extra
// workgroups at the end of sweep 1's grid.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void vector_mean_tile(const DevArgs& a, const VTile& tl) {
  const VecDesc& vd = a.vecs[tl.vec];
  auto* extra = gptr<float>(a.ghat ? a.ghat[vd.gidx] : nullptr);
  const float wf = (float)a.W;
  for (int i = 0; i < 4; ++i) {
    const int e = tl.el0 + i * 256 + threadIdx.x;
    if (e < vd.len) {
      float s = 0.0f;
      if (a.g_bf16) {
        for (int w = 0; w < a.W; ++w) s += grad_elem<true>(a.grads[(size_t)w * a.n_all + vd.gidx], (size_t)e);
      } else {
        for (int w = 0; w < a.W; ++w) s += grad_elem<false>(a.grads[(size_t)w * a.n_all + vd.gidx], (size_t)e);
      }
      s /= wf;
      a.vmean[vd.off + e] = s;
      if (extra) extra[e] = a.update ? fmaf(-a.eta, s, extra[e]) : s;
    }
  }
}

template <int RP>
__global__ __launch_bounds__(256) void back_project_kernel(DevArgs a, const Tile* __restrict__ tiles, int ntiles,
                                                           const VTile* __restrict__ vtiles, int reverse) {
  // fast path: 4 planes of 64 * 4 * RP floats (RP <= 16); generic path: 2 planes
  __shared__ float comb[(RP <= 16 ? 4 : 2) * kWave * 4 * RP];
  __shared__ float redmax[4];
  if ((int)blockIdx.x >= ntiles) {
    vector_mean_tile(a, vtiles[blockIdx.x - ntiles]);
    return;
  }
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  const Tile tl = tiles[reverse ? ntiles - 1 - blockIdx.x : blockIdx.x];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  if (ld.vec == 4) {
    if (ld.r == RP)
      back_project_tile<RP, 4, true>(a, ld, tl, layer, worker, comb, redmax, wave, lane);
    else
      back_project_tile<RP, 4, false>(a, ld, tl, layer, worker, comb, redmax, wave, lane);
  } else {
    back_project_tile<RP, 1, false>(a, ld, tl, layer, worker, comb, redmax, wave, lane);
  }
}

// ---------------------------------------------------------------------------
// sweep 1 on the matrix cores, for rank pad 32, where 4 x r accumulators per
// lane no longer fit the vector register file.
// v_mfma_f32_32x32x2_f32 computes D[32 x 32] += A[32 x 2] B[2 x 32] with
//   A: lane l holds A[i = l % 32][k = l / 32]
//   B: lane l holds B[k = l / 32][j = l % 32]
//   D: lane l, register v holds D[i = 8 (v / 4) + 4 (l / 32) + v % 4][j = l % 32]
// Here j = rank, k = two gradient rows per instruction, i = gradient column.
// Which column an index i stands for is free, as long as the result is read
// back the same way: lane (i, k) loads the float4 of columns 4 i .. 4 i + 3 of
// its row (so a half-wavefront reads 512 contiguous bytes of a row, a
// wavefront two rows, a workgroup 2 KiB of each row), and component s of that
// float4 feeds matrix instruction s, whose block D_s then belongs to columns
// 4 i + s.  No transposition and no LDS; a 32 x 32 block of Q_w accumulates in
// 16 registers.
// ---------------------------------------------------------------------------
typedef float v16f __attribute__((ext_vector_type(16)));

template <bool VEC4>
__device__ __forceinline__ void back_project_mfma_tile(const DevArgs& a, const LayerDesc& ld, const Tile& tl, int worker,
                                                       int wave, int lane) {
  const int cols = ld.cols, r = ld.r;
  const int c0 = tl.aux * kMfmaCols + wave * 128;
  if (c0 >= cols) return;
  const int li = lane & 31, h = lane >> 5;
  const float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  const float* Pb = a.Pbar + ld.p_off;
  const bool rankok = li < r;
  const int rend = tl.row0 + tl.nrows;
  const int cl = c0 + 4 * li;                      // first of this lane's four columns
  v16f acc[4];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[s][i] = 0.0f;
  constexpr int UI = LQSGD_BM_U;   // pairs of rows per step on interior strips
  constexpr int U = 4;             // ... and on the bounds-tested path
  int rb = tl.row0;
  if constexpr (VEC4) {
    // Interior strips (all 128 columns exist): whole groups of 2 UI rows with no bounds
    // tests, and the next group's loads are issued before this group's matrix instructions, so that a
    // wavefront overlaps its own loads with its own arithmetic (the last prefetch re-reads the last
    // group: every load stays unconditional and in bounds).
    if (c0 + 128 <= cols && rend - rb >= 2 * UI) {
      const int last = rb + ((rend - rb) / (2 * UI) - 1) * (2 * UI);   // first row of the last whole group
      Pk<4> am[UI], an[UI];
      float bp[UI], bn[UI];
      const int lic = min(li, r - 1);      // ranks beyond r: read a valid element, masked below
#pragma unroll
      for (int u = 0; u < UI; ++u) {
        const int row = rb + 2 * u + h;
        am[u] = ldrow<4, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(M + (size_t)row * cols), (unsigned)cl * 4u);
        bp[u] = Pb[(size_t)row * r + lic];
      }
      for (; rb <= last; rb += 2 * UI) {
        const int nb = min(rb + 2 * UI, last);
#pragma unroll
        for (int u = 0; u < UI; ++u) {
          const int row = nb + 2 * u + h;
          an[u] = ldrow<4, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(M + (size_t)row * cols), (unsigned)cl * 4u);
          bn[u] = Pb[(size_t)row * r + lic];
        }
        // the requests above stay ahead of the arithmetic below (left to itself the compiler moves the
        // P-bar loads down to their first use, and every group of matrix instructions then waits for
        // its operand and, requests completing in order, for the whole prefetch in front of it)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < UI; ++u)
#pragma unroll
          for (int s = 0; s < 4; ++s)
            acc[s] = __builtin_amdgcn_mfma_f32_32x32x2f32(am[u].v[s], keep_if(bp[u], rankok), acc[s], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < UI; ++u) { am[u] = an[u]; bp[u] = bn[u]; }
      }
    }
  }
  for (; rb < rend; rb += 2 * U) {
    Pk<4> am[U];
    float bp[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = rb + 2 * u + h;
      const bool ok = row < rend;
      const float* mrow = M + (size_t)row * cols;
      if constexpr (VEC4) {
        if (ok && cl < cols) {
          am[u] = ldrow<4, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(mrow), (unsigned)cl * 4u);
        } else {
#pragma unroll
          for (int s = 0; s < 4; ++s) am[u].v[s] = 0.0f;
        }
      } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) am[u].v[s] = (ok && cl + s < cols) ? mrow[cl + s] : 0.0f;
      }
      bp[u] = (ok && rankok) ? Pb[(size_t)row * r + li] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int s = 0; s < 4; ++s) acc[s] = __builtin_amdgcn_mfma_f32_32x32x2f32(am[u].v[s], bp[u], acc[s], 0, 0, 0);
  }
  float* Qp = a.Qpart + (size_t)worker * a.qpart_stride + ld.qpart_off + (size_t)(tl.row0 / ld.rbb) * ld.nq_pad;
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int col = c0 + 4 * (8 * (v >> 2) + 4 * h + (v & 3)) + s;
      if (col < cols && rankok) Qp[(size_t)col * r + li] = acc[s][v];
    }
}

// The same with NB blocks of 32 ranks (rank pad 64: NB = 2): one pass over M feeds both blocks.
template <bool VEC4, int NB>
__device__ __forceinline__ void back_project_mfma_tile_nb(const DevArgs& a, const LayerDesc& ld, const Tile& tl, int worker,
                                                       int wave, int lane) {
  const int cols = ld.cols, r = ld.r;
  const int c0 = tl.aux * kMfmaCols + wave * 128;
  if (c0 >= cols) return;
  const int li = lane & 31, h = lane >> 5;
  const float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  const float* Pb = a.Pbar + ld.p_off;
  bool rankok[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) rankok[nb] = 32 * nb + li < r;
  const int rend = tl.row0 + tl.nrows;
  const int cl = c0 + 4 * li;                      // first of this lane's four columns
  v16f acc[NB][4];                                  // [block of 32 ranks][column residue]
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[nb][s][i] = 0.0f;
  constexpr int UI = LQSGD_BM_U2;  // pairs of rows per step on interior strips
  constexpr int U = 4;             // ... and on the bounds-tested path
  int rb = tl.row0;
  if constexpr (VEC4) {
    // interior strips: as in the one-block form, whole groups of rows without bounds tests and the
    // next group's loads ahead of this group's matrix instructions; ranks beyond r are read from a
    // clamped index and masked
    if (c0 + 128 <= cols && rend - rb >= 2 * UI) {
      const int last = rb + ((rend - rb) / (2 * UI) - 1) * (2 * UI);
      Pk<4> am[UI], an[UI];
      float bp[NB][UI], bn[NB][UI];
      int rkc[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) rkc[nb] = min(32 * nb + li, r - 1);
#pragma unroll
      for (int u = 0; u < UI; ++u) {
        const int row = rb + 2 * u + h;
        am[u] = ldrow<4, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(M + (size_t)row * cols), (unsigned)cl * 4u);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bp[nb][u] = Pb[(size_t)row * r + rkc[nb]];
      }
      for (; rb <= last; rb += 2 * UI) {
        const int nxt = min(rb + 2 * UI, last);
#pragma unroll
        for (int u = 0; u < UI; ++u) {
          const int row = nxt + 2 * u + h;
          an[u] = ldrow<4, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(M + (size_t)row * cols), (unsigned)cl * 4u);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) bn[nb][u] = Pb[(size_t)row * r + rkc[nb]];
        }
        __builtin_amdgcn_sched_barrier(0);   // as in the one-block form: the requests stay ahead of the arithmetic
#pragma unroll
        for (int u = 0; u < UI; ++u)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const float bv = keep_if(bp[nb][u], rankok[nb]);
#pragma unroll
            for (int s = 0; s < 4; ++s)
              acc[nb][s] = __builtin_amdgcn_mfma_f32_32x32x2f32(am[u].v[s], bv, acc[nb][s], 0, 0, 0);
          }
#pragma unroll
        for (int u = 0; u < UI; ++u) {
          am[u] = an[u];
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) bp[nb][u] = bn[nb][u];
        }
      }
    }
  }
  for (; rb < rend; rb += 2 * U) {
    Pk<4> am[U];
    float bp[NB][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = rb + 2 * u + h;
      const bool ok = row < rend;
      const float* mrow = M + (size_t)row * cols;
      if constexpr (VEC4) {
        if (ok && cl < cols) {
          am[u] = ldrow<4, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(mrow), (unsigned)cl * 4u);
        } else {
#pragma unroll
          for (int s = 0; s < 4; ++s) am[u].v[s] = 0.0f;
        }
      } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) am[u].v[s] = (ok && cl + s < cols) ? mrow[cl + s] : 0.0f;
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) bp[nb][u] = (ok && rankok[nb]) ? Pb[(size_t)row * r + 32 * nb + li] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int s = 0; s < 4; ++s)
          acc[nb][s] = __builtin_amdgcn_mfma_f32_32x32x2f32(am[u].v[s], bp[nb][u], acc[nb][s], 0, 0, 0);
  }
  float* Qp = a.Qpart + (size_t)worker * a.qpart_stride + ld.qpart_off + (size_t)(tl.row0 / ld.rbb) * ld.nq_pad;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int col = c0 + 4 * (8 * (v >> 2) + 4 * h + (v & 3)) + s;
        if (col < cols && rankok[nb]) Qp[(size_t)col * r + 32 * nb + li] = acc[nb][s][v];
      }
}

template <int NB>
__global__ __launch_bounds__(256, 2) void back_project_mfma_kernel(DevArgs a, const Tile* __restrict__ tiles, int ntiles,
                                                                const VTile* __restrict__ vtiles, int reverse) {
  if ((int)blockIdx.x >= ntiles) {
    vector_mean_tile(a, vtiles[blockIdx.x - ntiles]);
    return;
  }
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  const Tile tl = tiles[reverse ? ntiles - 1 - blockIdx.x : blockIdx.x];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  if constexpr (NB == 1) {
    if (ld.vec == 4)
      back_project_mfma_tile<true>(a, ld, tl, worker, wave, lane);
    else
      back_project_mfma_tile<false>(a, ld, tl, worker, wave, lane);
  } else {
    if (ld.vec == 4)
      back_project_mfma_tile_nb<true, NB>(a, ld, tl, worker, wave, lane);
    else
      back_project_mfma_tile_nb<false, NB>(a, ld, tl, worker, wave, lane);
  }
}

// ---------------------------------------------------------------------------
// reduce_q: Q_w = sum over row blocks of the partials (fixed order), and
// absmax(Q_w) -> scaleQ.  The max over workgroups goes through an integer
// atomic max on the float's bit pattern (non-negative floats order like
// unsigned integers), which is exact and order-independent.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void reduce_q_kernel(DevArgs a, const RTile* __restrict__ tiles, int phase) {
  __shared__ float redmax[4];
  const RTile tl = tiles[blockIdx.x];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  float mx = 0.0f;
  // phase 1: Q_w from the row-block planes; phase 0 (aggregate-first order only): the raw P_w from
  // the column-segment planes, which is then what the P exchange quantises
  const int n_el = phase ? ld.nq_el : ld.np_el;
  const float* planes = phase ? a.Qpart + (size_t)worker * a.qpart_stride + ld.qpart_off
                              : a.Ppart + (size_t)worker * a.ppart_stride + ld.ppart_off;
  float* out = phase ? a.Qw + (size_t)worker * a.q_stride + ld.q_off : a.Ppre + (size_t)worker * a.p_stride + ld.p_off;
  const int nplanes = phase ? ld.nrb : ld.nseg;
  const size_t pitch = phase ? ld.nq_pad : ld.np_pad;
  for (int off = tid * 4; off < tl.n; off += 1024) {
    const int e = tl.el0 + off;                    // < n_el, and so are the elements of its float4 that are kept
    const float* Qp = planes + e;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    // planes are added in order; eight loads are in flight at a time
    int rb = 0;
    for (; rb + 8 <= nplanes; rb += 8) {
      float4 t[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) t[i] = *reinterpret_cast<const float4*>(Qp + (size_t)(rb + i) * pitch);
#pragma unroll
      for (int i = 0; i < 8; ++i) { s.x += t[i].x; s.y += t[i].y; s.z += t[i].z; s.w += t[i].w; }
    }
    for (; rb < nplanes; ++rb) {
      const float4 t = *reinterpret_cast<const float4*>(Qp + (size_t)rb * pitch);
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    float* dst = out + e;
    const int nv = min(4, n_el - e);
    if (nv == 4) {
      *reinterpret_cast<float4*>(dst) = s;
      mx = fmaxf(mx, fmaxf(fmaxf(fabsf(s.x), fabsf(s.y)), fmaxf(fabsf(s.z), fabsf(s.w))));
    } else {
      const float vals[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < nv) {
          dst[i] = vals[i];
          mx = fmaxf(mx, fabsf(vals[i]));
        }
    }
  }
  mx = wave_max(mx);
  if (lane == 0) redmax[wave] = mx;
  __syncthreads();
  if (tid == 0) {
    const float m = fmaxf(fmaxf(redmax[0], redmax[1]), fmaxf(redmax[2], redmax[3]));
    atomicMax(reinterpret_cast<unsigned int*>((phase ? a.scaleQ : a.scaleP) + (size_t)worker * a.L + layer),
              __float_as_uint(m));
  }
}

// ---------------------------------------------------------------------------
// sweep 2: E_w = M_w - P-bar Q-bar^T (Eq. (7), (8)) and / or G-hat = P-bar Q-bar^T.
//   kResidual      E for every worker                          (8 B / element)
//   kResidualGhat  E for every worker, G-hat from worker 0's items
//   kGhatOnly      G-hat only, one item list per layer (4 B / element / W);
//                  used when the residual update is deferred into the next
//                  iteration's sweep 0
// The four wavefronts of a workgroup split the rows of the item.
// ---------------------------------------------------------------------------
enum ResidualMode { kResidual = 0, kResidualGhat = 1, kGhatOnly = 2 };

template <int RP, int VEC, bool EXACT, int MODE>
__device__ __forceinline__ void residual_rows(float* __restrict__ M, const float* Pb, float* __restrict__ ghat,
                                              int cols, int r, int ra, int rb, unsigned boff,
                                              const float (&q)[VEC * RP], int update, float eta) {
  constexpr int U = 8;
  for (int i = ra; i < rb; i += U) {
    const int nu = min(U, rb - i);
    Pk<VEC> m[U];
    if constexpr (MODE != kGhatOnly) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (u < nu) {
          m[u] = ldrow<VEC, LQSGD_NT_M != 0>(reinterpret_cast<const char*>(M + (size_t)(i + u) * cols), boff);
        } else {
#pragma unroll
          for (int v = 0; v < VEC; ++v) m[u].v[v] = 0.0f;
        }
      }
    } else if (update) {
      // the parameters this pass updates, fetched for all U rows before the arithmetic starts
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (u < nu) {
          m[u] = ldrow<VEC, true>(reinterpret_cast<const char*>(ghat + (size_t)(i + u) * cols), boff);
        } else {
#pragma unroll
          for (int v = 0; v < VEC; ++v) m[u].v[v] = 0.0f;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (u < nu) {
        float p[RP];
        load_row_uniform<RP, EXACT>(Pb, i + u, r, p);
        Pk<VEC> gh, e;
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          float s = 0.0f;
#pragma unroll
          for (int k = 0; k < RP; ++k) s = fmaf(p[k], q[v * RP + k], s);
          gh.v[v] = s;
          if constexpr (MODE != kGhatOnly) e.v[v] = m[u].v[v] - s;
        }
        if constexpr (MODE != kGhatOnly)
          strow<VEC, false>(reinterpret_cast<char*>(M + (size_t)(i + u) * cols), boff, e);
        if constexpr (MODE == kGhatOnly) {
          if (update) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) gh.v[v] = fmaf(-eta, gh.v[v], m[u].v[v]);
          }
          strow<VEC, true>(reinterpret_cast<char*>(ghat + (size_t)(i + u) * cols), boff, gh);
        } else if (MODE == kResidualGhat && ghat) {
          emit_ghat<VEC>(ghat + (size_t)(i + u) * cols, boff, gh, update, eta);
        }
      }
    }
  }
}

template <int RP, int VEC, bool EXACT, int MODE>
__device__ __forceinline__ void residual_tile(const DevArgs& a, const LayerDesc& ld, const Tile& tl, int worker,
                                              float* __restrict__ ghat, int wave, int lane) {
  constexpr int NV = VEC * RP;
  const int cols = ld.cols, r = ld.r;
  float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  const float* Pb = a.Pbar + ld.p_off;
  const int c = tl.aux * (kWave * VEC) + lane * VEC;
  if (c >= cols) return;
  const int per = (tl.nrows + 3) >> 2;
  const int ra = min(tl.row0 + wave * per, tl.row0 + tl.nrows);
  const int rb = min(ra + per, tl.row0 + tl.nrows);
  float q[NV];
  load_slice<RP, VEC, EXACT>(a.Qbar + ld.q_off, c, r, q);
  residual_rows<RP, VEC, EXACT, MODE>(M, Pb, ghat, cols, r, ra, rb, (unsigned)c * 4u, q, a.update, a.eta);
}

template <int RP, int MODE>
__global__ __launch_bounds__(256) void residual_kernel(DevArgs a, const Tile* __restrict__ tiles, int ntiles, int reverse) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  const Tile tl = tiles[reverse ? ntiles - 1 - blockIdx.x : blockIdx.x];
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  float* ghat = nullptr;
  if (MODE != kResidual && worker == 0 && a.ghat) ghat = a.ghat[ld.gidx];
  if (MODE == kGhatOnly && !ghat) return;
  if (ld.vec == 4) {
    if (ld.r == RP)
      residual_tile<RP, 4, true, MODE>(a, ld, tl, worker, ghat, wave, lane);
    else
      residual_tile<RP, 4, false, MODE>(a, ld, tl, worker, ghat, wave, lane);
  } else {
    residual_tile<RP, 1, false, MODE>(a, ld, tl, worker, ghat, wave, lane);
  }
}

// ---------------------------------------------------------------------------
// Sweeps 0 and 2 on the matrix cores, rank pads 16 and 32.
// One workgroup per work item (32 rows x one column segment); its four
// wavefronts take the 64-column blocks of the segment in turn, so that the
// workgroup touches 1 KiB of every row at about the same time (with one item
// per wavefront, each walking its own segment in 256-byte runs, the same data
// movement reached only 4.3 TB/s; this order reaches 5.4-5.8), and their P
// partials meet in LDS, added in wavefront order.  A 32 x 64 tile is loaded and
// stored in "row layout" (float4 per lane, 16 lanes = 256 contiguous bytes of a
// row, 4 rows per instruction).
//
//   G-hat tile = P-bar[32 x r] Q-bar^T[r x 64]: i = row, j = column, k = rank.
//     Lane (i, h) holds P-bar[row i][h r/2 .. h r/2 + r/2) -- a contiguous run of
//     its factor row, so the wavefront reads one contiguous block of P-bar;
//     lane (h, j) holds Q-bar[col j][the same ranks].  Which rank a step k
//     stands for is free as long as both operands agree.
//   P tile += M[32 x 64] Q[64 x r]: i = row, j = rank, k = column.  Lanes index
//     rows here while memory runs along columns, so M goes through a
//     wave-private LDS tile ([row][column], pitch 68 floats): written in row
//     layout, read back as lane (i, h) -> columns 32 h .. 32 h + 31 of row i.
//   The G-hat block comes out of the matrix cores in their D layout (lanes =
//   columns); it takes the same LDS tile the other way to meet G and M in row
//   layout for  M_new = G + (M_old - G-hat).
// Modes: kMAdd (first iteration: M = G + E), kMAddFused (deferred residual),
// kMResidual / kMResidualGhat / kMGhatOnly (the residual sweep; G-hat uses the
// very same instruction sequence as in kMAddFused, so deferring the residual
// does not change a bit of the result).
// ---------------------------------------------------------------------------
enum MfmaMode { kMAdd = 0, kMAddFused = 1, kMResidual = 2, kMResidualGhat = 3, kMGhatOnly = 4 };
constexpr int kLP = 68;   // LDS pitch (floats): 16-byte aligned rows, 4-bank skew per row

__device__ __forceinline__ void wave_lds_fence() {
  // LDS traffic between the lanes of one wavefront: the hardware keeps DS
  // operations of a wavefront in order; this only stops the compiler.
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

template <int RP, int MODE, bool EXACT, bool GB16, bool NTS>
__device__ __forceinline__ void mfma_tile(const float* __restrict__ G, float* __restrict__ M,
                                          const float* Q, const float* Pb, float* __restrict__ Pp,
                                          float* __restrict__ ghat_out, int cols, int r, int row0, int nrows,
                                          int col0, int col1, int lane, int wave, float (*lds_all)[32 * kLP],
                                          int update, float eta) {
  float* lds = lds_all[wave];
  constexpr bool ADD = (MODE == kMAdd || MODE == kMAddFused);
  constexpr bool NEEDG = (MODE != kMAdd);
  constexpr bool HASM = (MODE != kMGhatOnly);
  constexpr int KH = RP / 2;                       // ranks per half-wavefront
  constexpr int NB = (RP + 31) / 32;               // blocks of 32 ranks in the P product (2 at rank pad 64)
  // EXACT: the rows of Q and Pb hold RP ranks (the layer's rank is RP, or the operands are the copies
  // padded with zeros); r is then only the row length of the P partials this item writes.
  const int rs = EXACT ? RP : r;
  const int li = lane & 31, h = lane >> 5;
  const int sr = lane >> 4, c4 = (lane & 15) * 4;  // row layout: rows 4 i + sr, columns c4 .. c4 + 3
  float pa[KH];
  if constexpr (NEEDG) {
    const int row = row0 + li;
    if constexpr (EXACT) {
      if (li < nrows) {
        const float4* src = reinterpret_cast<const float4*>(Pb + (size_t)row * RP + KH * h);
#pragma unroll
        for (int t = 0; t < KH / 4; ++t) {
          const float4 x = src[t];
          pa[4 * t] = x.x; pa[4 * t + 1] = x.y; pa[4 * t + 2] = x.z; pa[4 * t + 3] = x.w;
        }
      } else {
#pragma unroll
        for (int k = 0; k < KH; ++k) pa[k] = 0.0f;
      }
    } else {
#pragma unroll
      for (int k = 0; k < KH; ++k) pa[k] = (li < nrows && KH * h + k < r) ? Pb[(size_t)row * r + KH * h + k] : 0.0f;
    }
  }
  v16f accP[NB], accP2[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int i = 0; i < 16; ++i) { accP[nb][i] = 0.0f; accP2[nb][i] = 0.0f; }

  // the four wavefronts take the 64-column blocks of the segment in turn, so that together they
  // touch 1 KiB of each row at about the same time (a wavefront on its own reads 256-byte runs)
  // One 64-column block.  FULL: all 32 rows and all 64 columns of the block exist (every block of a
  // large layer except on its edges): no bounds tests, so nothing branches around a load.
  auto block = [&](auto full_tag, const int c) {
    constexpr bool FULL = decltype(full_tag)::value;
    const int cl = c + c4;
    const bool colok = FULL || cl < col1;
    Pk<4> g[8], e[8];
    // FULL blocks address memory as a wave-uniform base (scalar registers) plus one byte offset per
    // lane that is the same for every row group and block: lo = this lane's place in 4 rows.
    const unsigned lo = (unsigned)(sr * cols + c4) * 4u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rr = 4 * i + sr;
      const bool ok = FULL || (colok && rr < nrows);
      const size_t off = FULL ? (size_t)(row0 + 4 * i) * cols + c : (size_t)(row0 + rr) * cols;
      const unsigned bo = FULL ? lo : (unsigned)cl * 4u;
#pragma unroll
      for (int v = 0; v < 4; ++v) { g[i].v[v] = 0.0f; e[i].v[v] = 0.0f; }
      if (ok) {
        if constexpr (ADD) g[i] = ldgrad<4, LQSGD_NT_G != 0, GB16>(grad_row<GB16>(G, off), bo);
        if constexpr (HASM) e[i] = ldrow<4, (ADD ? NTS : LQSGD_NT_E != 0)>(reinterpret_cast<const char*>(M + off), bo);
      }
    }
    float bq[NB][32];
    auto load_bq = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int kk = 0; kk < 32; ++kk) {
          const int col = c + 32 * h + kk;
          const int rk = 32 * nb + li;
          if constexpr (FULL && EXACT)
            bq[nb][kk] = ldrow<1, false>(reinterpret_cast<const char*>(Q + (size_t)c * RP) + (kk * RP + 32 * nb) * 4,
                                         (unsigned)(32 * h * RP + li) * 4u).v[0];
          else
            bq[nb][kk] = (col < col1 && rk < rs) ? Q[(size_t)col * rs + rk] : 0.0f;
        }
    };
    // In the fused mode the Q slice of the P product is fetched only after the G-hat part, when
    // the registers of its operands are free again (fetched up front it does not fit the register file).
    constexpr bool BQ_LATE = ADD && NEEDG && LQSGD_BQ_LATE;
    if constexpr (ADD && !BQ_LATE) load_bq();
    if constexpr (NEEDG) {
      float qb[2][KH];
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int col = c + 32 * b + li;
        if constexpr (EXACT) {
          if constexpr (FULL) {
            const char* base = reinterpret_cast<const char*>(Q + (size_t)(c + 32 * b) * RP);
#pragma unroll
            for (int t = 0; t < KH / 4; ++t) {
              const Pk<4> x = ldrow<4, false>(base + 16 * t, (unsigned)(li * RP + KH * h) * 4u);
              qb[b][4 * t] = x.v[0]; qb[b][4 * t + 1] = x.v[1]; qb[b][4 * t + 2] = x.v[2]; qb[b][4 * t + 3] = x.v[3];
            }
          } else if (col < col1) {
            const float4* src = reinterpret_cast<const float4*>(Q + (size_t)col * RP + KH * h);
#pragma unroll
            for (int t = 0; t < KH / 4; ++t) {
              const float4 x = src[t];
              qb[b][4 * t] = x.x; qb[b][4 * t + 1] = x.y; qb[b][4 * t + 2] = x.z; qb[b][4 * t + 3] = x.w;
            }
          } else {
#pragma unroll
            for (int k = 0; k < KH; ++k) qb[b][k] = 0.0f;
          }
        } else {
#pragma unroll
          for (int k = 0; k < KH; ++k)
            qb[b][k] = ((FULL || col < col1) && KH * h + k < r) ? Q[(size_t)col * r + KH * h + k] : 0.0f;
        }
      }
      // the two 32-column blocks accumulate in turn: two independent chains on the matrix pipe
      v16f gh0, gh1;
#pragma unroll
      for (int i = 0; i < 16; ++i) { gh0[i] = 0.0f; gh1[i] = 0.0f; }
#pragma unroll
      for (int k = 0; k < KH; ++k) {
        gh0 = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[k], qb[0][k], gh0, 0, 0, 0);
        gh1 = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[k], qb[1][k], gh1, 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        lds[(8 * (v >> 2) + 4 * h + (v & 3)) * kLP + li] = gh0[v];
        lds[(8 * (v >> 2) + 4 * h + (v & 3)) * kLP + 32 + li] = gh1[v];
      }
      wave_lds_fence();
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int rr = 4 * i + sr;
        const float4 t = *reinterpret_cast<const float4*>(lds + rr * kLP + c4);
        if constexpr (HASM) {
          e[i].v[0] -= t.x; e[i].v[1] -= t.y; e[i].v[2] -= t.z; e[i].v[3] -= t.w;
        }
        if (MODE == kMGhatOnly || (MODE == kMResidualGhat && ghat_out)) {
          if constexpr (FULL) {
            const Pk<4> o{{t.x, t.y, t.z, t.w}};
            emit_ghat<4>(ghat_out + (size_t)(row0 + 4 * i) * cols + c, lo, o, update, eta);
          } else if (colok && rr < nrows) {
            const Pk<4> o{{t.x, t.y, t.z, t.w}};
            emit_ghat<4>(ghat_out + (size_t)(row0 + rr) * cols, (unsigned)cl * 4u, o, update, eta);
          }
        }
      }
      wave_lds_fence();
    }
    if constexpr (HASM) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int rr = 4 * i + sr;
        Pk<4> m;
#pragma unroll
        for (int v = 0; v < 4; ++v) m.v[v] = ADD ? g[i].v[v] + e[i].v[v] : e[i].v[v];
        if constexpr (FULL)
          strow<4, NTS>(reinterpret_cast<char*>(M + (size_t)(row0 + 4 * i) * cols + c), lo, m);
        else if (colok && rr < nrows)
          strow<4, NTS>(reinterpret_cast<char*>(M + (size_t)(row0 + rr) * cols), (unsigned)cl * 4u, m);
        if constexpr (ADD)
          *reinterpret_cast<float4*>(lds + rr * kLP + c4) = make_float4(m.v[0], m.v[1], m.v[2], m.v[3]);
      }
    }
    if constexpr (BQ_LATE) {
      __builtin_amdgcn_sched_barrier(0);
      load_bq();
    }
    if constexpr (ADD) {
      wave_lds_fence();
      // two accumulators (even / odd float4 of the lane's run of columns): two independent chains
#pragma unroll
      for (int t = 0; t < 8; t += 2) {
        const float4 a0 = *reinterpret_cast<const float4*>(lds + li * kLP + 32 * h + 4 * t);
        const float4 a1 = *reinterpret_cast<const float4*>(lds + li * kLP + 32 * h + 4 * t + 4);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          accP[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, bq[nb][4 * t + 0], accP[nb], 0, 0, 0);
          accP2[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, bq[nb][4 * t + 4], accP2[nb], 0, 0, 0);
          accP[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, bq[nb][4 * t + 1], accP[nb], 0, 0, 0);
          accP2[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, bq[nb][4 * t + 5], accP2[nb], 0, 0, 0);
          accP[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, bq[nb][4 * t + 2], accP[nb], 0, 0, 0);
          accP2[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, bq[nb][4 * t + 6], accP2[nb], 0, 0, 0);
          accP[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, bq[nb][4 * t + 3], accP[nb], 0, 0, 0);
          accP2[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, bq[nb][4 * t + 7], accP2[nb], 0, 0, 0);
        }
      }
      wave_lds_fence();
    }
  };
  const bool small_offsets = cols < (1 << 26);   // byte offsets within 4 rows fit 32 bits
  for (int c = col0 + 64 * wave; c < col1; c += 256) {
    if (nrows == 32 && c + 64 <= col1 && small_offsets)
      block(std::true_type{}, c);
    else
      block(std::false_type{}, c);
  }
  if constexpr (ADD) {
    // P partial of the item = sum over the four wavefronts, added in wavefront order
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        lds[(8 * (v >> 2) + 4 * h + (v & 3)) * kLP + 32 * nb + li] = accP[nb][v] + accP2[nb][v];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4 * NB; ++i) {
      const int e = (int)threadIdx.x + 256 * i;
      const int rr = e / (32 * NB), k = e % (32 * NB);
      const float t = ((lds_all[0][rr * kLP + k] + lds_all[1][rr * kLP + k]) + lds_all[2][rr * kLP + k]) +
                      lds_all[3][rr * kLP + k];
      if (rr < nrows && k < r) Pp[(size_t)(row0 + rr) * r + k] = t;
    }
  }
}

// ---------------------------------------------------------------------------
// The add modes at rank pad 32 in a narrower form: a wavefront takes 32 rows x 32
// columns per step instead of 32 x 64, which halves the registers of the
// streamed tile, of the G-hat operands and of the Q slice, so that two
// wavefronts fit on a SIMD (with 32 x 64 the fused mode needs more than half
// the register file and runs one wavefront per SIMD, every load exposed).
// Eight wavefronts per workgroup keep the 1 KiB-per-row access of the
// workgroup.  Row layout here: 8 lanes = 128 contiguous bytes of a row, 8 rows
// per instruction.  G-hat elements come out of the same sequence of matrix
// instructions as in the 32 x 64 form (the contraction over the ranks does not
// depend on the column blocking), so the residual modes, which keep that form,
// still match bit for bit.
// ---------------------------------------------------------------------------
constexpr int kLP32 = 36;   // LDS pitch (floats) of a 32 x 32 tile: 16-byte aligned rows

template <int RP, int MODE, bool EXACT, bool GB16, bool NTS>
__device__ __forceinline__ void mfma_tile32(const float* __restrict__ G, float* __restrict__ M,
                                            const float* Q, const float* Pb, float* __restrict__ Pp,
                                            int cols, int r, int row0, int nrows, int col0, int col1,
                                            int lane, int wave, float (*lds_all)[32 * kLP32]) {
  static_assert(RP == 32 && (MODE == kMAdd || MODE == kMAddFused), "narrow form: add modes at rank pad 32");
  float* lds = lds_all[wave];
  constexpr bool NEEDG = (MODE != kMAdd);
  constexpr int KH = RP / 2;
  const int rs = EXACT ? RP : r;   // row length of the operands Q and Pb (r: that of the P partials written)
  const int li = lane & 31, h = lane >> 5;
  const int sr = lane >> 3, c4 = (lane & 7) * 4;   // row layout: rows 8 i + sr, columns c4 .. c4 + 3
  float pa[KH];
  if constexpr (NEEDG) {
    const int row = row0 + li;
    if constexpr (EXACT) {
      if (li < nrows) {
        const float4* src = reinterpret_cast<const float4*>(Pb + (size_t)row * RP + KH * h);
#pragma unroll
        for (int t = 0; t < KH / 4; ++t) {
          const float4 x = src[t];
          pa[4 * t] = x.x; pa[4 * t + 1] = x.y; pa[4 * t + 2] = x.z; pa[4 * t + 3] = x.w;
        }
      } else {
#pragma unroll
        for (int k = 0; k < KH; ++k) pa[k] = 0.0f;
      }
    } else {
#pragma unroll
      for (int k = 0; k < KH; ++k) pa[k] = (li < nrows && KH * h + k < r) ? Pb[(size_t)row * r + KH * h + k] : 0.0f;
    }
  }
  v16f accP, accP2;
#pragma unroll
  for (int i = 0; i < 16; ++i) { accP[i] = 0.0f; accP2[i] = 0.0f; }

  // the G and E (or old M) values of one 32 x 32 block
  auto fetch = [&](auto full_tag, const int c, Pk<4>* g, Pk<4>* e) {
    constexpr bool FULL = decltype(full_tag)::value;
    const int cl = c + c4;
    const bool colok = FULL || cl < col1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rr = 8 * i + sr;
      const bool ok = FULL || (colok && rr < nrows);
      const size_t off = (size_t)(row0 + rr) * cols;
#pragma unroll
      for (int v = 0; v < 4; ++v) { g[i].v[v] = 0.0f; e[i].v[v] = 0.0f; }
      if (ok) {
        g[i] = ldgrad<4, LQSGD_NT_G != 0, GB16>(grad_row<GB16>(G, off), (unsigned)cl * 4u);
        e[i] = ldrow<4, NTS>(reinterpret_cast<const char*>(M + off), (unsigned)cl * 4u);
      }
    }
  };
  auto block = [&](auto full_tag, const int c, Pk<4>* g, Pk<4>* e) {
    constexpr bool FULL = decltype(full_tag)::value;
    const int cl = c + c4;
    const bool colok = FULL || cl < col1;
    if constexpr (NEEDG) {
      float qb[KH];
      const int col = c + li;
      if constexpr (EXACT) {
        if (FULL || col < col1) {
          const float4* src = reinterpret_cast<const float4*>(Q + (size_t)col * RP + KH * h);
#pragma unroll
          for (int t = 0; t < KH / 4; ++t) {
            const float4 x = src[t];
            qb[4 * t] = x.x; qb[4 * t + 1] = x.y; qb[4 * t + 2] = x.z; qb[4 * t + 3] = x.w;
          }
        } else {
#pragma unroll
          for (int k = 0; k < KH; ++k) qb[k] = 0.0f;
        }
      } else {
#pragma unroll
        for (int k = 0; k < KH; ++k)
          qb[k] = ((FULL || col < col1) && KH * h + k < r) ? Q[(size_t)col * r + KH * h + k] : 0.0f;
      }
      v16f gh;
#pragma unroll
      for (int i = 0; i < 16; ++i) gh[i] = 0.0f;
#pragma unroll
      for (int k = 0; k < KH; ++k) gh = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[k], qb[k], gh, 0, 0, 0);
#pragma unroll
      for (int v = 0; v < 16; ++v) lds[(8 * (v >> 2) + 4 * h + (v & 3)) * kLP32 + li] = gh[v];
      wave_lds_fence();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 t = *reinterpret_cast<const float4*>(lds + (8 * i + sr) * kLP32 + c4);
        e[i].v[0] -= t.x; e[i].v[1] -= t.y; e[i].v[2] -= t.z; e[i].v[3] -= t.w;
      }
      wave_lds_fence();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rr = 8 * i + sr;
      Pk<4> m;
#pragma unroll
      for (int v = 0; v < 4; ++v) m.v[v] = g[i].v[v] + e[i].v[v];
      if (FULL || (colok && rr < nrows))
        strow<4, NTS>(reinterpret_cast<char*>(M + (size_t)(row0 + rr) * cols), (unsigned)cl * 4u, m);
      *reinterpret_cast<float4*>(lds + rr * kLP32 + c4) = make_float4(m.v[0], m.v[1], m.v[2], m.v[3]);
    }
    // the Q slice of the P product is fetched only now: the registers of the G-hat operands are free again
    float bq[16];
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      const int col = c + 16 * h + kk;
      if constexpr (FULL && EXACT)
        bq[kk] = Q[(size_t)col * RP + li];
      else
        bq[kk] = (col < col1 && li < rs) ? Q[(size_t)col * rs + li] : 0.0f;
    }
    wave_lds_fence();
    {
      const float4 a0 = *reinterpret_cast<const float4*>(lds + li * kLP32 + 16 * h);
      const float4 a1 = *reinterpret_cast<const float4*>(lds + li * kLP32 + 16 * h + 4);
      const float4 a2 = *reinterpret_cast<const float4*>(lds + li * kLP32 + 16 * h + 8);
      const float4 a3 = *reinterpret_cast<const float4*>(lds + li * kLP32 + 16 * h + 12);
      accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, bq[0], accP, 0, 0, 0);
      accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, bq[4], accP2, 0, 0, 0);
      accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, bq[1], accP, 0, 0, 0);
      accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, bq[5], accP2, 0, 0, 0);
      accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, bq[2], accP, 0, 0, 0);
      accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, bq[6], accP2, 0, 0, 0);
      accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, bq[3], accP, 0, 0, 0);
      accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, bq[7], accP2, 0, 0, 0);
      accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.x, bq[8], accP, 0, 0, 0);
      accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a3.x, bq[12], accP2, 0, 0, 0);
      accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.y, bq[9], accP, 0, 0, 0);
      accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a3.y, bq[13], accP2, 0, 0, 0);
      accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.z, bq[10], accP, 0, 0, 0);
      accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a3.z, bq[14], accP2, 0, 0, 0);
      accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.w, bq[11], accP, 0, 0, 0);
      accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a3.w, bq[15], accP2, 0, 0, 0);
    }
    wave_lds_fence();
  };
  // Interior blocks (all 32 rows and 32 columns exist) run without bounds tests, as a software
  // pipeline inside the wavefront: the next block's G and E are requested before this block's matrix
  // instructions, and the next block's G-hat operand from Q as soon as this block's G-hat is done.
  // Requests complete in order, so everything a block waits for is requested before the prefetch.
  int c = col0 + 32 * wave;
  if (nrows == 32 && c + 32 <= col1 && cols < (1 << 26)) {   // (byte offsets within 8 rows fit 32 bits)
    const int last = c + ((col1 - 32 - c) / 256) * 256;   // this wavefront's last whole block
    Pk<4> g[4], e[4], gn[4], en[4];
    if constexpr (EXACT) {
      float qb[KH], bq[16];
      // Addresses are a wave-uniform base (scalar registers, advanced by scalar adds) plus a byte
      // offset per lane that does not change from block to block.
      const unsigned goff = (unsigned)(sr * cols + c4) * 4u;      // lane's place in a slab of 8 rows
      const unsigned qboff = (unsigned)(li * RP + KH * h) * 4u;   // ... in 32 rows of Q (G-hat operand)
      const unsigned bqoff = (unsigned)(16 * h * RP + li) * 4u;   // ... in 32 rows of Q (P operand)
      auto fetch_ge = [&](const int cb, Pk<4>* gg, Pk<4>* ee) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const size_t off = (size_t)(row0 + 8 * i) * cols + cb;
          if constexpr (GB16) {   // kept packed (two registers) until the block is worked on
            const auto* p = gptr<v2u>(grad_row<GB16>(G, off) + (goff >> 1));
            const v2u t = LQSGD_NT_G ? __builtin_nontemporal_load(p) : *p;
            gg[i].v[0] = __uint_as_float(t.x); gg[i].v[1] = __uint_as_float(t.y);
          } else {
            gg[i] = ldgrad<4, LQSGD_NT_G != 0, GB16>(grad_row<GB16>(G, off), goff);
          }
          ee[i] = ldrow<4, NTS>(reinterpret_cast<const char*>(M + off), goff);
        }
      };
      auto fetch_qb = [&](const int cb) {
        const char* base = reinterpret_cast<const char*>(Q + (size_t)cb * RP);
#pragma unroll
        for (int t = 0; t < KH / 4; ++t) {
          const Pk<4> x = ldrow<4, false>(base + 16 * t, qboff);
          qb[4 * t] = x.v[0]; qb[4 * t + 1] = x.v[1]; qb[4 * t + 2] = x.v[2]; qb[4 * t + 3] = x.v[3];
        }
      };
      fetch_ge(c, g, e);
      if constexpr (NEEDG) fetch_qb(c);
      // one block; MORE: another whole block follows (a constant, so that no branch joins two
      // request histories and every wait counts exactly)
      auto step = [&](auto more_tag, const int c, Pk<4>* g, Pk<4>* e, Pk<4>* gn, Pk<4>* en) {
        constexpr bool more = decltype(more_tag)::value;
        {
          const char* base = reinterpret_cast<const char*>(Q + (size_t)c * RP);
#pragma unroll
          for (int kk = 0; kk < 16; ++kk) bq[kk] = ldrow<1, false>(base + kk * RP * 4, bqoff).v[0];
        }
        if constexpr (more) fetch_ge(c + 256, gn, en);
        __builtin_amdgcn_sched_barrier(0);   // the requests above stay ahead of the arithmetic below
        if constexpr (NEEDG) {
          v16f gh;
#pragma unroll
          for (int i = 0; i < 16; ++i) gh[i] = 0.0f;
#pragma unroll
          for (int k = 0; k < KH; ++k) gh = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[k], qb[k], gh, 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (more) fetch_qb(c + 256);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int v = 0; v < 16; ++v) lds[(8 * (v >> 2) + 4 * h + (v & 3)) * kLP32 + li] = gh[v];
          wave_lds_fence();
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float4 t = *reinterpret_cast<const float4*>(lds + (8 * i + sr) * kLP32 + c4);
            e[i].v[0] -= t.x; e[i].v[1] -= t.y; e[i].v[2] -= t.z; e[i].v[3] -= t.w;
          }
          wave_lds_fence();
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int rr = 8 * i + sr;
          Pk<4> m, gv = g[i];
          if constexpr (GB16) {
            const unsigned x = __float_as_uint(g[i].v[0]), y = __float_as_uint(g[i].v[1]);
            gv.v[0] = __uint_as_float(x << 16); gv.v[1] = __uint_as_float(x & 0xffff0000u);
            gv.v[2] = __uint_as_float(y << 16); gv.v[3] = __uint_as_float(y & 0xffff0000u);
          }
#pragma unroll
          for (int v = 0; v < 4; ++v) m.v[v] = gv.v[v] + e[i].v[v];
          strow<4, NTS>(reinterpret_cast<char*>(M + (size_t)(row0 + 8 * i) * cols + c), goff, m);
          *reinterpret_cast<float4*>(lds + rr * kLP32 + c4) = make_float4(m.v[0], m.v[1], m.v[2], m.v[3]);
        }
        wave_lds_fence();
        {
          const float4 a0 = *reinterpret_cast<const float4*>(lds + li * kLP32 + 16 * h);
          const float4 a1 = *reinterpret_cast<const float4*>(lds + li * kLP32 + 16 * h + 4);
          const float4 a2 = *reinterpret_cast<const float4*>(lds + li * kLP32 + 16 * h + 8);
          const float4 a3 = *reinterpret_cast<const float4*>(lds + li * kLP32 + 16 * h + 12);
          accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, bq[0], accP, 0, 0, 0);
          accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, bq[4], accP2, 0, 0, 0);
          accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, bq[1], accP, 0, 0, 0);
          accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, bq[5], accP2, 0, 0, 0);
          accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, bq[2], accP, 0, 0, 0);
          accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, bq[6], accP2, 0, 0, 0);
          accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, bq[3], accP, 0, 0, 0);
          accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, bq[7], accP2, 0, 0, 0);
          accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.x, bq[8], accP, 0, 0, 0);
          accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a3.x, bq[12], accP2, 0, 0, 0);
          accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.y, bq[9], accP, 0, 0, 0);
          accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a3.y, bq[13], accP2, 0, 0, 0);
          accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.z, bq[10], accP, 0, 0, 0);
          accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a3.z, bq[14], accP2, 0, 0, 0);
          accP = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.w, bq[11], accP, 0, 0, 0);
          accP2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a3.w, bq[15], accP2, 0, 0, 0);
        }
        wave_lds_fence();
      };
      // two blocks per trip, the two register sets changing roles (no copies, so nothing waits for
      // a prefetch before its values are needed)
      for (; c + 256 < last; c += 512) {
        step(std::true_type{}, c, g, e, gn, en);
        step(std::true_type{}, c + 256, gn, en, g, e);
      }
      if (c < last) {
        step(std::true_type{}, c, g, e, gn, en);
        step(std::false_type{}, c + 256, gn, en, g, e);
        c += 512;
      } else {
        step(std::false_type{}, c, g, e, gn, en);
        c += 256;
      }
    } else {
      fetch(std::true_type{}, c, g, e);
      for (; c <= last; c += 256) {
        const bool more = c < last;
        if (more) fetch(std::true_type{}, c + 256, gn, en);
        block(std::true_type{}, c, g, e);
        if (more) {
#pragma unroll
          for (int i = 0; i < 4; ++i) { g[i] = gn[i]; e[i] = en[i]; }
        }
      }
    }
  }
  for (; c < col1; c += 256) {
    Pk<4> g[4], e[4];
    fetch(std::false_type{}, c, g, e);
    block(std::false_type{}, c, g, e);
  }
  // P partial of the item = sum over the eight wavefronts, added in wavefront order
#pragma unroll
  for (int v = 0; v < 16; ++v) lds[(8 * (v >> 2) + 4 * h + (v & 3)) * kLP32 + li] = accP[v] + accP2[v];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int e = (int)threadIdx.x + 512 * i;
    const int rr = e >> 5, k = e & 31;
    float t = lds_all[0][rr * kLP32 + k];
#pragma unroll
    for (int wv = 1; wv < 8; ++wv) t += lds_all[wv][rr * kLP32 + k];
    if (rr < nrows && k < r) Pp[(size_t)(row0 + rr) * r + k] = t;
  }
}

// Rows that are not 16-byte aligned (tiny layers): a plain loop, one wavefront over the rows of its
// share, lanes over columns; the r dot products of a row go through wave sums.
template <int MODE, bool GB16>
__device__ __forceinline__ void plain_rows_fallback(const DevArgs& a, const LayerDesc& ld, const Tile& tl,
                                                    const float* G, float* M, float* Pp, float* ghat_out,
                                                    int col0, int col1, int lane) {
  constexpr bool ADD = (MODE == kMAdd || MODE == kMAddFused);
  constexpr bool NEEDG = (MODE != kMAdd);
  const int cols = ld.cols, r = ld.r;
  const float* Pb = a.Pbar + ld.p_off;
  const float* Q = a.Qbar + ld.q_off;
  for (int row = tl.row0; row < tl.row0 + tl.nrows; ++row) {
    for (int k0 = 0; k0 < (ADD ? r : 1); ++k0) {
      // add modes: pass k0 forms P[row][k0]; the tile itself is updated in pass 0 only
      float dot = 0.0f;
      for (int c = col0 + lane; c < col1; c += kWave) {
        float m;
        if (k0 == 0) {
          float gh = 0.0f;
          if constexpr (NEEDG)
            for (int k = 0; k < r; ++k) gh = fmaf(Pb[(size_t)row * r + k], Q[(size_t)c * r + k], gh);
          if constexpr (MODE == kMGhatOnly) {
            const Pk<1> o{{gh}};
            emit_ghat<1>(ghat_out + (size_t)row * cols, (unsigned)c * 4u, o, a.update, a.eta);
            continue;
          } else {
            float e = M[(size_t)row * cols + c];
            if constexpr (NEEDG) e -= gh;
            m = ADD ? grad_elem<GB16>(G, (size_t)row * cols + c) + e : e;
            M[(size_t)row * cols + c] = m;
            if (MODE == kMResidualGhat && ghat_out) {
              const Pk<1> o{{gh}};
              emit_ghat<1>(ghat_out + (size_t)row * cols, (unsigned)c * 4u, o, a.update, a.eta);
            }
          }
        } else {
          m = M[(size_t)row * cols + c];            // this lane wrote it in pass 0
        }
        if constexpr (ADD) dot = fmaf(m, Q[(size_t)c * r + k0], dot);
      }
      if constexpr (ADD) {
        dot = wave_sum(dot);
        if (lane == 0) Pp[(size_t)row * r + k0] = dot;
      }
    }
  }
}

// Rows that are not 16-byte aligned (cols % 4 != 0; tiny layers) take the plain loop: the register-
// tiled vector code would set the register count of the whole kernel (rank pad x 4 accumulators and
// as many factor values per lane) and with it the number of wavefronts per SIMD of the main path.
template <int RP, int MODE, bool GB16>
__device__ __forceinline__ void mfma_mode_vector_fallback(const DevArgs& a, const LayerDesc& ld, const Tile& tl, int worker,
                                                          const float* G, float* M, float* Pp, float* ghat_out,
                                                          int col0, int col1, int lane) {
  plain_rows_fallback<MODE, GB16>(a, ld, tl, G, M, Pp, ghat_out, col0, col1, lane);
}

// Wavefronts per SIMD the register allocation aims for: two at rank pad 16 (2.65 -> 2.47 ms on
// 8192^2 x 16 workers), one at rank pad 32, where two would spill (3.0 -> 4.6 ms).
template <int RP, int MODE, bool GB16 = false, bool NTS = false>
__global__ __launch_bounds__(256, RP <= 16 ? 2 : 1) void mfma_sweep_kernel(DevArgs a, const Tile* __restrict__ tiles, int ntiles, int reverse) {
  __shared__ __attribute__((aligned(16))) float lds_all[4][32 * kLP];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  if ((MODE == kMAdd || MODE == kMAddFused) && blockIdx.x == 0) zero_absmax_cells(a, 256);
  const Tile tl = tiles[reverse ? ntiles - 1 - (int)blockIdx.x : (int)blockIdx.x];   // one item per workgroup
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const float* G = (MODE == kMAdd || MODE == kMAddFused) ? a.grads[(size_t)worker * a.n_all + ld.gidx] : nullptr;
  float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + ld.ppart_off + (size_t)tl.aux * ld.np_pad;
  float* ghat_out = nullptr;
  if ((MODE == kMResidualGhat || MODE == kMGhatOnly) && worker == 0 && a.ghat) ghat_out = a.ghat[ld.gidx];
  if (MODE == kMGhatOnly && !ghat_out) return;
  const int col0 = tl.aux * ld.segw;
  const int col1 = min(ld.cols, col0 + ld.segw);
  if (ld.vec != 4) {
    // tiny layers: the vector code, eight of the item's rows per wavefront
    Tile sub = tl;
    sub.row0 = tl.row0 + 8 * wave;
    sub.nrows = min(8, tl.nrows - 8 * wave);
    if (sub.nrows > 0) mfma_mode_vector_fallback<RP, MODE, GB16>(a, ld, sub, worker, G, M, Pp, ghat_out, col0, col1, lane);
    return;
  }
  if (a.Qpad)   // operands with rows of RP ranks, zero beyond the layer's rank
    mfma_tile<RP, MODE, true, GB16, NTS>(G, M, a.Qpad + ld.qpad_off, a.Ppad + ld.ppad_off, Pp, ghat_out, ld.cols, ld.r, tl.row0,
                              tl.nrows, col0, col1, lane, wave, lds_all, a.update, a.eta);
  else if (ld.r == RP)
    mfma_tile<RP, MODE, true, GB16, NTS>(G, M, a.Qbar + ld.q_off, a.Pbar + ld.p_off, Pp, ghat_out, ld.cols, ld.r, tl.row0,
                              tl.nrows, col0, col1, lane, wave, lds_all, a.update, a.eta);
  else
    mfma_tile<RP, MODE, false, GB16, NTS>(G, M, a.Qbar + ld.q_off, a.Pbar + ld.p_off, Pp, ghat_out, ld.cols, ld.r, tl.row0,
                               tl.nrows, col0, col1, lane, wave, lds_all, a.update, a.eta);
}

template <int RP, int MODE, bool GB16, bool NTS>
__global__ __launch_bounds__(512, 2) void mfma_sweep32_kernel(DevArgs a, const Tile* __restrict__ tiles, int ntiles, int reverse) {
  __shared__ __attribute__((aligned(16))) float lds_all[8][32 * kLP32];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  if (blockIdx.x == 0) zero_absmax_cells(a, 512);
  const Tile tl = tiles[reverse ? ntiles - 1 - (int)blockIdx.x : (int)blockIdx.x];   // one item per workgroup
  const int layer = tl.lw / a.W, worker = tl.lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const float* G = a.grads[(size_t)worker * a.n_all + ld.gidx];
  float* M = a.E + (size_t)worker * a.m_stride + ld.m_off;
  float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + ld.ppart_off + (size_t)tl.aux * ld.np_pad;
  const int col0 = tl.aux * ld.segw;
  const int col1 = min(ld.cols, col0 + ld.segw);
  if (ld.vec != 4) {
    // tiny layers: the vector code, four of the item's rows per wavefront
    Tile sub = tl;
    sub.row0 = tl.row0 + 4 * wave;
    sub.nrows = min(4, tl.nrows - 4 * wave);
    if (sub.nrows > 0) mfma_mode_vector_fallback<RP, MODE, GB16>(a, ld, sub, worker, G, M, Pp, nullptr, col0, col1, lane);
    return;
  }
  if (a.Qpad)
    mfma_tile32<RP, MODE, true, GB16, NTS>(G, M, a.Qpad + ld.qpad_off, a.Ppad + ld.ppad_off, Pp, ld.cols, ld.r, tl.row0, tl.nrows,
                                      col0, col1, lane, wave, lds_all);
  else if (ld.r == RP)
    mfma_tile32<RP, MODE, true, GB16, NTS>(G, M, a.Qbar + ld.q_off, a.Pbar + ld.p_off, Pp, ld.cols, ld.r, tl.row0, tl.nrows,
                                      col0, col1, lane, wave, lds_all);
  else
    mfma_tile32<RP, MODE, false, GB16, NTS>(G, M, a.Qbar + ld.q_off, a.Pbar + ld.p_off, Pp, ld.cols, ld.r, tl.row0, tl.nrows,
                                       col0, col1, lane, wave, lds_all);
}

// Copies of the aggregated factors with rows of RP ranks (zero beyond the layer's rank) for the
// matrix-core sweeps 0 / 2.  blockIdx.y = layer; which: 0 = P-bar, 1 = Q-bar.
__global__ __launch_bounds__(256) void pad_factor_kernel(DevArgs a, int RP, int which) {
  const LayerDesc& ld = a.layers[blockIdx.y];
  const int n = which ? ld.cols : ld.rows, r = ld.r;
  const float* src = which ? a.Qbar + ld.q_off : a.Pbar + ld.p_off;
  float* dst = which ? a.Qpad + ld.qpad_off : a.Ppad + ld.ppad_off;
  const long long total = (long long)n * RP;
  for (long long e = blockIdx.x * 256 + threadIdx.x; e < total; e += gridDim.x * 256) {
    const long long row = e / RP;
    const int k = (int)(e - row * RP);
    dst[e] = k < r ? src[row * r + k] : 0.0f;
  }
}

// ---------------------------------------------------------------------------
// orth of tall factors at rank pads >= 8: Cholesky-QR, applied twice.
// The column-by-column form above pays one exchange between the slices of a
// factor per column (about 10 us each: r = 32 columns cost 0.33 ms on a factor
// of 8192 rows, where all the arithmetic is a few microseconds).  Here the
// slices exchange the r x r Gram matrix G = P^T P once per pass instead:
//   G = R^T R (Cholesky),  P <- P R^-1.
// In exact arithmetic R is the triangular factor of the QR decomposition of P,
// so P R^-1 is what Gram-Schmidt (Algorithm 1's Orthogonalize) returns; in
// float32 one pass loses orthogonality in proportion to cond(P)^2, and a second
// pass on its result restores it to rounding level (the usual "CholeskyQR2").
// That only holds while cond(P)^2 stays well below 1/epsilon: if a pivot of
// either factorisation falls below kCholPivotFloor of its column's squared
// norm (or a column is zero), the pair is done again from the start by the
// column-by-column form, whose result does not depend on conditioning in that
// way.  Every slice of a pair factorises the same total, so all take the same
// decision.
// Steps of a pass, per workgroup (= 256 rows, one per thread, in registers):
//   * the slice's Gram matrix on the matrix cores (rows are re-read from the
//     plane this workgroup has just written, in "lane = column" layout), the
//     four wavefronts' parts added in wavefront order;
//   * exchange: entry e of the total is owned by slice e / ceil(NE / nslice),
//     which collects that entry from every slice, adds them up in slice order
//     and publishes the total; every slice then collects all totals.  Entries
//     are tagged 64-bit words as in orth_coop_kernel: two round trips per pass
//     instead of one per column, and no workgroup reads more than 2 NE words;
//   * wavefront 0 factorises (lane l keeps row l of G in registers; right-
//     looking elimination with lane broadcasts), every thread then applies
//     R^-1 to its row by forward substitution, reading R from LDS.
// phase -1 runs all of it in one cooperative launch.  Without one, phases 0, 1
// and 2 are three ordinary launches that pass the slices' Gram matrices through
// plain memory (cpart) and add them up in the same order, so that both forms
// give the same bits; pairs that need the column-by-column form raise redo[pair]
// and the guarded orth_wide_kernel launches that follow do them.
// ---------------------------------------------------------------------------
// On the CPU, in float32, two passes stay as close to the float64 Gram-Schmidt as float32 Gram-Schmidt
// itself down to pivot ratios of about 1e-6 (both 1e-6 .. 1e-5 away at ratios 2e-4 .. 1e-5); the floor
// keeps two orders of magnitude from where the factorisation starts to break down.
constexpr float kCholPivotFloor = 1e-4f;

template <int RP>
struct CholShape {
  static_assert(RP == 8 || RP == 16 || RP == 32 || RP == 64, "rank pads with a Cholesky-QR form");
  static constexpr int NB = RP <= 32 ? 1 : 3;                       // 32 x 32 blocks kept: (0,0) or (0,0), (0,1), (1,1)
  static constexpr int NE = RP <= 32 ? RP * RP : 3 * 1024;          // entries exchanged
  static constexpr int QN = (NE + 255) / 256;                       // ... per thread
  static constexpr int GN = (NE + kCoopMaxSlices + 255) / 256;      // entries a thread collects as an owner
  static constexpr int kPoolA = 4 * NE, kPoolB = (kCoopMaxSlices + 5) * RP;
  static constexpr int POOL = kPoolA > kPoolB ? kPoolA : kPoolB;    // LDS floats
};

// Where <column i, column j>, i <= j, sits among the exchanged entries.
template <int RP>
__device__ __forceinline__ int chol_entry(int i, int j) {
  if constexpr (RP <= 32) {
    return i * RP + j;
  } else {
    return j < 32 ? i * 32 + j : (i < 32 ? 1024 + i * 32 + (j - 32) : 2048 + (i - 32) * 32 + (j - 32));
  }
}

// The Gram matrix of the slice's 256 rows of `orth`: on return thread t holds entries t, t + 256, ...
// in gsum.  pool: 4 NE floats of LDS, free again on return.
template <int RP>
__device__ __forceinline__ void chol_slice_gram(const float* orth, int rows, int r, int row0, float* pool,
                                                float (&gsum)[CholShape<RP>::QN]) {
  using S = CholShape<RP>;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int li = lane & 31, h = lane >> 5;
  v16f acc[S::NB];
#pragma unroll
  for (int b = 0; b < S::NB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;
  constexpr int U = 16;                           // row pairs loaded ahead of their matrix instructions
  const int c0 = min(li, r - 1), c1 = min(32 + li, r - 1);
  const bool ok0 = li < r, ok1 = 32 + li < r;
#pragma unroll 1
  for (int b = 0; b < 32 / U; ++b) {
    float x0[U], x1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = row0 + wave * 64 + 2 * (b * U + u) + h;
      const float* src = orth + (size_t)min(row, rows - 1) * r;      // every load is in bounds; masked below
      x0[u] = keep_if(src[c0], ok0 && row < rows);
      if constexpr (RP == 64) x1[u] = keep_if(src[c1], ok1 && row < rows);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(x0[u], x0[u], acc[0], 0, 0, 0);
      if constexpr (RP == 64) {
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(x0[u], x1[u], acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(x1[u], x1[u], acc[2], 0, 0, 0);
      }
    }
  }
  // D layout: register v of lane (li, h) is element (8 (v / 4) + 4 h + v % 4, li) of the block
  float* mine = pool + wave * S::NE;
#pragma unroll
  for (int b = 0; b < S::NB; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int m = 8 * (v >> 2) + 4 * h + (v & 3);
      if constexpr (RP <= 32) {
        if (m < RP && li < RP) mine[m * RP + li] = acc[b][v];
      } else {
        mine[b * 1024 + m * 32 + li] = acc[b][v];
      }
    }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < S::QN; ++q) {
    const int e = tid + 256 * q;
    gsum[q] = (e < S::NE) ? (pool[e] + pool[S::NE + e]) + (pool[2 * S::NE + e] + pool[3 * S::NE + e]) : 0.0f;
  }
  __syncthreads();
}

__device__ __forceinline__ unsigned long long table_wait(const unsigned long long* p, unsigned long long x, unsigned tag,
                                                         int* status, unsigned max_polls) {
  unsigned polls = 0;
  while ((unsigned)(x >> 32) != tag) {
    if (++polls >= max_polls) {
      __hip_atomic_store(status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      break;
    }
    __builtin_amdgcn_s_sleep(1);
    x = table_load(p);
  }
  return x;
}

// The slices' Gram matrices -> their total, in LDS at pool + 2 NE, through the tagged table
// `tab` ([nslice_max + 1][NE]: one plane per slice, the totals in the last one).
template <int RP>
__device__ __forceinline__ void chol_exchange(const float (&gsum)[CholShape<RP>::QN], unsigned long long* tab, int slice,
                                              int nslice, int nslice_max, unsigned tag_part, unsigned tag_total, float* pool,
                                              int* status, unsigned max_polls) {
  using S = CholShape<RP>;
  const int tid = threadIdx.x;
#pragma unroll
  for (int q = 0; q < S::QN; ++q) {
    const int e = tid + 256 * q;
    if (e < S::NE)
      __hip_atomic_store(tab + (size_t)slice * S::NE + e, ((unsigned long long)tag_part << 32) | __float_as_uint(gsum[q]),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // the entries this slice owns, from every slice: item = (entry, slice)
  const int share = (S::NE + nslice - 1) / nslice;
  const int e0 = slice * share;
  const int cnt = max(0, min(S::NE - e0, share));
  const int nitem = cnt * nslice;                  // <= NE + nslice
  unsigned long long x[S::GN];
  const unsigned long long* src[S::GN];
#pragma unroll
  for (int i = 0; i < S::GN; ++i) {
    const int it = tid + 256 * i;
    const int el = it / nslice, sl = it - el * nslice;
    src[i] = tab + (size_t)sl * S::NE + e0 + el;
    x[i] = (it < nitem) ? table_load(src[i]) : ((unsigned long long)tag_part << 32);
  }
#pragma unroll
  for (int i = 0; i < S::GN; ++i) {
    const int it = tid + 256 * i;
    if (it < nitem) {
      x[i] = table_wait(src[i], x[i], tag_part, status, max_polls);
      pool[it] = __uint_as_float((unsigned)x[i]);
    }
  }
  __syncthreads();
  unsigned long long* totals = tab + (size_t)nslice_max * S::NE;
  for (int el = tid; el < cnt; el += 256) {
    float t = 0.0f;
    for (int sl = 0; sl < nslice; ++sl) t += pool[el * nslice + sl];
    __hip_atomic_store(totals + e0 + el, ((unsigned long long)tag_total << 32) | __float_as_uint(t), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  }
  unsigned long long y[S::QN];
#pragma unroll
  for (int q = 0; q < S::QN; ++q) {
    const int e = tid + 256 * q;
    y[q] = (e < S::NE) ? table_load(totals + e) : ((unsigned long long)tag_total << 32);
  }
#pragma unroll
  for (int q = 0; q < S::QN; ++q) {
    const int e = tid + 256 * q;
    if (e < S::NE) {
      y[q] = table_wait(totals + e, y[q], tag_total, status, max_polls);
      pool[2 * S::NE + e] = __uint_as_float((unsigned)y[q]);
    }
  }
  __syncthreads();
}

// The same total from the slices' matrices in plain memory (written by an earlier launch).
template <int RP>
__device__ __forceinline__ void chol_sum_parts(const float* parts, int nslice, float* pool) {
  using S = CholShape<RP>;
  const int tid = threadIdx.x;
#pragma unroll
  for (int q = 0; q < S::QN; ++q) {
    const int e = tid + 256 * q;
    if (e < S::NE) {
      float t = 0.0f;
      for (int sl = 0; sl < nslice; ++sl) t += parts[(size_t)sl * S::NE + e];
      pool[2 * S::NE + e] = t;
    }
  }
  __syncthreads();
}

__device__ __forceinline__ float lane_value(float x, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}

// One wavefront: G (total, at T) = L L^T.  Lane l works on row l.  Leaves L at Ls ([RP][RP], row
// major, lower triangle; the diagonal holds 1 / L_jj; rows and columns >= r are those of the
// identity) and returns whether every pivot stayed above the floor -- the same in every lane.
template <int RP>
__device__ __forceinline__ bool chol_factor(const float* T, float* Ls, int r, int lane) {
  const int l = min(lane, RP - 1);
  float g[RP];
#pragma unroll
  for (int k = 0; k < RP; ++k) g[k] = T[chol_entry<RP>(min(k, l), max(k, l))];
  float diag0 = 0.0f;
#pragma unroll
  for (int k = 0; k < RP; ++k)
    if (k == l) diag0 = g[k];
  bool ok = true;
  static_for<RP>([&](auto J) {
    constexpr int j = decltype(J)::value;
    if (j < r) {
      const float d = lane_value(g[j], j), d0 = lane_value(diag0, j);
      ok = ok && (d0 > FLT_MIN) && (d > kCholPivotFloor * d0);        // false for NaN as well
      const float rinv = 1.0f / sqrtf(d);
      const float lj = (lane >= j) ? g[j] * rinv : 0.0f;               // column j of L
#pragma unroll
      for (int k = j + 1; k < RP; ++k) g[k] = fmaf(-lj, lane_value(lj, k), g[k]);
      g[j] = (lane == j) ? rinv : lj;
    } else {
      g[j] = (lane == j) ? 1.0f : 0.0f;
    }
  });
  if (lane < RP) {
#pragma unroll
    for (int k = 0; k < RP; ++k) Ls[lane * RP + k] = g[k];
  }
  return ok;
}

// p <- p R^-1 with R = L^T: forward substitution along the row.
template <int RP>
__device__ __forceinline__ void chol_solve_row(float (&p)[RP], const float* Ls, int r) {
  static_for<RP>([&](auto J) {
    constexpr int j = decltype(J)::value;
    if (j < r) {                                   // p[j] is zero beyond the rank and stays so
      float acc = p[j];
#pragma unroll
      for (int i = 0; i < j; ++i) acc = fmaf(-p[i], Ls[j * RP + i], acc);
      p[j] = acc * Ls[j * RP + j];
    }
  });
}

// The slice's block of P_w = the sum of the sweep-0 planes, written to `pre` and `orth`.  The block is
// one contiguous run of nflt floats in every plane and in both outputs, so the threads walk it in
// 16-byte pieces, fully coalesced (a thread per row would touch 64 cache lines per load).
template <int RP>
__device__ __forceinline__ void chol_sum_planes(const float* planes, int nseg, size_t plane_stride, float* pre_s, float* orth_s,
                                                int nflt) {
  const int tid = threadIdx.x;
  const bool vec = (((reinterpret_cast<uintptr_t>(planes) | reinterpret_cast<uintptr_t>(pre_s) |
                      reinterpret_cast<uintptr_t>(orth_s)) & 15) == 0) && (plane_stride & 3) == 0;
  if (vec) {
    constexpr int NI = RP / 4;
    float4 acc[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) acc[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int sg = 0; sg < nseg; ++sg) {
      const float* src = planes + (size_t)sg * plane_stride;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int f = 4 * (tid + 256 * i);
        if (f + 4 <= nflt) {
          const float4 t = *reinterpret_cast<const float4*>(src + f);
          acc[i].x += t.x; acc[i].y += t.y; acc[i].z += t.z; acc[i].w += t.w;
        }
      }
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int f = 4 * (tid + 256 * i);
      if (f + 4 <= nflt) {
        *reinterpret_cast<float4*>(pre_s + f) = acc[i];
        *reinterpret_cast<float4*>(orth_s + f) = acc[i];
      }
    }
    const int f = (nflt & ~3) + tid;               // what is left of a block whose length is no multiple of 4
    if (tid < (nflt & 3)) {
      float t = 0.0f;
      for (int sg = 0; sg < nseg; ++sg) t += planes[(size_t)sg * plane_stride + f];
      pre_s[f] = t;
      orth_s[f] = t;
    }
  } else {
    float acc[RP];
#pragma unroll
    for (int i = 0; i < RP; ++i) acc[i] = 0.0f;
    for (int sg = 0; sg < nseg; ++sg) {
      const float* src = planes + (size_t)sg * plane_stride;
#pragma unroll
      for (int i = 0; i < RP; ++i) {
        const int f = tid + 256 * i;
        if (f < nflt) acc[i] += src[f];
      }
    }
#pragma unroll
    for (int i = 0; i < RP; ++i) {
      const int f = tid + 256 * i;
      if (f < nflt) {
        pre_s[f] = acc[i];
        orth_s[f] = acc[i];
      }
    }
  }
}

// Row `row` of a rows x r factor (zero beyond r and for a thread without a row): whole-row loads that may
// run into what follows the row, as in load_slice.
template <int RP>
__device__ __forceinline__ void chol_load_row(const float* F, int row, int rows, int r, float (&v)[RP]) {
  load_row<RP>(F, min(row, rows - 1), r, r == RP, v);
  const bool live = row < rows;
#pragma unroll
  for (int k = 0; k < RP; ++k) v[k] = keep_if(v[k], live);
}

template <int RP>
__device__ __forceinline__ void chol_store_row(float* F, int row, int rows, int r, const float (&v)[RP]) {
  if (row >= rows) return;
  if (r == RP) {
    float* b = F + (size_t)row * RP;
#pragma unroll
    for (int k = 0; k < RP; k += 4) *reinterpret_cast<float4*>(b + k) = make_float4(v[k], v[k + 1], v[k + 2], v[k + 3]);
  } else if ((r & 1) == 0) {
    float* b = F + (size_t)row * r;
#pragma unroll
    for (int k = 0; k < RP; k += 2)
      if (k < r) *reinterpret_cast<float2*>(b + k) = make_float2(v[k], v[k + 1]);
  } else {
    float* b = F + (size_t)row * r;
#pragma unroll
    for (int k = 0; k < RP; ++k)
      if (k < r) b[k] = v[k];
  }
}

template <int RP>
__global__ __launch_bounds__(256, 2) void orth_chol_kernel(DevArgs a, int nslice_max, int max_rank, int phase,
                                                        unsigned long long* ctable, float* cpart, int* redo,
                                                        unsigned long long epoch, unsigned max_polls) {
  using S = CholShape<RP>;
  __shared__ __attribute__((aligned(16))) float pool[S::POOL];
  __shared__ float redmax[4];
  __shared__ int flag;
  const int lw = blockIdx.x / nslice_max, slice = blockIdx.x - lw * nslice_max;
  const int layer = lw / a.W, worker = lw - layer * a.W;
  const LayerDesc& ld = a.layers[layer];
  const int rows = ld.rows, r = ld.r;
  const int nslice = (rows + 255) >> 8;
  if (slice >= nslice) return;                   // workgroup-uniform
  if (phase == 2 && redo[lw] != 0) return;       // raised in phase 1, or by a faster slice just now: the pair is done again anyway
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  const int row = slice * 256 + tid;
  float* pre = a.Ppre + (size_t)worker * a.p_stride + ld.p_off;
  float* orth = a.Porth + (size_t)worker * a.p_stride + ld.p_off;
  float* scale = a.scaleP + (size_t)worker * a.L + layer;
  unsigned long long* tab = ctable + (size_t)lw * (nslice_max + 1) * S::NE;
  float* parts = cpart + (size_t)lw * nslice_max * S::NE;
  float* Ls = pool;                              // [RP][RP], once the total has been read out of pool + 2 NE
  float v[RP];
#pragma unroll
  for (int k = 0; k < RP; ++k) v[k] = 0.0f;
  if (phase <= 0) {
    if (slice == 0 && tid == 0) {
      if (phase == 0) {
        redo[lw] = 0;
        if (!a.orth_shared) *scale = 0.0f;
      } else if (!a.orth_shared) {
        // shared by all slices, raised with atomics at the end; every slice reads an entry that
        // slice 0 publishes after this store before it gets there
        __hip_atomic_store(scale, 0.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
      }
    }
    {
      const float* Pp = a.Ppart + (size_t)worker * a.ppart_stride + (a.orth_shared ? ld.p_off : ld.ppart_off);
      const size_t base = (size_t)slice * 256 * r;
      chol_sum_planes<RP>(Pp + base, a.orth_shared ? 1 : ld.nseg, (size_t)ld.np_pad, pre + base, orth + base,
                          min(256, rows - slice * 256) * r);
    }
  }
  float gsum[S::QN];
  bool good = true;
  if (phase == 0) {
    __syncthreads();                             // the rows above, for the loads in "lane = column" layout
    chol_slice_gram<RP>(orth, rows, r, slice * 256, pool, gsum);
  } else {
    const int first = phase < 0 ? 0 : phase - 1, last = phase < 0 ? 1 : phase - 1;
    for (int pass = first; pass <= last; ++pass) {
      if (phase < 0) {
        __syncthreads();
        chol_slice_gram<RP>(orth, rows, r, slice * 256, pool, gsum);
        const unsigned tag = (unsigned)(epoch * 4ull) + 2u * (unsigned)pass;
        chol_exchange<RP>(gsum, tab, slice, nslice, nslice_max, tag + 1u, tag + 2u, pool, a.status, max_polls);
      } else {
        chol_sum_parts<RP>(parts, nslice, pool);
      }
      if (wave == 0) {
        const bool ok = chol_factor<RP>(pool + 2 * S::NE, Ls, r, lane);
        if (lane == 0) flag = ok ? 1 : 0;
      }
      __syncthreads();
      good = flag != 0;
      if (!good) break;
      // the thread's row as the previous step left it in memory (not kept in registers across the
      // factorisation, which needs them)
      chol_load_row<RP>(orth, row, rows, r, v);
      chol_solve_row<RP>(v, Ls, r);
      chol_store_row<RP>(orth, row, rows, r, v);
      __syncthreads();                           // Ls and flag are written again by the next pass
    }
    if (phase == 1 && good) chol_slice_gram<RP>(orth, rows, r, slice * 256, pool, gsum);
  }
  if (phase == 0 || (phase == 1 && good)) {
#pragma unroll
    for (int q = 0; q < S::QN; ++q) {
      const int e = tid + 256 * q;
      if (e < S::NE) parts[(size_t)slice * S::NE + e] = gsum[q];
    }
    return;
  }
  if (!good) {
    if (phase > 0) {
      if (slice == 0 && tid == 0) redo[lw] = 1;
      return;
    }
    // one launch: column by column from the sum of the planes, as orth_coop_kernel does
    chol_load_row<RP>(pre, row, rows, r, v);
    const size_t pstride = (size_t)a.L * a.W * nslice_max * RP;
    coop_columns<RP>(v, r, lw, slice, nslice, nslice_max, max_rank, a.orth_table, epoch, a.status, max_polls, pstride,
                     pool + kCoopMaxSlices * RP, pool + (kCoopMaxSlices + 4) * RP, pool);
    chol_store_row<RP>(orth, row, rows, r, v);
  }
  float mx = 0.0f;
#pragma unroll
  for (int k = 0; k < RP; ++k)
    if (k < r) mx = fmaxf(mx, fabsf(v[k]));
  mx = wave_max(mx);
  if (lane == 0) redmax[wave] = mx;
  __syncthreads();
  if (tid == 0 && !a.orth_shared) {
    const float m = fmaxf(fmaxf(redmax[0], redmax[1]), fmaxf(redmax[2], redmax[3]));
    atomicMax(reinterpret_cast<unsigned int*>(scale), __float_as_uint(m));
  }
}

}  // namespace

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
// Every launcher notes the device function it has just launched, template arguments included, in
// the form a profiler's kernel list shows it (without namespaces and parameter list), so that a
// timing slot of the API can be matched to a profile.
namespace {
thread_local char g_launched[96] = "";
__attribute__((format(printf, 1, 2))) void note_kernel(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  std::vsnprintf(g_launched, sizeof g_launched, fmt, ap);
  va_end(ap);
}
const char* tf(bool b) { return b ? "true" : "false"; }
}  // namespace
const char* last_launched_kernel() { return g_launched; }

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

// The Gram-Schmidt kernels also exist at rank pad 64 (the streaming sweeps run on the matrix cores there).
#define LQSGD_RP_SWITCH_ORTH(RPV, CALL)                 \
  if ((RPV) == 64) { constexpr int RP = 64; CALL; } else \
    LQSGD_RP_SWITCH(RPV, CALL)

hipError_t launch_add_project(int rp, const DevArgs& a, const Tile* tiles, int ntiles, int fuse_residual, int reverse,
                              hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  const dim3 grid((ntiles + 3) / 4), block(256);
#define LQSGD_LAUNCH_A(FUSE, GB) \
  if (a.nt_store) { LQSGD_RP_SWITCH(rp, (add_project_kernel<RP, FUSE, GB, true><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse))); } \
  else { LQSGD_RP_SWITCH(rp, (add_project_kernel<RP, FUSE, GB, false><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse))); }
  if (a.g_bf16) {
    if (fuse_residual) { LQSGD_LAUNCH_A(true, true) } else { LQSGD_LAUNCH_A(false, true) }
  } else if (fuse_residual) {
    LQSGD_LAUNCH_A(true, false)
  } else {
    LQSGD_LAUNCH_A(false, false)
  }
#undef LQSGD_LAUNCH_A
  note_kernel("add_project_kernel<%d, %s, %s, %s>", rp, tf(fuse_residual), tf(a.g_bf16), tf(a.nt_store));
  return hipGetLastError();
}

// Register-resident Gram-Schmidt where rows-per-lane x rank fits the register
// file comfortably; the in-memory kernel otherwise.
template <int RP, int RPT, int BS>
void launch_orth_reg(const DevArgs& a, dim3 grid, hipStream_t s) {
  if constexpr (RP * RPT <= (BS == 256 ? (RPT == 2 ? 128 : 64) : 48)) {
    orth_reg_kernel<RP, RPT, BS><<<grid, dim3(BS), 0, s>>>(a);
    note_kernel("orth_reg_kernel<%d, %d, %d>", RP, RPT, BS);
  } else {
    orth_kernel<RP><<<grid, dim3(256), 0, s>>>(a);
    note_kernel("orth_kernel<%d>", RP);
  }
}

// One cooperative launch if every workgroup of the grid can be resident at once; returns false
// (nothing launched) otherwise, and the caller takes the one-launch-per-column path.
template <int RP>
bool try_orth_coop(int nslice, int max_rank, const DevArgs& a, int nblocks, CoopState* cs, hipStream_t s) {
  if (cs->capacity < 0) {                        // resident workgroups of this kernel on the context's device
    int dev = 0, coop = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, orth_coop_kernel<RP>, 256, 0) != hipSuccess) {
      (void)hipGetLastError();
      cs->capacity = 0;
    } else {
      cs->capacity = coop ? cus * per_cu : 0;
    }
  }
  if (nblocks > cs->capacity) return false;
  DevArgs args = a;
  unsigned long long* table = a.orth_table;
  unsigned long long n = cs->epoch;
  int* status = a.status;
  unsigned max_polls = cs->max_polls ? cs->max_polls : kTablePolls;
  void* params[] = {&args, &nslice, &max_rank, &table, &n, &status, &max_polls};
  const hipError_t e = hipLaunchCooperativeKernel(reinterpret_cast<void*>(orth_coop_kernel<RP>), dim3(nblocks), dim3(256),
                                                  params, 0, s);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  cs->epoch += 1;                                // the tags of a launch are epoch * max_rank + 1 ... + max_rank
  note_kernel("orth_coop_kernel<%d>", RP);
  return true;
}

bool launch_orth_coop(int rp, int nslice, int max_rank, const DevArgs& a, int nblocks, CoopState* cs, hipStream_t s) {
#ifdef LQSGD_TUNING
  static const bool enabled = [] { const char* e = std::getenv("LQSGD_ORTH_COOP"); return !(e && e[0] == '0'); }();
  if (!enabled) return false;
#endif
  if (!cs || !a.orth_table || !a.status || nslice > kCoopMaxSlices) return false;
  // Under stream capture the launch would be replayed with this launch's epoch baked in, and the
  // tags of one replay would be indistinguishable from the next one's: take the per-column path.
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &cap) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  if (cap != hipStreamCaptureStatusNone) return false;
  switch (rp) {
    case 1: return try_orth_coop<1>(nslice, max_rank, a, nblocks, cs, s);
    case 2: return try_orth_coop<2>(nslice, max_rank, a, nblocks, cs, s);
    case 4: return try_orth_coop<4>(nslice, max_rank, a, nblocks, cs, s);
    case 8: return try_orth_coop<8>(nslice, max_rank, a, nblocks, cs, s);
    case 16: return try_orth_coop<16>(nslice, max_rank, a, nblocks, cs, s);
    case 32: return try_orth_coop<32>(nslice, max_rank, a, nblocks, cs, s);
    case 64: return try_orth_coop<64>(nslice, max_rank, a, nblocks, cs, s);
    default: return false;
  }
}

// The Cholesky-QR form in one cooperative launch; false (nothing launched) if the grid cannot be
// resident at once or the stream is being captured.
template <int RP>
bool try_orth_chol_coop(int nslice, int max_rank, const DevArgs& a, int nblocks, CoopState* cs, hipStream_t s) {
  if (cs->chol_capacity < 0) {
    int dev = 0, coop = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, orth_chol_kernel<RP>, 256, 0) != hipSuccess) {
      (void)hipGetLastError();
      cs->chol_capacity = 0;
    } else {
      cs->chol_capacity = coop ? cus * per_cu : 0;
    }
  }
  if (nblocks > cs->chol_capacity) return false;
  DevArgs args = a;
  int phase = -1;
  unsigned long long* table = a.chol_table;
  float* part = a.chol_part;
  int* redo = a.chol_redo;
  unsigned long long n = cs->epoch;
  unsigned max_polls = cs->max_polls ? cs->max_polls : kTablePolls;
  void* params[] = {&args, &nslice, &max_rank, &phase, &table, &part, &redo, &n, &max_polls};
  const hipError_t e = hipLaunchCooperativeKernel(reinterpret_cast<void*>(orth_chol_kernel<RP>), dim3(nblocks), dim3(256),
                                                  params, 0, s);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  cs->epoch += 1;                                // tags of this launch: 4 epoch + 1 .. + 4, and the columns' as above
  note_kernel("orth_chol_kernel<%d>", RP);
  return true;
}

bool launch_orth_chol_coop(int rp, int nslice, int max_rank, const DevArgs& a, int nblocks, CoopState* cs, hipStream_t s) {
  if (!cs || !a.chol_table || !a.orth_table || !a.status || nslice > kCoopMaxSlices) return false;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &cap) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  if (cap != hipStreamCaptureStatusNone) return false;      // a replay would repeat this launch's tags
  switch (rp) {
    case 8: return try_orth_chol_coop<8>(nslice, max_rank, a, nblocks, cs, s);
    case 16: return try_orth_chol_coop<16>(nslice, max_rank, a, nblocks, cs, s);
    case 32: return try_orth_chol_coop<32>(nslice, max_rank, a, nblocks, cs, s);
    case 64: return try_orth_chol_coop<64>(nslice, max_rank, a, nblocks, cs, s);
    default: return false;
  }
}

// Three launches of the Cholesky-QR kernel, then the column-by-column launches for the pairs that raised their word.
template <int RP>
void launch_orth_chol_split(int nslice, int max_rank, const DevArgs& a, int nblocks, hipStream_t s) {
  for (int phase = 0; phase < 3; ++phase)
    orth_chol_kernel<RP><<<dim3(nblocks), dim3(256), 0, s>>>(a, nslice, max_rank, phase, nullptr, a.chol_part, a.chol_redo, 0ull, 0u);
  for (int j = 0; j <= max_rank; ++j)
    orth_wide_kernel<RP><<<dim3(nblocks), dim3(256), 0, s>>>(a, j, nslice, a.chol_redo);
  note_kernel("orth_chol_kernel<%d> x 3 launches", RP);
}

int chol_entries(int rp) {
  return rp == 8 ? CholShape<8>::NE : rp == 16 ? CholShape<16>::NE : rp == 32 ? CholShape<32>::NE : rp == 64 ? CholShape<64>::NE : 0;
}

hipError_t launch_orth(int rp, int max_rows, int max_rank, const DevArgs& a, CoopState* coop, hipStream_t s) {
  if (a.L <= 0) return hipSuccess;
  const dim3 grid(a.L * a.W);
  const int nslice = (max_rows + 255) / 256;
  // Tall factors and too few (layer, worker) pairs to fill 256 CUs with one workgroup
  // each, or no register-resident variant for this rank: one launch per column.
  const bool reg_fits = (max_rows <= 512 && rp * 2 <= 128) || (max_rows <= 2048 && rp * 8 <= 64) ||
                        (max_rows <= 4096 && rp * 4 <= 48) || (max_rows <= 11264 && rp * 11 <= 48);
  if (a.orth_part && nslice >= 8 && ((int)grid.x < 128 || !reg_fits)) {
#ifdef LQSGD_TUNING
    static const bool chol = [] { const char* e = std::getenv("LQSGD_ORTH_CHOL"); return !(e && e[0] == '0'); }();
#else
    constexpr bool chol = true;
#endif
    if (chol && rp >= 8 && a.chol_part && a.chol_redo) {
      if (launch_orth_chol_coop(rp, nslice, max_rank, a, (int)grid.x * nslice, coop, s)) return hipSuccess;
      if (rp == 8) launch_orth_chol_split<8>(nslice, max_rank, a, (int)grid.x * nslice, s);
      else if (rp == 16) launch_orth_chol_split<16>(nslice, max_rank, a, (int)grid.x * nslice, s);
      else if (rp == 32) launch_orth_chol_split<32>(nslice, max_rank, a, (int)grid.x * nslice, s);
      else launch_orth_chol_split<64>(nslice, max_rank, a, (int)grid.x * nslice, s);
      return hipGetLastError();
    }
    if (launch_orth_coop(rp, nslice, max_rank, a, (int)grid.x * nslice, coop, s)) return hipSuccess;
    for (int j = 0; j <= max_rank; ++j) {
      LQSGD_RP_SWITCH_ORTH(rp, (orth_wide_kernel<RP><<<dim3(grid.x * nslice), dim3(256), 0, s>>>(a, j, nslice, nullptr)));
    }
    note_kernel("orth_wide_kernel<%d> x %d launches", rp, max_rank + 1);
    return hipGetLastError();
  }
  if (max_rows <= 512) {
    LQSGD_RP_SWITCH_ORTH(rp, (launch_orth_reg<RP, 2, 256>(a, grid, s)));
  } else if (max_rows <= 2048) {
    LQSGD_RP_SWITCH_ORTH(rp, (launch_orth_reg<RP, 8, 256>(a, grid, s)));
  } else if (max_rows <= 4096) {
    LQSGD_RP_SWITCH_ORTH(rp, (launch_orth_reg<RP, 4, 1024>(a, grid, s)));
  } else if (max_rows <= 11264) {
    LQSGD_RP_SWITCH_ORTH(rp, (launch_orth_reg<RP, 11, 1024>(a, grid, s)));
  } else {
    LQSGD_RP_SWITCH_ORTH(rp, (orth_kernel<RP><<<grid, dim3(256), 0, s>>>(a)));
    note_kernel("orth_kernel<%d>", rp);
  }
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
  note_kernel("exchange_kernel<%d>", mode);
  return hipGetLastError();
}

hipError_t launch_back_project(int rp, const DevArgs& a, const Tile* tiles, int ntiles, const VTile* vtiles, int nvtiles,
                               int reverse, hipStream_t s) {
  if (ntiles + nvtiles <= 0) return hipSuccess;
  const dim3 grid(ntiles + nvtiles), block(256);
  LQSGD_RP_SWITCH(rp, (back_project_kernel<RP><<<grid, block, 0, s>>>(a, tiles, ntiles, vtiles, reverse)));
  note_kernel("back_project_kernel<%d>", rp);
  return hipGetLastError();
}

hipError_t launch_back_project_mfma(int rp, const DevArgs& a, const Tile* tiles, int ntiles, const VTile* vtiles, int nvtiles,
                                    int reverse, hipStream_t s) {
  if (ntiles + nvtiles <= 0) return hipSuccess;
  if (rp == 64)
    back_project_mfma_kernel<2><<<dim3(ntiles + nvtiles), dim3(256), 0, s>>>(a, tiles, ntiles, vtiles, reverse);
  else
    back_project_mfma_kernel<1><<<dim3(ntiles + nvtiles), dim3(256), 0, s>>>(a, tiles, ntiles, vtiles, reverse);
  note_kernel("back_project_mfma_kernel<%d>", rp == 64 ? 2 : 1);
  return hipGetLastError();
}

hipError_t launch_reduce_q(int phase, const DevArgs& a, const RTile* tiles, int ntiles, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  reduce_q_kernel<<<dim3(ntiles), dim3(256), 0, s>>>(a, tiles, phase);
  note_kernel("reduce_q_kernel");
  return hipGetLastError();
}

hipError_t launch_residual(int rp, int mode, const DevArgs& a, const Tile* tiles, int ntiles, int reverse, hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  const dim3 grid(ntiles), block(256);
  switch (mode) {
    case kResidual: LQSGD_RP_SWITCH(rp, (residual_kernel<RP, kResidual><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse))); break;
    case kResidualGhat: LQSGD_RP_SWITCH(rp, (residual_kernel<RP, kResidualGhat><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse))); break;
    case kGhatOnly: LQSGD_RP_SWITCH(rp, (residual_kernel<RP, kGhatOnly><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse))); break;
    default: return hipErrorInvalidValue;
  }
  note_kernel("residual_kernel<%d, %d>", rp, mode);
  return hipGetLastError();
}

// A tuning build (-DLQSGD_TUNING) can keep the 32 x 64 form at rank pad 32 for comparisons (LQSGD_MFMA_NARROW32=0).
static bool narrow32() {
#ifdef LQSGD_TUNING
  static const bool on = [] { const char* e = std::getenv("LQSGD_MFMA_NARROW32"); return !(e && e[0] == '0'); }();
  return on;
#else
  return true;
#endif
}

template <int RP>
hipError_t launch_mfma_sweep_rp(int mode, int full_rank, const DevArgs& a, const Tile* tiles, int ntiles, int reverse,
                                hipStream_t s) {
  const dim3 grid(ntiles), block(256);
  switch (mode) {
    case kMAdd:
      // same form as the fused mode below, so that P comes out of one summation order whether or
      // not the residual update is deferred
      if constexpr (RP == 32) {
        if (narrow32() && full_rank) {
          if (a.g_bf16) { if (a.nt_store) mfma_sweep32_kernel<32, kMAdd, true, true><<<grid, dim3(512), 0, s>>>(a, tiles, ntiles, reverse);
                          else mfma_sweep32_kernel<32, kMAdd, true, false><<<grid, dim3(512), 0, s>>>(a, tiles, ntiles, reverse); }
          else { if (a.nt_store) mfma_sweep32_kernel<32, kMAdd, false, true><<<grid, dim3(512), 0, s>>>(a, tiles, ntiles, reverse);
                 else mfma_sweep32_kernel<32, kMAdd, false, false><<<grid, dim3(512), 0, s>>>(a, tiles, ntiles, reverse); }
          break;
        }
      }
      if (a.g_bf16) { if (a.nt_store) mfma_sweep_kernel<RP, kMAdd, true, true><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse);
                      else mfma_sweep_kernel<RP, kMAdd, true, false><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse); }
      else { if (a.nt_store) mfma_sweep_kernel<RP, kMAdd, false, true><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse);
             else mfma_sweep_kernel<RP, kMAdd, false, false><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse); }
      break;
    case kMAddFused:
      // the narrow form pays where the fused mode would otherwise run one wavefront per SIMD and every
      // layer fills the rank pad (measured on 8192^2 x 16: r = 32 2.77 -> 2.60 ms; at r = 30 it costs
      // 3.11 -> 3.22 ms, so ranks below the pad stay with the 32 x 64 form)
      if constexpr (RP == 32) {
        if (narrow32() && full_rank) {
          if (a.g_bf16) { if (a.nt_store) mfma_sweep32_kernel<32, kMAddFused, true, true><<<grid, dim3(512), 0, s>>>(a, tiles, ntiles, reverse);
                          else mfma_sweep32_kernel<32, kMAddFused, true, false><<<grid, dim3(512), 0, s>>>(a, tiles, ntiles, reverse); }
          else { if (a.nt_store) mfma_sweep32_kernel<32, kMAddFused, false, true><<<grid, dim3(512), 0, s>>>(a, tiles, ntiles, reverse);
                 else mfma_sweep32_kernel<32, kMAddFused, false, false><<<grid, dim3(512), 0, s>>>(a, tiles, ntiles, reverse); }
          break;
        }
      }
      if (a.g_bf16) { if (a.nt_store) mfma_sweep_kernel<RP, kMAddFused, true, true><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse);
                      else mfma_sweep_kernel<RP, kMAddFused, true, false><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse); }
      else { if (a.nt_store) mfma_sweep_kernel<RP, kMAddFused, false, true><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse);
             else mfma_sweep_kernel<RP, kMAddFused, false, false><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse); }
      break;
    case kMResidual: mfma_sweep_kernel<RP, kMResidual><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse); break;
    case kMResidualGhat: mfma_sweep_kernel<RP, kMResidualGhat><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse); break;
    case kMGhatOnly: mfma_sweep_kernel<RP, kMGhatOnly><<<grid, block, 0, s>>>(a, tiles, ntiles, reverse); break;
    default: return hipErrorInvalidValue;
  }
  {
    const bool add = mode == kMAdd || mode == kMAddFused;
    if (add && RP == 32 && narrow32() && full_rank)
      note_kernel("mfma_sweep32_kernel<32, %d, %s, %s>", mode, tf(a.g_bf16), tf(a.nt_store));
    else
      note_kernel("mfma_sweep_kernel<%d, %d, %s, %s>", RP, mode, tf(add && a.g_bf16), tf(add && a.nt_store));
  }
  return hipGetLastError();
}

hipError_t launch_mfma_sweep(int rp, int mode, int full_rank, const DevArgs& a, const Tile* tiles, int ntiles, int reverse,
                             hipStream_t s) {
  if (ntiles <= 0) return hipSuccess;
  if (rp == 16) return launch_mfma_sweep_rp<16>(mode, full_rank, a, tiles, ntiles, reverse, s);
  if (rp == 32) return launch_mfma_sweep_rp<32>(mode, full_rank, a, tiles, ntiles, reverse, s);
  if (rp == 64) return launch_mfma_sweep_rp<64>(mode, full_rank, a, tiles, ntiles, reverse, s);
  return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------
// Scratch memory for the entry point that allocates nothing: one block per GPU,
// part of the loaded code object, held until the process ends.  The name below
// is a host-side handle only; the block's device address is asked for once per
// device and that address is what kernels and copies use.  (The array itself
// is defined at file scope, at the top of this file.)
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)LQSGD_STATIC_SCRATCH_BYTES;

hipError_t static_scratch(int device, void** ptr, size_t* bytes) {
  constexpr int kMaxDev = 64;
  static void* addr[kMaxDev] = {};              // per device; the caller serialises calls
  if (device < 0 || device >= kMaxDev) return hipErrorInvalidDevice;
  if (!addr[device]) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return e;
    if (cur != device) return hipErrorInvalidDevice;     // the address belongs to the device that is current
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[device] = p;
  }
  *ptr = addr[device];
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

namespace {
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* p, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
    p[i] = make_uint4(0u, 0u, 0u, 0u);
}
}  // namespace

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if ((reinterpret_cast<uintptr_t>(p) | bytes) & 15u) return hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>(2048, (n16 + 255) / 256);
  fill_zero_kernel<<<dim3(grid), dim3(256), 0, s>>>(static_cast<uint4*>(p), n16);
  return hipGetLastError();
}

hipError_t launch_pad_factor(int RP, int which, const DevArgs& a, hipStream_t s) {
  if (a.L <= 0 || !a.Ppad || !a.Qpad) return hipSuccess;
  pad_factor_kernel<<<dim3(64, a.L), dim3(256), 0, s>>>(a, RP, which);
  return hipGetLastError();
}

}  // namespace lqsgd
