// Device-side argument block and the launchers of the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>

#include "lqsgd_plan.h"

namespace lqsgd {

// Passed by value to every kernel (lands in the kernarg segment, read with
// scalar loads).  All pointers are device pointers.
struct DevArgs {
  const LayerDesc* layers;
  const VecDesc* vecs;
  const float* const* grads;   // W * n_all gradient tensors (fp32, or bfloat16 behind the same pointer type if g_bf16)
  float* const* ghat;          // n_all optional outputs (entries may be null), or null
  float* E;                    // residual / M = G + E, per worker
  float* Ppart;                // sweep-0 partial products, per worker
  float* Ppre;                 // P_w before Gram-Schmidt
  float* Porth;                // P_w after Gram-Schmidt
  float* orth_part;            // [2][L*W][ceil(max_rows/256)][RP] slice partials of the many-workgroup Gram-Schmidt
  unsigned long long* orth_table;      // [2][L*W][ceil(max_rows/256)][RP] tagged partials of its one-launch form
  // Cholesky-QR form of the tall Gram-Schmidt (rank pads >= 16; all three null if the context has none):
  unsigned long long* chol_table;      // [L*W][ceil(max_rows/256) + 1][NE] tagged Gram matrices of the slices, their total last
  float* chol_part;            // [L*W][ceil(max_rows/256)][NE] the same matrices in plain memory, for the form of three launches
  int* chol_redo;              // [L*W] raised for a pair that has to be done column by column
  int* status;                 // pinned host word the kernels raise when a bounded device-side wait expires
  float* Pbar;                 // aggregated P (shared)
  float* Qpart;                // sweep-1 partial products, per worker
  float* Qw;                   // Q_w
  float* Qbar;                 // aggregated Q = warm-start Q (shared)
  float* Ppad; float* Qpad;    // copies of Pbar / Qbar with rows of RP ranks, zero beyond a layer's rank; null if unused
  uint8_t* magP; uint8_t* sgnP; float* scaleP;   // packets of the P exchange
  uint8_t* magQ; uint8_t* sgnQ; float* scaleQ;   // packets of the Q exchange
  const float* thrP; const float* levP;           // quantiser tables for b_p
  const float* thrQ; const float* levQ;           // ... and b_q
  float* vmean;
  int64_t m_stride, p_stride, q_stride, ppart_stride, qpart_stride;
  int64_t magp_stride, sgnp_stride, magq_stride, sgnq_stride;
  int32_t W, L, n_all, bits_p, bits_q;
  float alpha;                 // log scale of Eq. (5)
  float qscale_p, qscale_q;    // (2^b - 1) / log2(1 + alpha) for b_p, b_q
  int32_t agg_first;           // aggregate-first order: scaleP is an atomic-max accumulator (sweep 0 zeroes it)
  int32_t orth_shared;         // the Gram-Schmidt kernels run once per layer, in place on the plane at Ppart + p_off
  int32_t g_bf16;              // the gradient tensors hold bfloat16 values (G-hat / parameters stay fp32)
  int32_t update;              // G-hat outputs are parameters to update: w <- w - eta G-hat
  int32_t nt_store;            // sweep 0 streams the residual slabs: non-temporal loads of E and stores of M (the launchers pick the kernels built that way)
  float eta;
};

enum ExchangeMode { kQuantOnly = 0, kMeanOnly = 1, kFused = 2 };

// The device function the calling thread's most recent launcher call has launched, with its
// template arguments, as a profiler's kernel list names it (namespaces and parameters left out).
const char* last_launched_kernel();

// Each launcher enqueues one kernel on `s` and returns hipGetLastError().
// `reverse` walks the work list backwards: consecutive sweeps alternate direction so that
// each one starts on the data the previous one touched last (still in the memory-side cache).
// fuse_residual: the buffer E holds last iteration's M and the residual update
// E = M - P-bar Q-bar^T is applied on the fly (see add_project_kernel).
hipError_t launch_add_project(int RP, const DevArgs& a, const Tile* tiles, int ntiles, int fuse_residual, int reverse,
                              hipStream_t s);
// What a context keeps for the one-launch (cooperative) Gram-Schmidt of tall factors.
struct CoopState {
  unsigned long long epoch = 0;   // launches made so far: makes the tags in `a.orth_table` unique
  int capacity = -1;              // workgroups of that kernel that fit the context's device at once (-1: not asked yet)
  int chol_capacity = -1;         // the same for the Cholesky-QR kernel
  unsigned max_polls = 0;         // bound of a device-side wait; 0 = the default (about a second)
};
// Entries of the r x r Gram matrix that the slices of a factor exchange at rank pad RP (NE above); 0 if
// the Cholesky-QR form does not exist at that pad.
int chol_entries(int RP);
// coop: NULL disables the one-launch forms.
hipError_t launch_orth(int RP, int max_rows, int max_rank, const DevArgs& a, CoopState* coop, hipStream_t s);
hipError_t launch_exchange(int mode, int phase, const DevArgs& a, const XTile* tiles, int ntiles, hipStream_t s);
// Sweep 1 also runs the plain mean of the 1-D tensors (nvtiles extra workgroups).  Layers whose
// items cover all their rows (LayerDesc::direct_q) get Q_w and its absmax from this sweep itself.
hipError_t launch_back_project(int RP, const DevArgs& a, const Tile* tiles, int ntiles, const VTile* vtiles, int nvtiles,
                               int reverse, hipStream_t s);
// The same sweep on the matrix cores (rank pad 32 or 64; tiles are row block x 512-column group).
hipError_t launch_back_project_mfma(int RP, const DevArgs& a, const Tile* tiles, int ntiles, const VTile* vtiles, int nvtiles,
                                    int reverse, hipStream_t s);
// phase 1: Q_w from sweep 1's row-block planes; phase 0: the raw P_w from sweep 0's column-segment
// planes (aggregate-first order, where the exchange comes before Gram-Schmidt).
hipError_t launch_reduce_q(int phase, const DevArgs& a, const RTile* tiles, int ntiles, hipStream_t s);
// mode: 0 = residual for all workers, 1 = residual + G-hat, 2 = G-hat only (tiles of worker 0).
hipError_t launch_residual(int RP, int mode, const DevArgs& a, const Tile* tiles, int ntiles, int reverse, hipStream_t s);

// Sweeps 0 and 2 on the matrix cores (rank pad 16, 32 or 64), over the work list of
// sweep 0 (32-row items).  mode: 0 = M = G + E and P partials, 1 = the same with the deferred
// residual applied on the fly, 2 = residual, 3 = residual + G-hat, 4 = G-hat only (worker 0's items).
// full_rank: the largest effective rank of the layers equals RP (chooses between two forms of the fused add mode).
// Refreshes a.Ppad (which = 0) or a.Qpad (which = 1) from the tightly packed factor.
hipError_t launch_pad_factor(int RP, int which, const DevArgs& a, hipStream_t s);

// The per-GPU scratch block of the entry point that allocates nothing: device address and size of
// the block of `device`, which must be the current device on the first call for it.
#ifndef LQSGD_STATIC_SCRATCH_BYTES
#define LQSGD_STATIC_SCRATCH_BYTES (32u << 20)
#endif
hipError_t static_scratch(int device, void** ptr, size_t* bytes);
// Clears `bytes` (a multiple of 16) at the 16-byte aligned device address p with a kernel.
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);

hipError_t launch_mfma_sweep(int RP, int mode, int full_rank, const DevArgs& a, const Tile* tiles, int ntiles, int reverse,
                             hipStream_t s);

}  // namespace lqsgd
