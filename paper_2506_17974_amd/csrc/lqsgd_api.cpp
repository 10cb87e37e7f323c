// C ABI of the LQ-SGD compressor: context, device state, phase sequencing,
// taps and timing.  All arithmetic of the method runs in the kernels; this
// file only moves bytes and launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "lqsgd.h"
#include "lqsgd_kernels.h"
#include "lqsgd_plan.h"

using namespace lqsgd;

namespace {

thread_local std::string g_create_error;

enum State { kIdle = 0, kPCompressed = 1, kPDone = 2, kQCompressed = 3 };

struct EventPair {
  hipEvent_t a, b;
  int kernel;
};

}  // namespace

struct lqsgd_ctx {
  Plan plan;
  hipStream_t stream = nullptr;
  int device = 0;
  State state = kIdle;
  int sweep_dir = 0;        // direction of the next streaming sweep (alternates)
  bool flip = true;
  bool eager = false;       // LQSGD_FLAG_EAGER_RESIDUAL
  bool pending = false;     // E buffer holds M; E = M - P-bar Q-bar^T not applied yet
  CoopState coop;           // one-launch Gram-Schmidt: launch count, device capacity, wait bound
  int* status = nullptr;    // pinned, device-visible: non-zero once a bounded device-side wait has expired
  std::string err;
  std::vector<void*> allocs;
  // When set, device memory is carved out of this caller-provided block instead of being allocated
  // (the context then owns no device memory at all).
  unsigned char* arena = nullptr;
  size_t arena_cap = 0, arena_used = 0;
  DevArgs args{};
  // device copies of the work lists
  Tile* d_tilesA = nullptr; Tile* d_tilesB = nullptr; Tile* d_tilesG = nullptr; Tile* d_tilesBM = nullptr; Tile* d_tilesAG = nullptr;
  XTile* d_tilesXP = nullptr; XTile* d_tilesXQ = nullptr;
  RTile* d_tilesRQ = nullptr; RTile* d_tilesRP = nullptr; VTile* d_tilesV = nullptr;
  // pointer tables
  const float** d_grads = nullptr; float** d_ghat = nullptr;
  std::vector<const float*> h_grads; std::vector<float*> h_ghat;
  bool grads_valid = false, ghat_valid = false;
  bool ppad_stale = true, qpad_stale = true;   // the padded copies of P-bar / Q-bar lag behind the factors
  bool alias_checked = false;   // the bound gradient and output tables have been checked against each other
  // timing
  std::string launched[LQSGD_KERNEL_COUNT];   // device function last launched for each timing slot
  bool timing = false;
  std::vector<EventPair> events;
  size_t events_used = 0;
};

namespace {

int fail(lqsgd_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_create_error = msg;
  return code;
}

int fail_hip(lqsgd_ctx* c, hipError_t e, const char* what) {
  // Clear the sticky error so that a later call does not report it again.
  (void)hipGetLastError();
  return fail(c, LQSGD_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define HIP_TRY(ctx, expr)                                   \
  do {                                                       \
    hipError_t e_ = (expr);                                  \
    if (e_ != hipSuccess) return fail_hip(ctx, e_, #expr);   \
  } while (0)

template <typename T>
int dev_alloc(lqsgd_ctx* c, T** out, size_t count, bool zero) {
  *out = nullptr;
  if (count == 0) count = 1;
  if (c->arena) {     // bump allocation, 256-byte granules; the block is cleared as a whole by whoever set it up
    const size_t bytes = (count * sizeof(T) + 255) & ~(size_t)255;
    if (bytes > c->arena_cap - c->arena_used) {
      char buf[200];
      std::snprintf(buf, sizeof buf, "this configuration needs more scratch memory than the static buffer holds (%zu bytes)",
                    c->arena_cap);
      return fail(c, LQSGD_EUNSUPPORTED, buf);
    }
    *out = reinterpret_cast<T*>(c->arena + c->arena_used);
    c->arena_used += bytes;
    return LQSGD_OK;
  }
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, count * sizeof(T));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    char buf[160];
    std::snprintf(buf, sizeof buf, "hipMalloc of %zu bytes failed: %s", count * sizeof(T), hipGetErrorString(e));
    return fail(c, LQSGD_ENOMEM, buf);
  }
  c->allocs.push_back(p);
  if (zero) HIP_TRY(c, hipMemsetAsync(p, 0, count * sizeof(T), c->stream));
  *out = static_cast<T*>(p);
  return LQSGD_OK;
}

template <typename T>
int dev_upload(lqsgd_ctx* c, T** out, const std::vector<T>& v) {
  int rc = dev_alloc(c, out, v.size(), false);
  if (rc) return rc;
  if (!v.empty()) HIP_TRY(c, hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return LQSGD_OK;
}

struct Timed {
  lqsgd_ctx* c;
  int kernel;
  EventPair* ep = nullptr;
  Timed(lqsgd_ctx* ctx, int k) : c(ctx), kernel(k) {
    if (!c->timing) return;
    if (c->events_used == c->events.size()) {
      EventPair p{};
      if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) { (void)hipGetLastError(); return; }
      c->events.push_back(p);
    }
    ep = &c->events[c->events_used++];
    ep->kernel = kernel;
    (void)hipEventRecord(ep->a, c->stream);
  }
  ~Timed() {
    if (ep) (void)hipEventRecord(ep->b, c->stream);
    c->launched[kernel] = last_launched_kernel();
  }
};

// Waits for the context's stream and reports a device-side wait that expired.
int sync_stream(lqsgd_ctx* c) {
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (c->status && *static_cast<volatile int*>(c->status) != 0)
    return fail(c, LQSGD_EHIP, "a device-side barrier wait expired; results of this context are invalid");
  return LQSGD_OK;
}

int check_matrix_layer(lqsgd_ctx* c, int32_t layer, const LayerDesc** out) {
  if (layer < 0 || layer >= c->plan.n_all) return fail(c, LQSGD_ESHAPE, "layer index out of range");
  const int k = c->plan.kind_of[layer];
  if (k < 0) return fail(c, LQSGD_ESHAPE, "layer is a VECTOR layer");
  *out = &c->plan.layers[k];
  return LQSGD_OK;
}

int check_worker(lqsgd_ctx* c, int32_t worker) {
  if (worker < 0 || worker >= c->plan.W) return fail(c, LQSGD_ESHAPE, "worker index out of range");
  return LQSGD_OK;
}

// Copies the caller's pointer list to the device table when it changed.
int bind_grads(lqsgd_ctx* c, const float* const* grads) {
  const size_t n = (size_t)c->plan.W * c->plan.n_all;
  for (size_t i = 0; i < n; ++i) {
    if (!grads[i]) return fail(c, LQSGD_EINVAL, "NULL gradient pointer");
    if (reinterpret_cast<uintptr_t>(grads[i]) & 15u) return fail(c, LQSGD_EINVAL, "gradient pointer not 16-byte aligned");
  }
  if (c->grads_valid && std::memcmp(c->h_grads.data(), grads, n * sizeof(float*)) == 0) return LQSGD_OK;
  HIP_TRY(c, hipStreamSynchronize(c->stream));   // the old table may still be in use
  c->h_grads.assign(grads, grads + n);
  HIP_TRY(c, hipMemcpy(c->d_grads, c->h_grads.data(), n * sizeof(float*), hipMemcpyHostToDevice));
  c->grads_valid = true;
  c->alias_checked = false;
  return LQSGD_OK;
}

int bind_ghat(lqsgd_ctx* c, float* const* ghat) {
  if (!ghat) { c->args.ghat = nullptr; return LQSGD_OK; }
  const size_t n = (size_t)c->plan.n_all;
  for (size_t i = 0; i < n; ++i)
    if (ghat[i] && (reinterpret_cast<uintptr_t>(ghat[i]) & 15u))
      return fail(c, LQSGD_EINVAL, "G-hat pointer not 16-byte aligned");
  if (!(c->ghat_valid && std::memcmp(c->h_ghat.data(), ghat, n * sizeof(float*)) == 0)) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->h_ghat.assign(ghat, ghat + n);
    HIP_TRY(c, hipMemcpy(c->d_ghat, c->h_ghat.data(), n * sizeof(float*), hipMemcpyHostToDevice));
    c->ghat_valid = true;
    c->alias_checked = false;
  }
  c->args.ghat = c->d_ghat;
  return LQSGD_OK;
}

// ---- the phases -------------------------------------------------------------
int next_dir(lqsgd_ctx* c) {
  const int d = c->sweep_dir;
  if (c->flip) c->sweep_dir ^= 1;
  return d;
}

// Matrix-core sweeps 0 / 2 read P-bar and Q-bar from copies with padded rows when some layer has
// fewer ranks than the register pad; whoever writes a factor marks its copy stale.
int refresh_padded(lqsgd_ctx* c, bool need_p, bool need_q) {
  if (!c->plan.padded) return LQSGD_OK;
  // While the stream is being captured the flags describe the moment of the capture, not of a later
  // replay (a host upload may come in between): every copy that is needed is then refreshed, and
  // the flags are left as they were.
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(c->stream, &cap) != hipSuccess) { (void)hipGetLastError(); cap = hipStreamCaptureStatusNone; }
  const bool capturing = cap != hipStreamCaptureStatusNone;
  if (need_p && (c->ppad_stale || capturing)) {
    HIP_TRY(c, launch_pad_factor(c->plan.RP, 0, c->args, c->stream));
    if (!capturing) c->ppad_stale = false;
  }
  if (need_q && (c->qpad_stale || capturing)) {
    HIP_TRY(c, launch_pad_factor(c->plan.RP, 1, c->args, c->stream));
    if (!capturing) c->qpad_stale = false;
  }
  return LQSGD_OK;
}
int full_rank(const lqsgd_ctx* c) { return (c->plan.max_rank == c->plan.RP || c->plan.padded) ? 1 : 0; }

// The one-launch Gram-Schmidt's state, or null where the context must not launch cooperatively.
CoopState* coop_state(lqsgd_ctx* c) {
  return (c->plan.cfg.flags & LQSGD_FLAG_NO_COOPERATIVE_LAUNCH) ? nullptr : &c->coop;
}

int run_sweep0(lqsgd_ctx* c) {
  if (c->plan.mfma_a)
    if (int rc = refresh_padded(c, c->pending, true)) return rc;
  { Timed t(c, LQSGD_KERNEL_ADD_PROJECT);
    if (c->plan.mfma_a)
      HIP_TRY(c, launch_mfma_sweep(c->plan.RP, c->pending ? 1 : 0, full_rank(c), c->args, c->d_tilesA, (int)c->plan.tilesA.size(),
                                   next_dir(c), c->stream));
    else
      HIP_TRY(c, launch_add_project(c->plan.RP, c->args, c->d_tilesA, (int)c->plan.tilesA.size(), c->pending ? 1 : 0,
                                    next_dir(c), c->stream)); }
  c->pending = false;
  if (c->plan.agg_first) {   // the exchange comes first: only add up the partial planes (and take the absmax)
    Timed t(c, LQSGD_KERNEL_REDUCE_P);
    HIP_TRY(c, launch_reduce_q(0, c->args, c->d_tilesRP, (int)c->plan.tilesRP.size(), c->stream));
  } else {
    Timed t(c, LQSGD_KERNEL_ORTH);
    HIP_TRY(c, launch_orth(c->plan.RP, c->plan.max_rows, c->plan.max_rank, c->args, coop_state(c), c->stream));
  }
  return LQSGD_OK;
}
// Aggregate-first order: Gram-Schmidt once per layer, in place on the aggregated P; the aggregate
// as it was before goes to worker 0's slot of the (otherwise unused) per-worker Gram-Schmidt output.
int run_orth_shared(lqsgd_ctx* c) {
  Timed t(c, LQSGD_KERNEL_ORTH);
  DevArgs a = c->args;
  a.W = 1;
  a.orth_shared = 1;
  a.Ppart = c->args.Pbar; a.ppart_stride = 0;
  a.Ppre = c->args.Porth;
  a.Porth = c->args.Pbar;
  HIP_TRY(c, launch_orth(c->plan.RP, c->plan.max_rows, c->plan.max_rank, a, coop_state(c), c->stream));
  c->ppad_stale = true;
  return LQSGD_OK;
}
int run_exchange(lqsgd_ctx* c, int mode, int phase) {
  { Timed t(c, phase ? LQSGD_KERNEL_EXCHANGE_Q : LQSGD_KERNEL_EXCHANGE_P);
    const auto& tl = phase ? c->plan.tilesXQ : c->plan.tilesXP;
    DevArgs a = c->args;
    if (c->plan.agg_first && phase == 0) a.Porth = c->args.Ppre;   // the raw factors are what gets quantised
    HIP_TRY(c, launch_exchange(mode, phase, a, phase ? c->d_tilesXQ : c->d_tilesXP, (int)tl.size(), c->stream));
    if (mode != kQuantOnly) (phase ? c->qpad_stale : c->ppad_stale) = true; }
  if (c->plan.agg_first && phase == 0 && mode != kQuantOnly) return run_orth_shared(c);
  return LQSGD_OK;
}
int run_sweep1(lqsgd_ctx* c, bool with_vectors) {
  { Timed t(c, LQSGD_KERNEL_BACK_PROJECT);
    const int nv = with_vectors ? (int)c->plan.tilesV.size() : 0;
    if (c->plan.mfma)
      HIP_TRY(c, launch_back_project_mfma(c->plan.RP, c->args, c->d_tilesBM, (int)c->plan.tilesBM.size(), c->d_tilesV, nv,
                                          next_dir(c), c->stream));
    else
      HIP_TRY(c, launch_back_project(c->plan.RP, c->args, c->d_tilesB, (int)c->plan.tilesB.size(), c->d_tilesV, nv,
                                     next_dir(c), c->stream)); }
  if (!c->plan.tilesRQ.empty()) {      // layers whose sweep-1 items each cover all rows have stored Q_w themselves
    Timed t(c, LQSGD_KERNEL_REDUCE_Q);
    HIP_TRY(c, launch_reduce_q(1, c->args, c->d_tilesRQ, (int)c->plan.tilesRQ.size(), c->stream)); }
  return LQSGD_OK;
}
// End of an iteration: either apply E = M - P-bar Q-bar^T now (eager), or leave M
// in place and let the next iteration's first sweep apply it on the fly; G-hat,
// when asked for, is then written by a pass of its own over the layers.
int run_sweep2(lqsgd_ctx* c, bool write_ghat) {
  const Plan& p = c->plan;
  if (p.mfma_a && (c->eager || write_ghat))
    if (int rc = refresh_padded(c, true, true)) return rc;
  Timed t(c, LQSGD_KERNEL_RESIDUAL);
  if (c->eager) {
    if (p.mfma_a)
      HIP_TRY(c, launch_mfma_sweep(p.RP, write_ghat ? 3 : 2, full_rank(c), c->args, c->d_tilesA, (int)p.tilesA.size(), next_dir(c), c->stream));
    else
      HIP_TRY(c, launch_residual(p.RP, write_ghat ? 1 : 0, c->args, c->d_tilesB, (int)p.tilesB.size(), next_dir(c), c->stream));
  } else {
    if (write_ghat) {
      if (p.mfma_a)
        HIP_TRY(c, launch_mfma_sweep(p.RP, 4, full_rank(c), c->args, c->d_tilesAG, (int)p.tilesAG.size(), 0, c->stream));
      else
        HIP_TRY(c, launch_residual(p.RP, 2, c->args, c->d_tilesG, (int)p.tilesG.size(), 0, c->stream));
    }
    c->pending = true;
  }
  return LQSGD_OK;
}
// Applies a deferred residual update, so that the buffer holds E again.
int materialise(lqsgd_ctx* c) {
  if (!c->pending) return LQSGD_OK;
  const Plan& p = c->plan;
  if (p.mfma_a)
    if (int rc = refresh_padded(c, true, true)) return rc;
  Timed t(c, LQSGD_KERNEL_RESIDUAL);
  if (p.mfma_a)
    HIP_TRY(c, launch_mfma_sweep(p.RP, 2, full_rank(c), c->args, c->d_tilesA, (int)p.tilesA.size(), next_dir(c), c->stream));
  else
    HIP_TRY(c, launch_residual(p.RP, 0, c->args, c->d_tilesB, (int)p.tilesB.size(), next_dir(c), c->stream));
  c->pending = false;
  return LQSGD_OK;
}

struct PacketLoc {
  uint8_t* mag; uint8_t* sgn; float* scale;
  int64_t n_el, groups, mag_len, sign_len;
  int bits;
};

int locate_packet(lqsgd_ctx* c, int32_t phase, int32_t layer, int32_t worker, PacketLoc* out) {
  if (phase != LQSGD_PHASE_P && phase != LQSGD_PHASE_Q) return fail(c, LQSGD_EINVAL, "phase must be LQSGD_PHASE_P or LQSGD_PHASE_Q");
  const LayerDesc* ld = nullptr;
  int rc = check_matrix_layer(c, layer, &ld);
  if (rc) return rc;
  if ((rc = check_worker(c, worker))) return rc;
  const int li = c->plan.kind_of[layer];
  const DevArgs& a = c->args;
  out->bits = phase ? a.bits_q : a.bits_p;
  if (out->bits == 0) return fail(c, LQSGD_EUNSUPPORTED, "quantisation is off for this phase: the packet is the fp32 factor");
  out->n_el = phase ? ld->nq_el : ld->np_el;
  out->groups = (out->n_el + kXGroup - 1) / kXGroup;
  out->mag_len = out->groups * out->bits;
  out->sign_len = out->groups;
  if (phase) {
    out->mag = a.magQ + (size_t)worker * a.magq_stride + ld->magq_off;
    out->sgn = a.sgnQ + (size_t)worker * a.sgnq_stride + ld->sgnq_off;
    out->scale = a.scaleQ + (size_t)worker * a.L + li;
  } else {
    out->mag = a.magP + (size_t)worker * a.magp_stride + ld->magp_off;
    out->sgn = a.sgnP + (size_t)worker * a.sgnp_stride + ld->sgnp_off;
    out->scale = a.scaleP + (size_t)worker * a.L + li;
  }
  return LQSGD_OK;
}

}  // namespace

// =============================================================================
extern "C" {

int lqsgd_plan_query(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers, lqsgd_plan_info* out) {
  if (!out) return fail(nullptr, LQSGD_EINVAL, "NULL output");
  Plan p;
  const int rc = p.build(cfg, layers, n_layers);
  if (rc) return fail(nullptr, rc, p.err);
  out->device_bytes = p.device_bytes;
  out->wire_bytes = p.wire_bytes;
  out->matrix_elements = p.matrix_elements;
  out->n_matrix = p.L;
  out->n_vector = p.V;
  out->rank_pad = p.RP;
  out->tiles[0] = (int32_t)p.tilesA.size();
  out->tiles[1] = (int32_t)(p.mfma ? p.tilesBM.size() : p.tilesB.size());
  out->tiles[2] = (int32_t)(p.mfma_a ? p.tilesA.size() : p.tilesB.size());
  out->residual_stride = p.m_stride;
  out->warm_q_floats = p.q_stride + kFactorSlack;
  return LQSGD_OK;
}

int64_t lqsgd_plan_tiles(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers, int32_t sweep,
                         int32_t* out, int64_t cap) {
  if (sweep < 0 || sweep > 3) return fail(nullptr, LQSGD_EINVAL, "sweep must be 0, 1, 2 or 3");
  Plan p;
  const int rc = p.build(cfg, layers, n_layers);
  if (rc) return fail(nullptr, rc, p.err);
  const bool bm = sweep == 1 && p.mfma;
  const bool as0 = sweep == 0 || (sweep >= 2 && p.mfma_a);     // items of sweep 0's kind
  const std::vector<Tile>& tl = sweep == 3 ? (p.mfma_a ? p.tilesAG : p.tilesG)
                                           : as0 ? p.tilesA : (bm ? p.tilesBM : p.tilesB);
  if (out) {
    const int64_t n = std::min<int64_t>(cap, (int64_t)tl.size());
    for (int64_t i = 0; i < n; ++i) {
      const Tile& t = tl[i];
      const int li = t.lw / p.W;
      const LayerDesc& d = p.layers[li];
      int32_t* o = out + 6 * i;
      o[0] = d.gidx;
      o[1] = t.lw - li * p.W;
      o[2] = t.row0;
      o[3] = t.nrows;
      if (as0) {
        o[4] = t.aux * d.segw;
        o[5] = std::min(d.cols, o[4] + d.segw) - o[4];
      } else {
        const int cw = bm ? kMfmaCols : kWave * d.vec;
        o[4] = t.aux * cw;
        o[5] = std::min(d.cols, o[4] + cw) - o[4];
      }
    }
  }
  return (int64_t)tl.size();
}

namespace {
// Fills c->args and uploads the tables of c->plan.  Device memory comes from hipMalloc or, when
// c->arena is set, from that block: then the residual slabs and the warm-start Q are not allocated
// (the caller's buffers are bound per call), and the one-launch Gram-Schmidt of tall factors, which
// needs a pinned status word and a table that starts from zero, is off (its forms of several launches run).
// On failure the caller releases c->allocs / c->status.
int setup_device(lqsgd_ctx* c, uint32_t flags) {
  int rc;
  const bool ext = c->arena != nullptr;
  c->eager = ext || (flags & LQSGD_FLAG_EAGER_RESIDUAL) != 0;
  HIP_TRY(c, hipGetDevice(&c->device));
  const Plan& p = c->plan;
  DevArgs& a = c->args;
  a.W = p.W; a.L = p.L; a.n_all = p.n_all; a.bits_p = p.cfg.bits_p; a.bits_q = p.cfg.bits_q;
  a.alpha = p.cfg.alpha;
  a.agg_first = p.agg_first ? 1 : 0; a.orth_shared = 0; a.update = 0; a.eta = 0.0f;
  a.g_bf16 = (flags & LQSGD_FLAG_BF16_GRADIENTS) ? 1 : 0;
  // The residual / M slabs are read and written once per sweep.  While they are about the size of
  // the memory-side cache (256 MB), plain loads and stores in sweep 0 are faster (ResNet-18 set,
  // 357 MB: a step takes 276 us; 284 us with non-temporal loads of E, 295 us with non-temporal
  // stores as well).  Far beyond it, the dirty lines that plain stores leave in that cache are
  // written back underneath the following reads, and streaming both ways wins (8192^2 x 16,
  // 4.3 GB: sweep 0 2.27 -> 2.04 - 2.14 ms).  Measured crossover: 0.55 - 0.7 GB.
  {
    const int64_t slab_bytes = 4 * (int64_t)p.W * p.m_stride;
    a.nt_store = slab_bytes >= ((int64_t)640 << 20) ? 1 : 0;
#ifdef LQSGD_TUNING     // a tuning build can force the choice and switch the alternating sweep direction off
    if (const char* f = std::getenv("LQSGD_NT_STORE")) {
      if (f[0] == '1') a.nt_store = 1;
      if (f[0] == '2') a.nt_store = 0;
    }
    if (const char* f = std::getenv("LQSGD_FLIP")) c->flip = (f[0] != '0');
#endif
  }
  a.qscale_p = (float)(((1 << p.cfg.bits_p) - 1) / std::log2(1.0 + (double)p.cfg.alpha));
  a.qscale_q = (float)(((1 << p.cfg.bits_q) - 1) / std::log2(1.0 + (double)p.cfg.alpha));
  a.m_stride = p.m_stride; a.p_stride = p.p_stride; a.q_stride = p.q_stride;
  a.ppart_stride = p.ppart_stride; a.qpart_stride = p.qpart_stride;
  a.magp_stride = p.magp_stride; a.sgnp_stride = p.sgnp_stride;
  a.magq_stride = p.magq_stride; a.sgnq_stride = p.sgnq_stride;
  const size_t W = (size_t)p.W;
  LayerDesc* d_layers = nullptr; VecDesc* d_vecs = nullptr;
  float *thrP = nullptr, *levP = nullptr, *thrQ = nullptr, *levQ = nullptr;
  std::vector<float> tP, lP, tQ, lQ;
  quantiser_tables(p.cfg.bits_p, (double)p.cfg.alpha, tP, lP);
  quantiser_tables(p.cfg.bits_q, (double)p.cfg.alpha, tQ, lQ);
#define TRY_(x) do { if ((rc = (x))) return rc; } while (0)
  // Loaders for ranks below their register pad fetch whole padded rows and may run up to 31 floats
  // past the last row of a factor: every factor buffer ends with this much readable slack.
  constexpr size_t kSlack = kFactorSlack;
  const size_t orth_cells = 2 * W * (size_t)std::max(p.L, 1) * ((p.max_rows + 255) / 256) * p.RP;
  a.E = nullptr; a.Qbar = nullptr; a.orth_table = nullptr; a.status = nullptr;
  a.chol_table = nullptr; a.chol_part = nullptr; a.chol_redo = nullptr;
  if (!ext) TRY_(dev_alloc(c, &a.E, W * p.m_stride, true));
  TRY_(dev_alloc(c, &a.Ppart, W * p.ppart_stride + kSlack, true));
  TRY_(dev_alloc(c, &a.Ppre, W * p.p_stride + kSlack, true));
  TRY_(dev_alloc(c, &a.Porth, W * p.p_stride + kSlack, true));
  TRY_(dev_alloc(c, &a.orth_part, orth_cells, true));
  {
    // Tall factors at rank pads >= 16 exchange whole Gram matrices instead of single columns
    // (launch_orth decides per call; the same lower height limit as there).  A caller-provided block
    // and factors of more than 64 slices get the buffers of the form of three launches only, which
    // gives the same bits.
    const size_t nslice = (size_t)(p.max_rows + 255) / 256, pairs = W * (size_t)std::max(p.L, 1);
    const size_t ne = (size_t)chol_entries(p.RP);
    if (ne && nslice >= 8 && pairs * (nslice + 1) * ne * 12 <= ((size_t)1 << 30)) {
      if (!ext && nslice <= 64) TRY_(dev_alloc(c, &a.chol_table, pairs * (nslice + 1) * ne, true));   // the one-launch form's limit
      TRY_(dev_alloc(c, &a.chol_part, pairs * nslice * ne, true));
      TRY_(dev_alloc(c, &a.chol_redo, pairs, true));
    }
  }
  if (!ext) {
    TRY_(dev_alloc(c, &a.orth_table, orth_cells, true));
    void* hp = nullptr;
    hipError_t e = hipHostMalloc(&hp, sizeof(int), hipHostMallocDefault);
    if (e != hipSuccess) { fail_hip(c, e, "hipHostMalloc"); return LQSGD_ENOMEM; }
    c->status = static_cast<int*>(hp);
    *c->status = 0;
    a.status = c->status;
  }
  TRY_(dev_alloc(c, &a.Pbar, (size_t)p.p_stride + kSlack, true));
  TRY_(dev_alloc(c, &a.Qpart, W * p.qpart_stride + kSlack, true));
  TRY_(dev_alloc(c, &a.Qw, W * p.q_stride + kSlack, true));
  if (!ext) TRY_(dev_alloc(c, &a.Qbar, (size_t)p.q_stride + kSlack, true));
  a.Ppad = nullptr; a.Qpad = nullptr;
  if (p.padded) {
    TRY_(dev_alloc(c, &a.Ppad, (size_t)p.ppad_total + kSlack, true));
    TRY_(dev_alloc(c, &a.Qpad, (size_t)p.qpad_total + kSlack, true));
  }
  TRY_(dev_alloc(c, &a.magP, W * p.magp_stride, true));
  TRY_(dev_alloc(c, &a.sgnP, W * p.sgnp_stride, true));
  TRY_(dev_alloc(c, &a.scaleP, W * (size_t)std::max(p.L, 1), true));
  TRY_(dev_alloc(c, &a.magQ, W * p.magq_stride, true));
  TRY_(dev_alloc(c, &a.sgnQ, W * p.sgnq_stride, true));
  TRY_(dev_alloc(c, &a.scaleQ, W * (size_t)std::max(p.L, 1), true));
  TRY_(dev_alloc(c, &a.vmean, (size_t)p.v_total, true));
  TRY_(dev_alloc(c, &c->d_grads, W * p.n_all, true));
  TRY_(dev_alloc(c, &c->d_ghat, (size_t)p.n_all, true));
  // In a caller-provided block everything above is cleared here, by a kernel, before the tables
  // below are copied in (the block keeps whatever its last user left).
  if (ext) HIP_TRY(c, launch_fill_zero(c->arena, c->arena_used, c->stream));
  if (ext) HIP_TRY(c, hipStreamSynchronize(c->stream));
  TRY_(dev_upload(c, &d_layers, p.layers));
  TRY_(dev_upload(c, &d_vecs, p.vecs));
  TRY_(dev_upload(c, &thrP, tP)); TRY_(dev_upload(c, &levP, lP));
  TRY_(dev_upload(c, &thrQ, tQ)); TRY_(dev_upload(c, &levQ, lQ));
  TRY_(dev_upload(c, &c->d_tilesA, p.tilesA));
  TRY_(dev_upload(c, &c->d_tilesB, p.tilesB));
  TRY_(dev_upload(c, &c->d_tilesG, p.tilesG));
  TRY_(dev_upload(c, &c->d_tilesBM, p.tilesBM));
  TRY_(dev_upload(c, &c->d_tilesAG, p.tilesAG));
  TRY_(dev_upload(c, &c->d_tilesXP, p.tilesXP));
  TRY_(dev_upload(c, &c->d_tilesXQ, p.tilesXQ));
  TRY_(dev_upload(c, &c->d_tilesRQ, p.tilesRQ));
  TRY_(dev_upload(c, &c->d_tilesRP, p.tilesRP));
  TRY_(dev_upload(c, &c->d_tilesV, p.tilesV));
#undef TRY_
  a.layers = d_layers; a.vecs = d_vecs;
  a.thrP = thrP; a.levP = levP; a.thrQ = thrQ; a.levQ = levQ;
  a.grads = c->d_grads; a.ghat = nullptr;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return LQSGD_OK;
}
}  // namespace

int lqsgd_create(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers, void* hip_stream,
                 lqsgd_ctx** out) {
  if (!out) return fail(nullptr, LQSGD_EINVAL, "NULL output pointer");
  *out = nullptr;
  lqsgd_ctx* c = new (std::nothrow) lqsgd_ctx();
  if (!c) return fail(nullptr, LQSGD_ENOMEM, "out of host memory");
  int rc = c->plan.build(cfg, layers, n_layers);
  if (rc) {
    g_create_error = c->plan.err;
    delete c;
    return rc;
  }
  c->stream = static_cast<hipStream_t>(hip_stream);
  // The bound of the device-side waits of the one-launch Gram-Schmidt can be shortened for a test
  // of the expiry path (read once, here; nothing else in the library reads the environment).
  if (const char* e = std::getenv("LQSGD_TABLE_POLLS")) {
    const long v = std::strtol(e, nullptr, 10);
    if (v >= 1) c->coop.max_polls = (unsigned)v;
  }
  if ((rc = setup_device(c, cfg->flags))) {
    g_create_error = c->err;
    for (void* p : c->allocs) (void)hipFree(p);
    if (c->status) (void)hipHostFree(c->status);
    delete c;
    return rc;
  }
  *out = c;
  return LQSGD_OK;
}

int lqsgd_destroy(lqsgd_ctx* c) {
  if (!c) return LQSGD_OK;
  (void)hipStreamSynchronize(c->stream);
  for (EventPair& e : c->events) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->status) (void)hipHostFree(c->status);
  (void)hipGetLastError();
  delete c;
  return LQSGD_OK;
}

int lqsgd_synchronize(lqsgd_ctx* c) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  if (int rcs = sync_stream(c)) return rcs;
  return LQSGD_OK;
}

const char* lqsgd_last_error(const lqsgd_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

int lqsgd_set_q(lqsgd_ctx* c, int32_t layer, const float* host_q) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  if (!host_q) return fail(c, LQSGD_EINVAL, "NULL host_q");
  return lqsgd_set_state(c, layer, 0, nullptr, host_q);
}

int lqsgd_get_state(lqsgd_ctx* c, int32_t layer, int32_t worker, float* host_e, float* host_q) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  const LayerDesc* ld = nullptr;
  int rc = check_matrix_layer(c, layer, &ld);
  if (rc) return rc;
  if ((rc = check_worker(c, worker))) return rc;
  if (host_e && (rc = materialise(c))) return rc;
  if (int rcs = sync_stream(c)) return rcs;
  if (host_e)
    HIP_TRY(c, hipMemcpy(host_e, c->args.E + (size_t)worker * c->args.m_stride + ld->m_off,
                         (size_t)ld->rows * ld->cols * sizeof(float), hipMemcpyDeviceToHost));
  if (host_q)
    HIP_TRY(c, hipMemcpy(host_q, c->args.Qbar + ld->q_off, (size_t)ld->nq_el * sizeof(float), hipMemcpyDeviceToHost));
  return LQSGD_OK;
}

int lqsgd_set_state(lqsgd_ctx* c, int32_t layer, int32_t worker, const float* host_e, const float* host_q) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  const LayerDesc* ld = nullptr;
  int rc = check_matrix_layer(c, layer, &ld);
  if (rc) return rc;
  if ((rc = check_worker(c, worker))) return rc;
  if ((rc = materialise(c))) return rc;      // a deferred update depends on the old E buffer and the old Q
  if (int rcs = sync_stream(c)) return rcs;
  if (host_e)
    HIP_TRY(c, hipMemcpy(c->args.E + (size_t)worker * c->args.m_stride + ld->m_off, host_e,
                         (size_t)ld->rows * ld->cols * sizeof(float), hipMemcpyHostToDevice));
  if (host_q) {
    HIP_TRY(c, hipMemcpy(c->args.Qbar + ld->q_off, host_q, (size_t)ld->nq_el * sizeof(float), hipMemcpyHostToDevice));
    c->qpad_stale = true;
  }
  return LQSGD_OK;
}

int lqsgd_compress(lqsgd_ctx* c, int32_t phase, const float* const* grads) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  int rc;
  if (phase == LQSGD_PHASE_P) {
    if (c->state != kIdle) return fail(c, LQSGD_ESTATE, "compress(P) must start an iteration");
    if (!grads) return fail(c, LQSGD_EINVAL, "NULL gradient list");
    if ((rc = bind_grads(c, grads))) return rc;
    if ((rc = run_sweep0(c))) return rc;
    if ((rc = run_exchange(c, kQuantOnly, 0))) return rc;
    c->state = kPCompressed;
    return LQSGD_OK;
  }
  if (phase == LQSGD_PHASE_Q) {
    if (c->state != kPDone) return fail(c, LQSGD_ESTATE, "compress(Q) must follow decompress(P)");
    if ((rc = run_sweep1(c, false))) return rc;
    if ((rc = run_exchange(c, kQuantOnly, 1))) return rc;
    c->state = kQCompressed;
    return LQSGD_OK;
  }
  return fail(c, LQSGD_EINVAL, "phase must be LQSGD_PHASE_P or LQSGD_PHASE_Q");
}

int lqsgd_decompress(lqsgd_ctx* c, int32_t phase) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  int rc;
  if (phase == LQSGD_PHASE_P) {
    if (c->state != kPCompressed) return fail(c, LQSGD_ESTATE, "decompress(P) must follow compress(P)");
    if ((rc = run_exchange(c, kMeanOnly, 0))) return rc;
    c->state = kPDone;
    return LQSGD_OK;
  }
  if (phase == LQSGD_PHASE_Q) {
    if (c->state != kQCompressed) return fail(c, LQSGD_ESTATE, "decompress(Q) must follow compress(Q)");
    if ((rc = run_exchange(c, kMeanOnly, 1))) return rc;
    c->args.ghat = nullptr;
    if ((rc = run_sweep2(c, false))) return rc;
    c->state = kIdle;
    return LQSGD_OK;
  }
  return fail(c, LQSGD_EINVAL, "phase must be LQSGD_PHASE_P or LQSGD_PHASE_Q");
}

namespace {
int step_impl(lqsgd_ctx* c, const float* const* grads, float* const* ghat);
}

int lqsgd_step(lqsgd_ctx* c, const float* const* grads, float* const* ghat) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  return step_impl(c, grads, ghat);
}

int lqsgd_step_update(lqsgd_ctx* c, const float* const* grads, float* const* params, float eta) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  if (!params) return fail(c, LQSGD_EINVAL, "NULL parameter list");
  if (!std::isfinite(eta)) return fail(c, LQSGD_EINVAL, "eta must be finite");
  c->args.update = 1;
  c->args.eta = eta;
  const int rc = step_impl(c, grads, params);
  c->args.update = 0;
  c->args.eta = 0.0f;
  return rc;
}

namespace {
int step_impl(lqsgd_ctx* c, const float* const* grads, float* const* ghat) {
  if (c->state != kIdle) return fail(c, LQSGD_ESTATE, "a staged iteration is in progress");
  if (!grads) return fail(c, LQSGD_EINVAL, "NULL gradient list");
  int rc;
  if ((rc = bind_grads(c, grads))) return rc;
  if ((rc = bind_ghat(c, ghat))) return rc;
  if (ghat && !c->alias_checked) {   // both tables are the host copies just compared equal or re-bound
    const size_t n = (size_t)c->plan.W * c->plan.n_all;
    for (int i = 0; i < c->plan.n_all; ++i)
      if (ghat[i])
        for (size_t j = 0; j < n; ++j)
          if (grads[j] == ghat[i]) return fail(c, LQSGD_EINVAL, "an output pointer aliases a gradient");
    c->alias_checked = true;
  }
  if ((rc = run_sweep0(c))) return rc;
  if ((rc = run_exchange(c, kFused, 0))) return rc;
  if ((rc = run_sweep1(c, true))) return rc;
  if ((rc = run_exchange(c, kFused, 1))) return rc;
  if ((rc = run_sweep2(c, ghat != nullptr))) return rc;
  return LQSGD_OK;
}
}  // namespace

int lqsgd_get_packet_raw(lqsgd_ctx* c, int32_t phase, int32_t layer, int32_t worker, uint8_t* mag_plane,
                         int64_t* mag_len, uint8_t* sign_plane, int64_t* sign_len) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  PacketLoc loc{};
  int rc = locate_packet(c, phase, layer, worker, &loc);
  if (rc) return rc;
  if (mag_len) *mag_len = loc.mag_len;
  if (sign_len) *sign_len = loc.sign_len;
  if (!mag_plane && !sign_plane) return LQSGD_OK;
  if (int rcs = sync_stream(c)) return rcs;
  if (mag_plane) HIP_TRY(c, hipMemcpy(mag_plane, loc.mag, (size_t)loc.mag_len, hipMemcpyDeviceToHost));
  if (sign_plane) HIP_TRY(c, hipMemcpy(sign_plane, loc.sgn, (size_t)loc.sign_len, hipMemcpyDeviceToHost));
  return LQSGD_OK;
}

int lqsgd_packet_device(lqsgd_ctx* c, int32_t phase, int32_t layer, int32_t worker, uint8_t** mag_plane,
                        int64_t* mag_len, uint8_t** sign_plane, int64_t* sign_len, float** scale) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  PacketLoc loc{};
  int rc = locate_packet(c, phase, layer, worker, &loc);
  if (rc) return rc;
  if (mag_plane) *mag_plane = loc.mag;
  if (mag_len) *mag_len = loc.mag_len;
  if (sign_plane) *sign_plane = loc.sgn;
  if (sign_len) *sign_len = loc.sign_len;
  if (scale) *scale = loc.scale;
  return LQSGD_OK;
}

int lqsgd_get_packet(lqsgd_ctx* c, int32_t phase, int32_t layer, int32_t worker, uint8_t* mag_codes,
                     uint8_t* sign_bits, float* scale) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  PacketLoc loc{};
  int rc = locate_packet(c, phase, layer, worker, &loc);
  if (rc) return rc;
  if (int rcs = sync_stream(c)) return rcs;
  if (scale) HIP_TRY(c, hipMemcpy(scale, loc.scale, sizeof(float), hipMemcpyDeviceToHost));
  if (mag_codes) {
    std::vector<uint8_t> raw((size_t)loc.mag_len);
    HIP_TRY(c, hipMemcpy(raw.data(), loc.mag, raw.size(), hipMemcpyDeviceToHost));
    const unsigned mask = (1u << loc.bits) - 1u;
    for (int64_t e = 0; e < loc.n_el; ++e) {
      const int64_t bit = e * loc.bits;
      unsigned v = raw[(size_t)(bit >> 3)] >> (bit & 7);
      if ((bit & 7) + loc.bits > 8) v |= (unsigned)raw[(size_t)(bit >> 3) + 1] << (8 - (bit & 7));
      mag_codes[e] = (uint8_t)(v & mask);
    }
  }
  if (sign_bits) {
    std::vector<uint8_t> raw((size_t)loc.sign_len);
    HIP_TRY(c, hipMemcpy(raw.data(), loc.sgn, raw.size(), hipMemcpyDeviceToHost));
    for (int64_t e = 0; e < loc.n_el; ++e) sign_bits[e] = (raw[(size_t)(e >> 3)] >> (e & 7)) & 1u;
  }
  return LQSGD_OK;
}

int lqsgd_set_packet(lqsgd_ctx* c, int32_t phase, int32_t layer, int32_t worker, const uint8_t* mag_codes,
                     const uint8_t* sign_bits, float scale) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  if (!mag_codes || !sign_bits) return fail(c, LQSGD_EINVAL, "NULL code array");
  PacketLoc loc{};
  int rc = locate_packet(c, phase, layer, worker, &loc);
  if (rc) return rc;
  const unsigned mask = (1u << loc.bits) - 1u;
  std::vector<uint8_t> mag((size_t)loc.mag_len, 0), sgn((size_t)loc.sign_len, 0);
  for (int64_t e = 0; e < loc.n_el; ++e) {
    if (mag_codes[e] > mask) return fail(c, LQSGD_EINVAL, "magnitude code exceeds 2^b - 1");
    const int64_t bit = e * loc.bits;
    const unsigned v = (unsigned)mag_codes[e] << (bit & 7);
    mag[(size_t)(bit >> 3)] |= (uint8_t)v;
    if ((bit & 7) + loc.bits > 8) mag[(size_t)(bit >> 3) + 1] |= (uint8_t)(v >> 8);
    if (sign_bits[e] & 1u) sgn[(size_t)(e >> 3)] |= (uint8_t)(1u << (e & 7));
  }
  if (int rcs = sync_stream(c)) return rcs;
  HIP_TRY(c, hipMemcpy(loc.mag, mag.data(), mag.size(), hipMemcpyHostToDevice));
  HIP_TRY(c, hipMemcpy(loc.sgn, sgn.data(), sgn.size(), hipMemcpyHostToDevice));
  HIP_TRY(c, hipMemcpy(loc.scale, &scale, sizeof(float), hipMemcpyHostToDevice));
  return LQSGD_OK;
}

int lqsgd_get_factor(lqsgd_ctx* c, int32_t which, int32_t layer, int32_t worker, float* host) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  if (!host) return fail(c, LQSGD_EINVAL, "NULL host buffer");
  const DevArgs& a = c->args;
  if (which == LQSGD_FACTOR_VMEAN) {
    if (layer < 0 || layer >= c->plan.n_all) return fail(c, LQSGD_ESHAPE, "layer index out of range");
    const int k = c->plan.kind_of[layer];
    if (k >= 0) return fail(c, LQSGD_ESHAPE, "layer is not a VECTOR layer");
    const VecDesc& vd = c->plan.vecs[-k - 1];
    if (int rcs = sync_stream(c)) return rcs;
    HIP_TRY(c, hipMemcpy(host, a.vmean + vd.off, (size_t)vd.len * sizeof(float), hipMemcpyDeviceToHost));
    return LQSGD_OK;
  }
  const LayerDesc* ld = nullptr;
  int rc = check_matrix_layer(c, layer, &ld);
  if (rc) return rc;
  const float* src = nullptr;
  size_t n = 0;
  const bool per_worker = which == LQSGD_FACTOR_P_PRE || which == LQSGD_FACTOR_P_ORTH || which == LQSGD_FACTOR_Q_W;
  if (per_worker && (rc = check_worker(c, worker))) return rc;
  if (which == LQSGD_FACTOR_P_ORTH && c->plan.agg_first)
    return fail(c, LQSGD_EINVAL, "no per-worker Gram-Schmidt output in the aggregate-first order");
  if (which == LQSGD_FACTOR_P_MEAN && !c->plan.agg_first)
    return fail(c, LQSGD_EINVAL, "LQSGD_FACTOR_P_MEAN exists in the aggregate-first order only");
  switch (which) {
    case LQSGD_FACTOR_P_MEAN: src = a.Porth + ld->p_off; n = ld->np_el; break;
    case LQSGD_FACTOR_P_PRE: src = a.Ppre + (size_t)worker * a.p_stride + ld->p_off; n = ld->np_el; break;
    case LQSGD_FACTOR_P_ORTH: src = a.Porth + (size_t)worker * a.p_stride + ld->p_off; n = ld->np_el; break;
    case LQSGD_FACTOR_P_BAR: src = a.Pbar + ld->p_off; n = ld->np_el; break;
    case LQSGD_FACTOR_Q_W: src = a.Qw + (size_t)worker * a.q_stride + ld->q_off; n = ld->nq_el; break;
    case LQSGD_FACTOR_Q_BAR: src = a.Qbar + ld->q_off; n = ld->nq_el; break;
    default: return fail(c, LQSGD_EINVAL, "unknown factor id");
  }
  if (int rcs = sync_stream(c)) return rcs;
  HIP_TRY(c, hipMemcpy(host, src, n * sizeof(float), hipMemcpyDeviceToHost));
  return LQSGD_OK;
}

int lqsgd_set_factor(lqsgd_ctx* c, int32_t which, int32_t layer, const float* host) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  if (!host) return fail(c, LQSGD_EINVAL, "NULL host buffer");
  const LayerDesc* ld = nullptr;
  int rc = check_matrix_layer(c, layer, &ld);
  if (rc) return rc;
  float* dst = nullptr;
  size_t n = 0;
  if (which == LQSGD_FACTOR_P_BAR) { dst = c->args.Pbar + ld->p_off; n = ld->np_el; }
  else if (which == LQSGD_FACTOR_Q_BAR) { dst = c->args.Qbar + ld->q_off; n = ld->nq_el; }
  else return fail(c, LQSGD_EINVAL, "only P-bar and Q-bar can be set");
  if ((rc = materialise(c))) return rc;      // a deferred update is defined by the old factors
  if (int rcs = sync_stream(c)) return rcs;
  HIP_TRY(c, hipMemcpy(dst, host, n * sizeof(float), hipMemcpyHostToDevice));
  (which == LQSGD_FACTOR_P_BAR ? c->ppad_stale : c->qpad_stale) = true;
  return LQSGD_OK;
}

int64_t lqsgd_wire_bytes(const lqsgd_ctx* c) { return c ? c->plan.wire_bytes : (int64_t)LQSGD_EINVAL; }

int lqsgd_timing_enable(lqsgd_ctx* c, int32_t on) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  if (int rcs = sync_stream(c)) return rcs;
  c->timing = on != 0;
  c->events_used = 0;
  return LQSGD_OK;
}

int lqsgd_timing_read(lqsgd_ctx* c, double* total_ms, int64_t* launches) {
  if (!c) return fail(nullptr, LQSGD_EINVAL, "NULL context");
  if (!total_ms || !launches) return fail(c, LQSGD_EINVAL, "NULL output array");
  if (int rcs = sync_stream(c)) return rcs;
  for (int k = 0; k < LQSGD_KERNEL_COUNT; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
  for (size_t i = 0; i < c->events_used; ++i) {
    float ms = 0.0f;
    HIP_TRY(c, hipEventElapsedTime(&ms, c->events[i].a, c->events[i].b));
    total_ms[c->events[i].kernel] += ms;
    launches[c->events[i].kernel] += 1;
  }
  return LQSGD_OK;
}

const char* lqsgd_launched_kernel(const lqsgd_ctx* c, int32_t kernel) {
  if (!c || kernel < 0 || kernel >= LQSGD_KERNEL_COUNT) return "";
  return c->launched[kernel].c_str();
}

const char* lqsgd_kernel_name(int32_t kernel) {
  switch (kernel) {
    case LQSGD_KERNEL_ADD_PROJECT: return "sweep0_add_project";
    case LQSGD_KERNEL_ORTH: return "gram_schmidt";
    case LQSGD_KERNEL_EXCHANGE_P: return "exchange_p";
    case LQSGD_KERNEL_BACK_PROJECT: return "sweep1_back_project";
    case LQSGD_KERNEL_REDUCE_Q: return "reduce_q";
    case LQSGD_KERNEL_EXCHANGE_Q: return "exchange_q";
    case LQSGD_KERNEL_RESIDUAL: return "sweep2_residual_ghat";
    case LQSGD_KERNEL_REDUCE_P: return "reduce_p";
    default: return "";
  }
}

// ---- the entry point that allocates nothing ----------------------------------------------------
namespace {
// One slot per device: the host-side plan of the last configuration run there, whose device tables
// still lie in that device's static scratch block.
struct StaticSlot {
  lqsgd_ctx* ctx = nullptr;
  lqsgd_config cfg{};
  std::vector<lqsgd_layer> layers;
};
constexpr int kMaxDevices = 64;
StaticSlot g_static[kMaxDevices];
std::mutex g_static_mu;

bool same_config(const StaticSlot& s, const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n, hipStream_t stream) {
  if (!s.ctx || s.ctx->stream != stream || (int32_t)s.layers.size() != n) return false;
  if (s.cfg.rank != cfg->rank || s.cfg.bits_p != cfg->bits_p || s.cfg.bits_q != cfg->bits_q ||
      s.cfg.workers != cfg->workers || s.cfg.alpha != cfg->alpha || s.cfg.flags != cfg->flags)
    return false;
  for (int32_t i = 0; i < n; ++i)
    if (s.layers[i].rows != layers[i].rows || s.layers[i].cols != layers[i].cols || s.layers[i].flags != layers[i].flags)
      return false;
  return true;
}
}  // namespace

int lqsgd_step_static(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers, void* hip_stream,
                      const float* const* grads, float* residual, float* warm_q, float* const* ghat) {
  if (!cfg || !layers) return fail(nullptr, LQSGD_EINVAL, "NULL config or layer list");
  if (!grads) return fail(nullptr, LQSGD_EINVAL, "NULL gradient list");
  std::lock_guard<std::mutex> lock(g_static_mu);
  int dev = 0;
  {
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(nullptr, e, "hipGetDevice");
  }
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, LQSGD_EUNSUPPORTED, "device index beyond the table of static scratch blocks");
  void* block = nullptr;
  size_t block_bytes = 0;
  {
    hipError_t e = static_scratch(dev, &block, &block_bytes);
    if (e != hipSuccess) return fail_hip(nullptr, e, "hipGetSymbolAddress(scratch)");
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  StaticSlot& slot = g_static[dev];
  if (!same_config(slot, cfg, layers, n_layers, stream)) {
    // A new configuration lays the block out anew: whatever the last one enqueued must have finished.
    if (slot.ctx) {
      (void)hipStreamSynchronize(slot.ctx->stream);
      (void)hipGetLastError();
      delete slot.ctx;
      slot.ctx = nullptr;
    }
    lqsgd_ctx* c = new (std::nothrow) lqsgd_ctx();
    if (!c) return fail(nullptr, LQSGD_ENOMEM, "out of host memory");
    int rc = c->plan.build(cfg, layers, n_layers);
    if (rc) {
      g_create_error = c->plan.err;
      delete c;
      return rc;
    }
    c->stream = stream;
    c->arena = static_cast<unsigned char*>(block);
    c->arena_cap = block_bytes;
    if ((rc = setup_device(c, cfg->flags))) {
      g_create_error = c->err;
      delete c;
      return rc;
    }
    slot.ctx = c;
    slot.cfg = *cfg;
    slot.layers.assign(layers, layers + n_layers);
  }
  lqsgd_ctx* c = slot.ctx;
  const bool has_matrix = c->plan.L > 0;
  if (has_matrix && (!residual || !warm_q)) { g_create_error = "NULL residual or warm-start buffer"; return LQSGD_EINVAL; }
  if ((reinterpret_cast<uintptr_t>(residual) | reinterpret_cast<uintptr_t>(warm_q)) & 15u) {
    g_create_error = "residual / warm-start buffer not 16-byte aligned";
    return LQSGD_EINVAL;
  }
  c->args.E = residual;
  c->args.Qbar = warm_q;
  c->pending = false;                        // the caller's buffer holds E, and holds E again on return
  c->ppad_stale = c->qpad_stale = true;      // the warm-start Q is the caller's: any padded copy is out of date
  c->state = kIdle;
  const int rc = step_impl(c, grads, ghat);
  if (rc) g_create_error = c->err;
  return rc;
}

}  // extern "C"
