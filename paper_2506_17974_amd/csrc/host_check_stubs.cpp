// Stand-ins for the kernel launchers, for the host-only sanitizer build: the planner and the
// argument checking of the C ABI are linked without any device code.  Nothing here is part of
// the library; every launcher reports that it cannot run.
#include "lqsgd_kernels.h"

namespace lqsgd {

const char* last_launched_kernel() { return ""; }
hipError_t launch_add_project(int, const DevArgs&, const Tile*, int, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_orth(int, int, int, const DevArgs&, CoopState*, hipStream_t) { return hipErrorNotSupported; }
int chol_entries(int) { return 0; }
hipError_t launch_exchange(int, int, const DevArgs&, const XTile*, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_back_project(int, const DevArgs&, const Tile*, int, const VTile*, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_back_project_mfma(int, const DevArgs&, const Tile*, int, const VTile*, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_reduce_q(int, const DevArgs&, const RTile*, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_residual(int, int, const DevArgs&, const Tile*, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_pad_factor(int, int, const DevArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_mfma_sweep(int, int, int, const DevArgs&, const Tile*, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t static_scratch(int, void**, size_t*) { return hipErrorNotSupported; }
hipError_t launch_fill_zero(void*, size_t, hipStream_t) { return hipErrorNotSupported; }

}  // namespace lqsgd
