// Host-only build of the library for sanitizer runs: every kernel launcher is replaced by a stub that
// reports LL_ERR_DEVICE, so that the F2 algebra, the planners, the gather chooser and the argument
// checks of the C ABI can run under AddressSanitizer / UndefinedBehaviorSanitizer on a machine
// without a GPU (tests/test_host_sanitizers.py).
#include "../../paper_2505_23819_amd/csrc/kernels.hpp"
#include "../../paper_2505_23819_amd/csrc/layout.hpp"

namespace ll {
ll_status launch_gather_general(const GatherGenArgs &, int, int, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
ll_status launch_gather_phased(const GatherGenArgs &, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
ll_status launch_gather_global(const GatherGenArgs &, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
ll_status launch_lds_elem(const LdsElemArgs &, int, int, int, int, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
ll_status launch_vec(const VecArgs &, int, int, int, int, int, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
ll_status launch_lds_tr(const LdsElemArgs &, int, int, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
ll_status launch_pull(const PullArgs &, int, int, int, int, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
ll_status launch_gather(const GatherArgs &, int, int, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
ll_status launch_copy(const void *, void *, long long, int, void *) { return fail(LL_ERR_DEVICE, "stub: no device code in this build"); }
}  // namespace ll
