// Launchers of the kernel interface without kernels: the sanitizer driver never launches anything, it only needs the
// geometry these return for dry runs.
#include "../../paper_2304_11745_amd/csrc/kernels.h"
namespace gacer {
thread_local const LaunchTimer *launch_timer = nullptr;
static LaunchInfo geometry(const char *name, int phases)
{
    LaunchInfo li;
    li.workgroups = 1; li.threads = 256; li.lds_bytes = 0; li.wg_per_cu = 8; li.kernel = name; li.phases = phases;
    return li;
}
LaunchInfo launch_igemm(const GemmArgs &a, hipStream_t, bool, int phase) { return geometry(phase == 2 ? "splitk_finish" : "igemm", a.ksplit > 1 ? 2 : 1); }
LaunchInfo launch_dwconv(const StreamArgs &, hipStream_t, bool) { return geometry("dwconv", 1); }
LaunchInfo launch_maxpool(const StreamArgs &, hipStream_t, bool) { return geometry("maxpool", 1); }
LaunchInfo launch_gavgpool(const StreamArgs &, hipStream_t, bool) { return geometry("gavgpool", 1); }
LaunchInfo launch_eltwise(const StreamArgs &, hipStream_t, bool) { return geometry("eltwise", 1); }
LaunchInfo launch_concat(const StreamArgs &, hipStream_t, bool) { return geometry("concat", 1); }
LaunchInfo launch_layernorm(const StreamArgs &, hipStream_t, bool) { return geometry("layernorm", 1); }
LaunchInfo launch_softmax(const StreamArgs &, hipStream_t, bool) { return geometry("softmax", 1); }
void launch_spin(hipStream_t, unsigned long long) {}
}  // namespace gacer
