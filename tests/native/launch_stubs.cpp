// Stand-ins for the kernel launchers, for the host-only sanitizer build of the library's host side
// (tests/test_host_sanitizers.py).  Host-only plans (device = -1) never reach a launch, so every stub
// reports failure if it is called after all.
#include "bwd.h"
#include "common.h"
#include "logprob.h"

namespace pa {
int launch_pass_bf16(const PassArgs&, void*) { return 1; }
int launch_pass_f32(const PassArgs&, void*) { return 1; }
int launch_vt_images(const VtArgs&, void*) { return 1; }
int launch_merge(const MergeArgs&, void*) { return 1; }
int launch_merge_n(const MergeNArgs&, void*) { return 1; }
int launch_lse_export(const float*, float*, int64_t, int32_t, void*) { return 1; }
int launch_bwd_prep(const BwdPrepArgs&, void*) { return 1; }
int launch_bwd_dq_bf16(const BwdDqArgs&, void*) { return 1; }
int launch_bwd_dkv_bf16(const BwdDkvArgs&, void*) { return 1; }
int launch_bwd_dq_f32(const BwdF32Args&, void*) { return 1; }
int launch_bwd_dkv_f32(const BwdF32Args&, void*) { return 1; }
int launch_logprob(const LogprobArgs&, void*) { return 1; }
int launch_group_advantages(const float*, float*, int, int, void*) { return 1; }
}  // namespace pa
