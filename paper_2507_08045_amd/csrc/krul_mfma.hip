// Dispatch of the 16-bit matrix-core similarity kernel (krul_mfma_kernel.h) over its tile shapes; the
// shapes are instantiated in krul_mfma_<shape><head_dim>.hip.
#include "krul_common.h"

namespace krul {

hipError_t launch_sim_mfma_wide128(const SimParams &p, int n_workgroups, hipStream_t st);
hipError_t launch_sim_mfma_wide64(const SimParams &p, int n_workgroups, hipStream_t st);
hipError_t launch_sim_mfma_mid128(const SimParams &p, int n_workgroups, hipStream_t st);
hipError_t launch_sim_mfma_mid64(const SimParams &p, int n_workgroups, hipStream_t st);
hipError_t launch_sim_mfma_slim128(const SimParams &p, int n_workgroups, hipStream_t st);
hipError_t launch_sim_mfma_slim64(const SimParams &p, int n_workgroups, hipStream_t st);

hipError_t launch_sim_mfma(const SimParams &p, int n_workgroups, hipStream_t st)
{
    const bool d128 = p.d > 64;   // (head sizes below the kernel's ride in zero-padded LDS rows)
    switch (p.lay.variant) {
    case kMfmaBig:
        return launch_sim_mfma_big(p, n_workgroups, st);
    case kMfmaWide:
    case kMfmaWideShort:
        return d128 ? launch_sim_mfma_wide128(p, n_workgroups, st) : launch_sim_mfma_wide64(p, n_workgroups, st);
    case kMfmaMid:
    case kMfmaMidShort:
        return d128 ? launch_sim_mfma_mid128(p, n_workgroups, st) : launch_sim_mfma_mid64(p, n_workgroups, st);
    case kMfmaSlim:
    case kMfmaSlimDeep:
    case kMfmaSlimShort:
        return d128 ? launch_sim_mfma_slim128(p, n_workgroups, st) : launch_sim_mfma_slim64(p, n_workgroups, st);
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace krul
