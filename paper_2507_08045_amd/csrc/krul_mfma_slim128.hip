// Instantiations of the similarity kernel: the slim tile shapes at head_dim 128 (one translation unit per
// group of shapes, so that they compile side by side).  Tile shapes must match make_plan().
#include "krul_mfma_kernel.h"

namespace krul {

hipError_t launch_sim_mfma_slim128(const SimParams &p, int n_workgroups, hipStream_t st)
{
    switch (p.lay.variant) {   //                      D  WR WK KBW NC
    case kMfmaSlim:
        return launch_cfg<Cfg<128, 1, 8, 1, 2>>(p, n_workgroups, st);   //  32 x 512, 8 waves, ring 2 x 256 keys
    case kMfmaSlimDeep:
        return launch_cfg<Cfg<128, 1, 4, 1, 4>>(p, n_workgroups, st);   //  32 x 512, 4 waves, ring 4 x 128 keys: three chunks in flight
    case kMfmaSlimShort:
        return launch_cfg<Cfg<128, 1, 4, 1, 2>>(p, n_workgroups, st);   //  32 x 256, 4 waves, ring 2 x 128 keys: two workgroups per CU
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace krul
