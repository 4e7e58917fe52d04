// Instantiations of the similarity kernel: the mid tile shapes at head_dim 128 (one translation unit per
// group of shapes, so that they compile side by side).  Tile shapes must match make_plan().
#include "krul_mfma_kernel.h"

namespace krul {

hipError_t launch_sim_mfma_mid128(const SimParams &p, int n_workgroups, hipStream_t st)
{
    switch (p.lay.variant) {   //                      D  WR WK KBW NC
    case kMfmaMid:
        return launch_cfg<Cfg<128, 2, 4, 1, 4>>(p, n_workgroups, st);   //  64 x 512, 8 waves, ring 4 x 128 keys
    case kMfmaMidShort:
        return launch_cfg<Cfg<128, 2, 2, 1, 2>>(p, n_workgroups, st);   //  64 x 128, 4 waves, ring 2 x  64 keys: problems too small to fill the chip
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace krul
