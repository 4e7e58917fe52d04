// Instantiations of the similarity kernel: the wide tile shapes at head_dim 64 (one translation unit per
// group of shapes, so that they compile side by side).  Tile shapes must match make_plan().
#include "krul_mfma_kernel.h"

namespace krul {

hipError_t launch_sim_mfma_wide64(const SimParams &p, int n_workgroups, hipStream_t st)
{
    switch (p.lay.variant) {   //                      D  WR WK KBW NC
    case kMfmaWide:
        return launch_cfg<Cfg<64, 4, 2, 1, 4>>(p, n_workgroups, st);   // 128 x 256, 8 waves, ring 4 x  64 keys
    case kMfmaWideShort:
        return launch_cfg<Cfg<64, 4, 2, 1, 2>>(p, n_workgroups, st);   // 128 x 128, 8 waves, ring 2 x  64 keys: problems too small to fill the chip
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace krul
