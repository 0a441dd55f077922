// More compiled on-chip kernels (depth 3): channel counts 2 .. 10 of the paper's experiments (Section 4), with
// the prefix depth that keeps a lane's sub-tree at about 64 floats or fewer.
#include "sig_onchip.h"

namespace sig {

namespace {
const OnChipKernelInfo kTable[] = {
    SIG_ON_CHIP_ENTRY(3, 3, 1),
    SIG_ON_CHIP_ENTRY(3, 3, 2),
    SIG_ON_CHIP_ENTRY(4, 3, 1),
    SIG_ON_CHIP_ENTRY(4, 3, 2),
    SIG_ON_CHIP_ENTRY(5, 3, 1),
    SIG_ON_CHIP_ENTRY(5, 3, 2),
    SIG_ON_CHIP_ENTRY(6, 3, 1),
    SIG_ON_CHIP_ENTRY(6, 3, 2),
    SIG_ON_CHIP_ENTRY(7, 3, 1),
    SIG_ON_CHIP_ENTRY(7, 3, 2),
    SIG_ON_CHIP_ENTRY(8, 3, 2),
    SIG_ON_CHIP_ENTRY(10, 3, 2),
    {0, 0, 0, 0, 0, 0, nullptr, nullptr, nullptr},
};
}  // namespace

const OnChipKernelInfo *on_chip_table_depth3() { return kTable; }

}  // namespace sig
