// More compiled on-chip kernels (depths 5 and 6): channel counts 2 .. 10 of the paper's experiments (Section 4), with
// the prefix depth that keeps a lane's sub-tree at about 64 floats or fewer.
#include "sig_onchip.h"

namespace sig {

namespace {
const OnChipKernelInfo kTable[] = {
    SIG_ON_CHIP_ENTRY(2, 5, 1),
    SIG_ON_CHIP_ENTRY(2, 5, 2),
    SIG_ON_CHIP_ENTRY(3, 5, 2),
    SIG_ON_CHIP_ENTRY(3, 5, 3),
    SIG_ON_CHIP_ENTRY(4, 5, 3),
    SIG_ON_CHIP_ENTRY(5, 5, 3),
    SIG_ON_CHIP_ENTRY(6, 5, 3),
    SIG_ON_CHIP_ENTRY(2, 6, 1),
    SIG_ON_CHIP_ENTRY(2, 6, 2),
    SIG_ON_CHIP_ENTRY(2, 6, 3),
    SIG_ON_CHIP_ENTRY(3, 6, 3),
    SIG_ON_CHIP_ENTRY(3, 6, 4),
    SIG_ON_CHIP_ENTRY(4, 6, 4),
    SIG_ON_CHIP_ENTRY(5, 6, 4),
    {0, 0, 0, 0, 0, 0, nullptr, nullptr, nullptr},
};
}  // namespace

const OnChipKernelInfo *on_chip_table_depth56() { return kTable; }

}  // namespace sig
