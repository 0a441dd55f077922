// More compiled on-chip kernels (depth 4): channel counts 2 .. 10 of the paper's experiments (Section 4), with
// the prefix depth that keeps a lane's sub-tree at about 64 floats or fewer.
#include "sig_onchip.h"

namespace sig {

namespace {
const OnChipKernelInfo kTable[] = {
    SIG_ON_CHIP_ENTRY(2, 4, 1),
    SIG_ON_CHIP_ENTRY(3, 4, 1),
    SIG_ON_CHIP_ENTRY(6, 4, 2),
    SIG_ON_CHIP_ENTRY(7, 4, 2),
    SIG_ON_CHIP_ENTRY(8, 4, 2),
    SIG_ON_CHIP_ENTRY(10, 4, 2),
    {0, 0, 0, 0, 0, 0, nullptr, nullptr, nullptr},
};
}  // namespace

const OnChipKernelInfo *on_chip_table_depth4() { return kTable; }

}  // namespace sig
