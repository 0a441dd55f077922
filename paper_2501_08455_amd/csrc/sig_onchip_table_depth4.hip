// More compiled on-chip kernels (depth 4): channel counts 2 .. 10 of the paper's experiments (Section 4), with
// the prefix depth that keeps a lane's sub-tree at about 64 floats or fewer.  8 and 10 channels also have a deeper
// prefix (a lane state of 9 / 11 floats, 512 / 1,000 lanes per path) for batches too small to fill the chip with
// 64 / 100 lanes per path: 1.2-2.2x up to about 128 paths, 1.7-2x slower from 1,024 paths on.
#include "sig_onchip.h"

namespace sig {

namespace {
const OnChipKernelInfo kTable[] = {
    SIG_ON_CHIP_ENTRY(2, 4, 1),
    SIG_ON_CHIP_ENTRY(2, 4, 2),
    SIG_ON_CHIP_ENTRY(3, 4, 1),
    SIG_ON_CHIP_ENTRY(3, 4, 2),
    SIG_ON_CHIP_ENTRY(3, 4, 3),
    SIG_ON_CHIP_ENTRY(6, 4, 2),
    SIG_ON_CHIP_ENTRY(6, 4, 3),
    SIG_ON_CHIP_ENTRY(7, 4, 2),
    SIG_ON_CHIP_ENTRY(8, 4, 2),
    SIG_ON_CHIP_ENTRY(8, 4, 3),
    SIG_ON_CHIP_ENTRY(10, 4, 2),
    SIG_ON_CHIP_ENTRY(10, 4, 3),
    {0, 0, 0, 0, 0, 0, nullptr, nullptr, nullptr},
};
}  // namespace

const OnChipKernelInfo *on_chip_table_depth4() { return kTable; }

}  // namespace sig
