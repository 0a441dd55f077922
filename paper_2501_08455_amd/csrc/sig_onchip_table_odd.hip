// More compiled on-chip kernels: the channel counts the other tables leave out (7 at depth 2, 9 at depths 2-5) and
// depth 5 for 7-10 channels, so that every d = 2 .. 10 has a register kernel up to depth 4 (up to 5 from d = 3),
// with the prefix depth that keeps a lane's sub-tree near 64 floats (larger ones run at fewer wavefronts per SIMD,
// like the (10, 6, 4) kernel of the large-signature configuration).
#include "sig_onchip.h"

namespace sig {

namespace {
const OnChipKernelInfo kTable[] = {
    SIG_ON_CHIP_ENTRY(7, 2, 1),
    SIG_ON_CHIP_ENTRY(9, 2, 1),
    SIG_ON_CHIP_ENTRY(9, 3, 2),
    SIG_ON_CHIP_ENTRY(9, 4, 2),
    SIG_ON_CHIP_ENTRY(9, 4, 3),   // for batches too small to fill the chip with 81 lanes per path
    SIG_ON_CHIP_ENTRY(7, 5, 3),
    SIG_ON_CHIP_ENTRY(8, 5, 3),
    SIG_ON_CHIP_ENTRY(9, 5, 3),
    SIG_ON_CHIP_ENTRY(10, 5, 3),
    {0, 0, 0, 0, 0, 0, nullptr, nullptr, nullptr},
};
}  // namespace

const OnChipKernelInfo *on_chip_table_odd() { return kTable; }

}  // namespace sig
