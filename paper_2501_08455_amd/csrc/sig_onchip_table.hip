// Table of the compiled on-chip kernels: one entry per (d, depth, prefix depth).
#include "sig_onchip.h"

namespace sig {

namespace {
const OnChipKernelInfo kTable[] = {
    SIG_ON_CHIP_ENTRY(2, 3, 0),
    SIG_ON_CHIP_ENTRY(2, 3, 1),
    SIG_ON_CHIP_ENTRY(4, 4, 1),
    SIG_ON_CHIP_ENTRY(4, 4, 2),
    SIG_ON_CHIP_ENTRY(4, 4, 3),
    SIG_ON_CHIP_ENTRY(5, 4, 1),
    SIG_ON_CHIP_ENTRY(5, 4, 2),
    SIG_ON_CHIP_ENTRY(5, 4, 3),
    SIG_ON_CHIP_ENTRY(10, 6, 4),
    {0, 0, 0, 0, 0, 0, nullptr, nullptr, nullptr},
};
}  // namespace

const OnChipKernelInfo *on_chip_table_base() { return kTable; }

const OnChipKernelInfo *on_chip_subtable(int i)
{
    switch (i) {
    case 0: return on_chip_table_base();
    case 1: return on_chip_table_depth2();
    case 2: return on_chip_table_depth3();
    case 3: return on_chip_table_depth4();
    case 4: return on_chip_table_depth56();
    case 5: return on_chip_table_odd();
    default: return nullptr;
    }
}

const OnChipKernelInfo *find_on_chip(int d, int depth, int p)
{
    for (int t = 0; on_chip_subtable(t); ++t)
        for (const OnChipKernelInfo *e = on_chip_subtable(t); e->launch; ++e)
            if (e->d == d && e->depth == depth && e->p == p) return e;
    return nullptr;
}

}  // namespace sig
