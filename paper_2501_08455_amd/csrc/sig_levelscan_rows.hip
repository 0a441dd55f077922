// Level-scan family, stream mode: the launch of the top level, which writes whole output rows (its own level and the
// lower levels it has read).  A translation unit of its own so that the two halves of the family compile side by side.
#include "sig_levelscan.h"

namespace sig {
namespace levelscan {

hipError_t launch_rows_level(int d, int n, const LevelScanArgs &A, int vec, int blocks, int threads, size_t lds, hipStream_t st)
{
    return launch_level_d<true>(d, n, A, vec, blocks, threads, lds, st);
}

}  // namespace levelscan
}  // namespace sig
