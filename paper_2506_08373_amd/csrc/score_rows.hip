// The row-statistics sweep (pass 1) of the importance scoring: see score_sweep.h.  A translation
// unit of its own so that the two sweeps can be compiled with different scheduling strategies.
#include "score_sweep.h"

namespace speckv {

hipError_t launch_row_statistics_sweep(const ScoreArgs &A, hipStream_t st) { return dispatch_sweep<1>(A, st); }

}  // namespace speckv
