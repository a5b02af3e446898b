// The column-reduction sweep (pass 2) of the importance scoring: see score_sweep.h.  A translation
// unit of its own: it is compiled with the compiler's iterative-ILP scheduling strategy, which
// makes this sweep 5 % faster and the row-statistics sweep 3 % slower (build.py).
#include "score_sweep.h"

namespace speckv {

hipError_t launch_column_sweep(const ScoreArgs &A, hipStream_t st) { return dispatch_sweep<2>(A, st); }

}  // namespace speckv
