// The paper's timing model for synchronous model-distributed training (Sec. 3.1, App. C): host
// arithmetic only.  A accelerators in sequence, M micro-batches per mini-batch, window N (clamped to
// A); one slot - a forward or a backward of one micro-batch on one accelerator - costs
// c(M) = c0 + c1 / M.
#include <cmath>
#include <cstdint>

#include "../../include/interlock.h"

extern "C" {

double il_time_per_batch(int32_t A, int32_t M, int32_t N, double c0, double c1) {
  if (A < 1 || M < 1 || N < 1) return NAN;
  if (N > A) N = A;
  const double c = c0 + c1 / M;
  if (M == 1) return 2.0 * N * M * c;                    // N forward slots, then N backward slots
  if (M == 2 || A >= 2 * N - 1) return (N + 1.0) * M * c; // the middle accelerator: 1 forward + N backwards per micro-batch
  return (2.0 + A - N) * M * c + 2.0 * (2 * N - A - 1) * c;
}

int32_t il_optimal_microbatches(int32_t A, int32_t N, double c0, double c1, int32_t max_m) {
  if (A < 1 || N < 1 || max_m < 1) return IL_E_ARG;
  int32_t best = 1;
  double best_t = INFINITY;
  for (int64_t m = 1; m <= max_m; m *= 2) {
    const double t = il_time_per_batch(A, (int32_t)m, N, c0, c1);
    if (t < best_t) { best_t = t; best = (int32_t)m; }
  }
  return best;
}

}  // extern "C"
