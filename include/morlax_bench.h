/*
 * morlax_bench.h -- timing aid of the benchmark driver; not part of the method's interface
 * (include/morlax.h).  Exported by the same library.
 */
#ifndef MORLAX_BENCH_H
#define MORLAX_BENCH_H

#include "morlax.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Between morlax_profile_begin() and
 * morlax_profile_end() every grouped-GEMM launch of policy_fwd / policy_bwd on this ctx is bracketed
 * by a pair of HIP events recorded on the launch stream.  morlax_profile_end() waits for the last
 * event (it synchronises with the stream) and returns, per GEMM kind k in
 * {0 forward first layer, 1 forward hidden layer, 2 dX hidden layer, 3 dW hidden layer, 4 dW first
 * layer, 5 fused forward of all hidden layers in one launch}: ms[k] total kernel time, launches[k],
 * flops[k] total algorithmic flops (2 * rows * cols * depth summed over layers and preferences; tile
 * padding not counted).  The three arrays are HOST pointers of length 6.  Profiling stops at
 * morlax_profile_end(). */
int morlax_profile_begin(morlax_ctx* ctx);
int morlax_profile_end(morlax_ctx* ctx, double* ms, int64_t* launches, double* flops);

#ifdef __cplusplus
}
#endif
#endif /* MORLAX_BENCH_H */
