/* Synthetic residual driver for benchmarks and tests of moe_spec (not part of the method).
 *
 * The workloads have no attention; what happens to the residual stream between two MoE blocks
 * is replaced by  v = r + O,  r' = a*v + b*(|v|_2/sqrt(H))*eps  per row, with eps a seeded
 * standard-normal draw supplied by the caller.  All pointers are device memory, row-major
 * [batch, hidden] float; r_next_dev may alias r_dev.  Runs on `stream` (a hipStream_t).
 * Returns 0, -1 on bad arguments, -4 on a launch failure.
 */
#ifndef MOE_SPEC_SYNTH_H
#define MOE_SPEC_SYNTH_H
#ifdef __cplusplus
extern "C" {
#endif
int moe_spec_synth_advance(void *stream, const float *r_dev, const float *out_dev, const float *eps_dev,
                           double a, double b, int batch, int hidden, float *r_next_dev);
#ifdef __cplusplus
}
#endif
#endif
