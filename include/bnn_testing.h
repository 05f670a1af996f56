/*
 * bnn_testing.h -- switches for tests and measurements; NOT part of the library's ABI and
 * not meant for applications.  They set process-wide state and are not thread-safe; a test
 * that uses one restores the default afterwards.  None of them changes any result: every
 * kernel variant they select computes the values bnn.h specifies.
 */
#ifndef BNN_TESTING_H_
#define BNN_TESTING_H_

#include "bnn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Force the tile configuration of the Xnor-Bitcount GEMM (section 3.2) instead of the size
 * heuristic, for bnn_xnor_gemm, bnn_xnor_gemm_epilogue, bnn_conv2d and bnn_conv2d_packed:
 *   -1  heuristic (default)
 *    1  32 x 256 tile      2  32 x 64       3  64 x 256      4  32 x 128      6  64 x 128
 *    7  one wave per 8 x 64 tile, operand B read straight from memory (small problems)
 *    8  one wave per 8 x 128 tile, likewise
 *    9  as 7 with the reduction axis split over the four waves of a workgroup
 * A value that a call cannot use (the packed epilogue needs the 64 x 256 tile) is ignored
 * by that call.  Other values select the heuristic.
 */
BNN_API void bnn_internal_force_gemm_cfg(int cfg);

/*
 * 1 (default): convolutions whose geometry allows it gather their patches with the
 * table-driven loader; 0: always the general loader.
 */
BNN_API void bnn_internal_lean_gather(int on);

/*
 * Selects what bnn_valu_peak_probe runs.  Each mode issues the same number of vector
 * lane-operations per launch for given (blocks, iters), so rates compare directly.
 *    0  (default) independent xor + popcount pairs, both operands in vector registers
 *    1  the GEMM's pattern: xor operand in a scalar register, each xor directly followed by
 *       the popcount that consumes it
 *    2  xor only;  3  popcount-accumulate only;  4  dependent pairs, vector operands
 *    5, 6  the GEMM's own row statements for 2 / 4 column groups per lane (with the yield)
 *    7, 8  the same without the yield
 *    9, 10 fp32 multiply-add chains, multiplier in a vector (9) / a scalar (10) register
 * Unknown values run mode 0.
 */
BNN_API void bnn_internal_probe_mode(int mode);

#ifdef __cplusplus
}
#endif
#endif /* BNN_TESTING_H_ */
