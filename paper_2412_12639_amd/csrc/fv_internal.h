/* Internal surface of libfalcon_verify: tuning switches and bring-up aids that are not part of the
 * public C ABI (include/falcon_verify.h).  Every setting computes the same step and is held to the
 * same parity tests.
 *
 * Environment switches, read once by fv_create:
 *   FV_GEMM = paired | direct | shared   GEMM kernel for steps of up to 64 rows.  Default: paired
 *       (two 32-row strips per wavefront) wherever the K range is long enough, else direct (one
 *       strip).  shared: the LDS-shared-activation kernel that steps of more than 64 rows always use.
 *   FV_GEMM_ALIGN = 0 | 1     force the stream-K split (0) or whole row groups per workgroup (1);
 *       default: whole groups only where that idles at most 10 % of the workgroups.
 *   FV_GEMM_PAIRED_SET = mask over (QKV, O, gate/up, down, head): matrices that may use the paired form.
 *   FV_GEMM_WGS = n           workgroups the GEMMs are split over (default 256, one per compute unit).
 *   FV_GEMM_FIX = 0           steps of more than 64 rows: let the last workgroup to arrive reduce a row
 *       group's partial tiles inside the GEMM launch (default: a second launch reduces them, one
 *       wavefront per tile, for the QKV, O and down projections).
 *   FV_ATTN = invariant       contexts start with step-invariant rows switched on (fv_set_step_invariant(ctx, 1)).
 *   FV_EXCHANGE_TEST = timeout   test of the bounded wait in the direct / paired GEMM kernels: contributors leave their
 *       partial tiles unmarked and finishers give up after two looks, so every step of more than one
 *       workgroup per row group returns FV_E_EXCHANGE_TIMEOUT (every kernel still ends normally).
 *   FV_DEBUG = 1              print the failing HIP call of an FV_E_HIP status to stderr.
 */
#ifndef FV_INTERNAL_H
#define FV_INTERNAL_H
#include "../../include/falcon_verify.h"
#endif
