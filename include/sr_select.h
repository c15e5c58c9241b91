/*
 * sr_select.h -- offline dictionary selection (paper section III-A: Eq. 6/7,
 * the selection strategy of Alg. 1, the regression scales of Eq. 9), the step
 * that produces the kept-atom list and the scales gamma which
 * sr_dict_assemble_selective consumes.
 *
 * With the dictionary query and the filtering taken together, the image the
 * path produces with selector beta is, for a sample p (one HR pixel of one
 * channel),
 *
 *     y_p(beta) = sum_l beta_l r_{p,l},    r_{p,l} = Phi_{p,l} * (D_l . B_p)
 *
 * so Eq. 7 is a LASSO regression of ground-truth pixels h_p on the per-atom
 * responses.  sr_atom_gram forms its normal equations on the GPU (the only
 * part whose cost grows with the image); sr_select_atoms runs Alg. 1 on them
 * on the host.
 *
 * Fixed semantics (the paper leaves them open): the data term is averaged over
 * the M samples; the samples are the HR pixels whose row and column are
 * multiples of `stride`, all channels, all images (a deterministic stand-in
 * for the paper's random sampling); LASSO problems are solved by cyclic
 * coordinate descent; the lambda search is doubling followed by ordinary
 * bisection between the last lambda that left too many atoms and the first
 * that did not; between rounds the kept atoms are rescaled by the regression
 * scales of Eq. 9; alpha is not stepped below the target.
 *
 * Status codes are those of sr_dict.h.
 */
#ifndef SR_SELECT_H
#define SR_SELECT_H

#include <stddef.h>

#include "sr_dict.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SR_SELECT_MAX_ATOMS 128
#define SR_SELECT_STATIC_MAX_ATOMS 79      /* sr_atom_gram_static: what its built-in scratch holds */

/* Bytes of DEVICE scratch sr_atom_gram needs for L atoms (0 if L is out of
 * range).  The caller allocates it; its contents before and after are
 * meaningless. */
size_t sr_atom_gram_workspace_bytes(int L);

/*
 * Normal equations of Eq. 7.
 *
 *   up      [N][C][H][W]  f32   the up-sampled image (output of sr_bicubic_upsample)
 *   coeff   [N][L][H][W]  f32, f16, bf16 or f8e4m3   Phi
 *   dict    [1][L][k][k]  f32   D
 *   target  [N][C][H][W]  f32   ground truth h
 *   stride  >= 1: HR pixels (Y, X) with Y % stride == 0 and X % stride == 0 are the samples
 *   workspace, workspace_bytes   DEVICE scratch, >= sr_atom_gram_workspace_bytes(L), 16-byte aligned
 *   normal  DEVICE, L*L + L + 2 doubles, written:
 *             G[l][m] = sum_p r_pl r_pm   (L*L, row-major, symmetric)
 *             b[l]    = sum_p r_pl h_p    (L)
 *             hh      = sum_p h_p^2
 *             M       = number of samples p
 *
 * k in {3,5,7}, 1 <= L <= SR_SELECT_MAX_ATOMS, 1 <= C <= SR_MAX_CHANNELS.
 * Responses are formed in fp32, summed in fp32 over runs of 64 samples and in
 * double from there on, in a fixed order: the result is the same from run to
 * run.  Enqueued on `stream`, no synchronisation; nothing is allocated.
 * N = 0 or an empty image writes all zeros.
 */
int sr_atom_gram(const sr_tensor* up, const sr_tensor* coeff, const sr_tensor* dict,
                 const sr_tensor* target, int L, int k, int channels, int stride,
                 void* workspace, size_t workspace_bytes, double* normal, void* stream);

/*
 * sr_atom_gram for callers that cannot allocate device memory or pass a workspace: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments and result as sr_atom_gram without `workspace`: the per-workgroup partial
 * sums go to a 15 MiB buffer that is part of the library's device image (every GPU the
 * library is used on holds its own copy until the process ends).  It holds the scratch of
 * at most SR_SELECT_STATIC_MAX_ATOMS atoms; more is SR_ERR_SCRATCH, nothing is launched.
 * The call allocates nothing and frees nothing.  All calls on one GPU share that buffer:
 * two of them that overlap in time (different streams, or different host threads) race;
 * calls in stream order on one stream are fine, and nothing needs to be cleared between them.
 */
int sr_atom_gram_static(const sr_tensor* up, const sr_tensor* coeff, const sr_tensor* dict,
                        const sr_tensor* target, int L, int k, int channels, int stride,
                        double* normal, void* stream);

/*
 * Alg. 1 on the normal equations (HOST arrays; no GPU work).
 *
 *   normal        L*L + L + 2 doubles as written by sr_atom_gram (copied to the host)
 *   alpha         target fraction of atoms to keep, 0 < alpha <= 1
 *   delta_alpha   step of the outer loop, > 0
 *   lambda0       starting lambda, > 0
 *   eps           tolerance of the bisection on the kept fraction, >= 0
 *   kept          room for L ints: the kept atom indices, ascending
 *   n_kept        their number (<= alpha * L; may be 0 if nothing survives)
 *   gamma         room for L floats: the scale of each kept atom (product of the
 *                 regression scales of all rounds)
 *   lambda_out    the lambda reached, or NULL
 *
 * Returns SR_OK, SR_ERR_NULL, or SR_ERR_UNSUPPORTED for values out of range.
 */
int sr_select_atoms(const double* normal, int L, double alpha, double delta_alpha,
                    double lambda0, double eps,
                    int* kept, int* n_kept, float* gamma, double* lambda_out);

#ifdef __cplusplus
}
#endif
#endif /* SR_SELECT_H */
