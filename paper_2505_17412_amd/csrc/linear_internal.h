// Pieces of the linear-projection kernels that the layer composition calls directly (gfx950 only).
#pragma once

#include "ssa_internal.h"

// d_in, d_out multiples of 128 up to 16384; SSA_OK or the error the entry points report
int lin_check(int n_tokens, int d_in, int d_out);

// Y [M][O] (bf16) = sum over n_src <= 3 pairs of X_i [M][K_i] W_i[O][K_i]^T (+ bias [O]); every K_i a multiple of 128
int lin_nt_multi(int n_src, const void *const *X, const void *const *W, const int *K, const void *bias, int M, int O,
                 void *Y, hipStream_t s);

// wt [d_in][d_out] = w [d_out][d_in]^T
void lin_transpose_w(const void *w, int d_out, int d_in, void *wt, hipStream_t s);

// dw [d_out][d_in] (fp32) = dy^T x, dbias [d_out] (fp32, optional) = column sums of dy; ws: lin_dw_workspace() bytes,
// 256-byte aligned
size_t lin_dw_workspace(int M, int d_in, int d_out);
int lin_dw(int M, int d_in, int d_out, const void *x, const void *dy, float *dw, float *dbias, void *ws, hipStream_t s);
