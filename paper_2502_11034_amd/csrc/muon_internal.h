// Launchers of the Muon path (muon.hip, muon_gemm.hip), called from api.cpp.  Kept apart from adagc_internal.h, which
// holds what the streaming kernels of the AdaGC step are compiled from.
#ifndef ADAGC_MUON_INTERNAL_H
#define ADAGC_MUON_INTERNAL_H

#include "adagc_internal.h"

namespace adagc {

// bf16 matrix-core GEMM of the Newton-Schulz iteration (muon_gemm.hip): C = bf16(alpha P Q^T + beta D), D given
// through its transpose Dt, result written row-major (C), transposed (Ct) or both; batch products of one shape per
// launch, matrix z of each array at base + z * stride elements.
hipError_t launch_gemm_nt_bf16(const void* P, int ldp, const void* Q, int ldq, int M, int N, int K, float alpha,
                               float beta, const void* Dt, int lddt, void* C, int ldc, void* Ct, int ldct,
                               hipStream_t stream, bool symmetric = false, int batch = 1, int64_t stride_p = 0,
                               int64_t stride_q = 0, int64_t stride_dt = 0, int64_t stride_c = 0, int64_t stride_ct = 0);
// Muon (muon.hip): momentum update with the clipped gradient and the partial sums of squares of U; X0 of one matrix
// into the padded workspace; the parameter update.
hipError_t launch_muon_momentum(const DeviceTables& t, double mu, int nesterov, int grad_bf16, int grid, hipStream_t stream);
hipError_t launch_muon_normalise(const void* g, const void* m, int64_t rows, int64_t cols, int64_t rows_p, int64_t cols_p,
                                 const double* coef, const double* sumsq, double mu, int nesterov, int grad_bf16,
                                 void* same, int64_t ld_same, void* trans, int64_t ld_trans, hipStream_t stream);
hipError_t launch_muon_apply(void* theta, const void* o, int64_t ld_o, int64_t rows, int64_t cols, double lr, double wd,
                             double scale, void* copy, hipStream_t stream);

}  // namespace adagc
#endif
