// Process-wide switches for tests and measurements (not part of the public ABI of include/heta.h; the
// symbols are exported so that the Python tests can reach them).  Not thread-safe.
#pragma once

#include "heta.h"

#ifdef __cplusplus
extern "C" {
#endif

/* 0 = by size (the default): a relation of at least 2^18 edges + rows is ingested by the per-relation device
 * kernels; the smaller relations of a graph together by the whole-block device ingest when they add up
 * to 2^16 edges + rows, else on the host.  1 = everything on the host, 2 = everything by the
 * per-relation device kernels, 3 = small relations always by the whole-block device ingest.  All paths
 * produce identical index arrays. */
heta_status heta_ingest_force(int32_t mode);

/* When on, every projection runs the register-staged kernel that otherwise only serves operands whose
 * rows are not 16-byte aligned; off (the default) prefers the direct-to-LDS pipeline.  Results agree to
 * rounding order. */
heta_status heta_projection_force_staged(int32_t on);

/* fp32 x fp32 projections on the direct pipeline form every product from three bf16 terms per operand (six
 * bf16 MFMAs, fp32 accumulation: products exact to 2^-25).  When on, they run on the fp32 MFMA (32x32x2)
 * instead: the same results to rounding order at about 2.5 times the matrix-pipe time. */
heta_status heta_projection_f32_native(int32_t on);

#ifdef __cplusplus
}
#endif
