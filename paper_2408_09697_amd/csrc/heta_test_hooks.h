// Process-wide switches for tests and measurements (not part of the public ABI of include/heta.h; the
// symbols are exported so that the Python tests can reach them).  Not thread-safe.
#pragma once

#include "heta.h"

#ifdef __cplusplus
extern "C" {
#endif

/* 0 = relations of at least 2^18 edges + rows are ingested by device kernels and smaller ones on the
 * host (the default), 1 = always on the host, 2 = always on the device.  Both paths produce identical
 * index arrays. */
heta_status heta_ingest_force(int32_t mode);

/* When on, every projection runs the register-staged kernel that otherwise only serves operands whose
 * rows are not 16-byte aligned; off (the default) prefers the direct-to-LDS pipeline.  Results agree to
 * rounding order. */
heta_status heta_projection_force_staged(int32_t on);

#ifdef __cplusplus
}
#endif
