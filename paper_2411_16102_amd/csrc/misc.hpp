// Launchers of the small kernels (see misc.hip).
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

namespace bs {
hipError_t launch_norm_prep(const uint16_t *x, const uint16_t *g, uint16_t *xg, float *rstd, int rows, int d,
                            float eps, unsigned *zero_words, int n_zero, hipStream_t stream);
hipError_t launch_rstd_finalize(const float *part, int n_part, int stride, float *rstd, int rows, int d, float eps,
                                hipStream_t stream);
hipError_t launch_rope_table(float *cos_t, float *sin_t, int max_pos, int half, double theta, hipStream_t stream);
hipError_t launch_kv_pack(const uint16_t *k, const uint16_t *v, uint16_t *pool, long n_pages, int hkv, int dh,
                          hipStream_t stream);
hipError_t launch_kv_unpack(const uint16_t *pool, uint16_t *k, uint16_t *v, long n_pages, int hkv, int dh,
                            hipStream_t stream);
}  // namespace bs
