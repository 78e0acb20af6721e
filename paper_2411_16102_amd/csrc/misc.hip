// Small kernels around the GEMMs: RMSNorm preparation of the layer input, the
// RoPE angle table, and conversion between token-major K/V arrays and the
// library's KV page layout.
#include "misc.hpp"
#include "common.hpp"

namespace bs {
namespace {

// One wavefront per row: xg = bf16(x * g) (the GEMM operand of the normalised
// row; the 1/rms factor commutes with the contraction and is applied in the GEMM
// epilogue) and rstd = 1 / sqrt(mean(x^2) + eps).
__global__ __launch_bounds__(256) void norm_prep_kernel(const uint16_t *x, const uint16_t *g, uint16_t *xg,
                                                       float *rstd, int rows, int d, float eps, unsigned *zero_words,
                                                       int n_zero) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // the first kernel of a step also clears the step's counters (a fill in a kernel, not a
  // memset on the stream, so that a captured step replays it like any other launch)
  if (blockIdx.x == 0 && (int)threadIdx.x < n_zero) zero_words[threadIdx.x] = 0u;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows) return;
  const uint16_t *xr = x + (size_t)row * d;
  uint16_t *outr = xg + (size_t)row * d;
  float s = 0.f;
  for (int c = lane * 8; c < d; c += 64 * 8) {
    const u32x4_t xv = *reinterpret_cast<const u32x4_t *>(xr + c);
    const u32x4_t gv = *reinterpret_cast<const u32x4_t *>(g + c);
    u32x4_t ov;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float x0 = __uint_as_float(xv[i] << 16), x1 = __uint_as_float(xv[i] & 0xFFFF0000u);
      const float g0 = __uint_as_float(gv[i] << 16), g1 = __uint_as_float(gv[i] & 0xFFFF0000u);
      s += x0 * x0 + x1 * x1;
      ov[i] = pack_bf16x2(x0 * g0, x1 * g1);
    }
    *reinterpret_cast<u32x4_t *>(outr + c) = ov;
  }
  s = wave_sum(s);
  if (lane == 0) rstd[row] = rsqrtf(s / (float)d + eps);
}

// rstd[m] = 1 / sqrt(sum_p part[p][m] / d + eps): closes the row sums of squares that
// the output projection's epilogue leaves per column tile.  A workgroup covers 64 rows;
// its four wavefronts each add every fourth partial (coalesced along the rows, the loads
// of a thread independent of each other) and meet in LDS.
__global__ __launch_bounds__(256) void rstd_finalize_kernel(const float *part, int n_part, int stride, float *rstd,
                                                            int rows, float d, float eps) {
  __shared__ float sh[4][64];
  const int r = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int m = blockIdx.x * 64 + r;
  float s = 0.f;
  if (m < rows) {
#pragma unroll 8
    for (int p = q; p < n_part; p += 4) s += part[(size_t)p * stride + m];
  }
  sh[q][r] = s;
  __syncthreads();
  if (q == 0 && m < rows) rstd[m] = rsqrtf((sh[0][r] + sh[1][r] + sh[2][r] + sh[3][r]) / d + eps);
}

// cos/sin of pos * theta^(-2i/dh), evaluated in double and stored as float
__global__ void rope_table_kernel(float *cos_t, float *sin_t, int max_pos, int half, double theta) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)max_pos * half) return;
  const int pos = (int)(idx / half), i = (int)(idx % half);
  const double freq = pow(theta, -(double)i / (double)half);
  double s, c;
  sincos((double)pos * freq, &s, &c);
  cos_t[idx] = (float)c;
  sin_t[idx] = (float)s;
}

// token-major k, v [n_pages][16][Hkv][dh]  <->  pages of K [Hkv][16][dh] and V^T [Hkv][dh][16]
__global__ void kv_pack_kernel(const uint16_t *k, const uint16_t *v, uint16_t *pool, long n_pages, int hkv, int dh,
                               int unpack, uint16_t *k_out, uint16_t *v_out) {
  const long per_page = (long)16 * hkv * dh;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_pages * per_page) return;
  const long page = idx / per_page;
  long r = idx % per_page;
  const int slot = (int)(r / (hkv * dh));
  r %= (long)hkv * dh;
  const int head = (int)(r / dh), e = (int)(r % dh);
  const long tile = (long)16 * dh;
  const long kd = ((page * 2 + 0) * hkv + head) * tile + (long)slot * dh + e;
  const long vd = ((page * 2 + 1) * hkv + head) * tile + (long)e * 16 + slot;
  if (unpack) {
    k_out[idx] = pool[kd];
    v_out[idx] = pool[vd];
  } else {
    pool[kd] = k[idx];
    pool[vd] = v[idx];
  }
}

}  // namespace

hipError_t launch_norm_prep(const uint16_t *x, const uint16_t *g, uint16_t *xg, float *rstd, int rows, int d,
                            float eps, unsigned *zero_words, int n_zero, hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(norm_prep_kernel, dim3((rows + 3) / 4), dim3(256), 0, stream, x, g, xg, rstd, rows, d, eps,
                     zero_words, zero_words ? n_zero : 0);
  return hipGetLastError();
}

hipError_t launch_rstd_finalize(const float *part, int n_part, int stride, float *rstd, int rows, int d, float eps,
                                hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(rstd_finalize_kernel, dim3((rows + 63) / 64), dim3(256), 0, stream, part, n_part, stride, rstd,
                     rows, (float)d, eps);
  return hipGetLastError();
}

hipError_t launch_rope_table(float *cos_t, float *sin_t, int max_pos, int half, double theta, hipStream_t stream) {
  const long n = (long)max_pos * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, cos_t, sin_t,
                     max_pos, half, theta);
  return hipGetLastError();
}

hipError_t launch_kv_pack(const uint16_t *k, const uint16_t *v, uint16_t *pool, long n_pages, int hkv, int dh,
                          hipStream_t stream) {
  const long n = n_pages * 16 * hkv * dh;
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_pack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, k, v, pool, n_pages,
                     hkv, dh, 0, nullptr, nullptr);
  return hipGetLastError();
}

hipError_t launch_kv_unpack(const uint16_t *pool, uint16_t *k, uint16_t *v, long n_pages, int hkv, int dh,
                            hipStream_t stream) {
  const long n = n_pages * 16 * hkv * dh;
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_pack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, nullptr, nullptr,
                     const_cast<uint16_t *>(pool), n_pages, hkv, dh, 1, k, v);
  return hipGetLastError();
}

}  // namespace bs
