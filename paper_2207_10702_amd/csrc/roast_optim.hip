// Optimizer step on the shared array M: the "update weights" leg of the paper's training workload
// (Appendix tables "update weights (optim.step())": SGD, Adagrad and Adam on the |M|-sized
// parameter).  One streaming pass over |M| floats that also does what would otherwise be two more
// passes: it clears the gradient for the next step and refreshes the bf16 shadow of M that the bf16
// ROAST-MM kernels read.  HBM-bound: 8 (SGD) to 24 (Adam) bytes read and 4 to 16 bytes written per
// parameter, 4 parameters per thread.
#include "roast_internal.hpp"

namespace roast {
namespace {

typedef float vfloat4 __attribute__((ext_vector_type(4)));

struct OptimArgs {
  int kind;
  float lr, wd, b1, b2, eps;
  float omb1, omb2;       // 1 - beta, computed on the host in double (1.f - 0.999f is off by 1e-5)
  float bc1, bc2;         // Adam bias corrections 1 - beta^t, computed on the host in double
  int zero_grad;
  int64_t n, stride;      // |M|, distance between the two copies of the shadow
};

__device__ inline float update(const OptimArgs& a, float m, float g, float* s1, float* s2) {
  g = fmaf(a.wd, m, g);
  if (a.kind == ROAST_OPT_SGD) return m - a.lr * g;
  if (a.kind == ROAST_OPT_ADAGRAD) {
    *s1 = fmaf(g, g, *s1);
    return m - a.lr * g / (sqrtf(*s1) + a.eps);
  }
  *s1 = a.b1 * *s1 + a.omb1 * g;
  *s2 = a.b2 * *s2 + a.omb2 * g * g;
  return m - a.lr * (*s1 / a.bc1) / (sqrtf(*s2 / a.bc2) + a.eps);
}

__device__ inline uint16_t to_bf16(float v) { return __builtin_bit_cast(uint16_t, (__bf16)v); }

__global__ __launch_bounds__(256) void k_optim(OptimArgs a, float* __restrict__ M, float* __restrict__ dM,
                                               float* __restrict__ st1, float* __restrict__ st2,
                                               uint16_t* __restrict__ shadow) {
  const int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i0 >= a.n) return;
  if (i0 + 4 <= a.n) {
    vfloat4 m = *reinterpret_cast<const vfloat4*>(M + i0);
    const vfloat4 g = *reinterpret_cast<const vfloat4*>(dM + i0);
    vfloat4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
    if (a.kind != ROAST_OPT_SGD) s1 = *reinterpret_cast<const vfloat4*>(st1 + i0);
    if (a.kind == ROAST_OPT_ADAM) s2 = *reinterpret_cast<const vfloat4*>(st2 + i0);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float x = s1[k], y = s2[k];
      m[k] = update(a, m[k], g[k], &x, &y);
      s1[k] = x; s2[k] = y;
    }
    *reinterpret_cast<vfloat4*>(M + i0) = m;
    if (a.kind != ROAST_OPT_SGD) *reinterpret_cast<vfloat4*>(st1 + i0) = s1;
    if (a.kind == ROAST_OPT_ADAM) *reinterpret_cast<vfloat4*>(st2 + i0) = s2;
    if (a.zero_grad) *reinterpret_cast<vfloat4*>(dM + i0) = vfloat4{0.f, 0.f, 0.f, 0.f};
    if (shadow) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint16_t h = to_bf16(m[k]);
        shadow[i0 + k] = h;                                   // copy 0: shadow[i] = bf16(M[i])
        if (i0 + k >= 1) shadow[a.stride + i0 + k - 1] = h;   // copy 1: shadow[stride + i] = bf16(M[i + 1])
      }
    }
  } else {
    for (int64_t i = i0; i < a.n; ++i) {
      float x = a.kind != ROAST_OPT_SGD ? st1[i] : 0.f, y = a.kind == ROAST_OPT_ADAM ? st2[i] : 0.f;
      const float m = update(a, M[i], dM[i], &x, &y);
      M[i] = m;
      if (a.kind != ROAST_OPT_SGD) st1[i] = x;
      if (a.kind == ROAST_OPT_ADAM) st2[i] = y;
      if (a.zero_grad) dM[i] = 0.f;
      if (shadow) {
        shadow[i] = to_bf16(m);
        if (i >= 1) shadow[a.stride + i - 1] = to_bf16(m);
      }
    }
  }
}

}  // namespace

roast_status optim_launch(const roast_optim_desc& d, int64_t m_size, float* M, float* dM, float* st1, float* st2,
                          void* shadow, hipStream_t s) {
  OptimArgs a{};
  a.kind = (int)d.kind; a.lr = d.lr; a.wd = d.weight_decay; a.b1 = d.beta1; a.b2 = d.beta2; a.eps = d.eps;
  a.omb1 = (float)(1.0 - (double)d.beta1);
  a.omb2 = (float)(1.0 - (double)d.beta2);
  a.bc1 = (float)(1.0 - pow((double)d.beta1, (double)d.step));
  a.bc2 = (float)(1.0 - pow((double)d.beta2, (double)d.step));
  a.zero_grad = d.zero_grad ? 1 : 0;
  a.n = m_size; a.stride = shadow_stride(m_size);
  const int64_t blocks = (m_size + 1023) / 1024;
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_optim, dim3((unsigned)blocks), dim3(256), 0, s, a, M, dM, st1, st2, (uint16_t*)shadow);
  return hip_status(hipGetLastError());
}

}  // namespace roast
