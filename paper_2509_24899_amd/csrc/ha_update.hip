// Parameter update of the attention-distillation loop (Attention Surgery, Sec. 3.3, Alg. "distil": the line
// phi <- phi - eta grad_phi L; the training details name AdamW with learning rate 1e-3 for this stage), gfx950.
// Elementwise and HBM-bound: one pass over the fp32 master copy, the gradient and (AdamW) the two moments, which also
// writes the parameter in the dtype the forward reads.  fp32 arithmetic; the bias corrections of AdamW are formed on
// the host in double precision.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "../../include/hybrid_attn.h"

namespace {

struct UpdateArgs {
  float *master;
  const float *grad;
  float *m, *v;
  void *param_io;
  int64_t n;
  float lr, grad_scale, beta1, beta2, eps, decay_factor, step_size, inv_sqrt_bc2;
};

template <bool ADAMW, int IO>   // IO 0: no copy, 1: bf16, 2: fp32
__global__ __launch_bounds__(256) void param_update_kernel(UpdateArgs a) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.n) return;
  const float g = a.grad_scale * a.grad[i];
  float p = a.master[i];
  if constexpr (ADAMW) {
    p *= a.decay_factor;
    const float m = a.beta1 * a.m[i] + (1.0f - a.beta1) * g;
    const float v = a.beta2 * a.v[i] + (1.0f - a.beta2) * g * g;
    a.m[i] = m;
    a.v[i] = v;
    p -= a.step_size * m / (sqrtf(v) * a.inv_sqrt_bc2 + a.eps);
  } else {
    p -= a.lr * g;
  }
  a.master[i] = p;
  if constexpr (IO == 1) static_cast<__bf16 *>(a.param_io)[i] = static_cast<__bf16>(p);
  if constexpr (IO == 2) static_cast<float *>(a.param_io)[i] = p;
}

}  // namespace

extern "C" ha_status hybrid_attn_param_update(const ha_optimizer *opt, size_t n, float *master, const float *grad, float *m,
                                              float *v, void *param_io, int32_t io_dtype, void *hip_stream) {
  if (!opt || !master || !grad) return HA_ERR_NULL;
  if (opt->kind != HA_OPT_SGD && opt->kind != HA_OPT_ADAMW) return HA_ERR_UNSUPPORTED;
  const bool adamw = opt->kind == HA_OPT_ADAMW;
  if (adamw && (!m || !v)) return HA_ERR_NULL;
  if (param_io && io_dtype != HA_BF16 && io_dtype != HA_F32) return HA_ERR_UNSUPPORTED;
  auto finite = [](float x) { return std::isfinite(x); };
  if (!finite(opt->lr) || !finite(opt->grad_scale) || opt->lr < 0.f) return HA_ERR_SHAPE;
  if (adamw) {
    if (opt->step < 1) return HA_ERR_SHAPE;
    if (!(opt->beta1 >= 0.f && opt->beta1 < 1.f) || !(opt->beta2 >= 0.f && opt->beta2 < 1.f)) return HA_ERR_SHAPE;
    if (!finite(opt->eps) || opt->eps < 0.f || !finite(opt->weight_decay) || opt->weight_decay < 0.f) return HA_ERR_SHAPE;
  }
  for (const void *t : {static_cast<const void *>(master), static_cast<const void *>(grad), static_cast<const void *>(m),
                        static_cast<const void *>(v)})
    if (reinterpret_cast<uintptr_t>(t) & 3u) return HA_ERR_ALIGN;
  if (param_io && (reinterpret_cast<uintptr_t>(param_io) & (io_dtype == HA_BF16 ? 1u : 3u))) return HA_ERR_ALIGN;
  if (param_io == master) return HA_ERR_SHAPE;
  if (n == 0) return HA_OK;
  if (n > ((size_t)1 << 40)) return HA_ERR_SHAPE;
  UpdateArgs a;
  a.master = master; a.grad = grad; a.m = m; a.v = v; a.param_io = param_io; a.n = (int64_t)n;
  a.lr = opt->lr; a.grad_scale = opt->grad_scale; a.beta1 = opt->beta1; a.beta2 = opt->beta2; a.eps = opt->eps;
  a.decay_factor = 1.f; a.step_size = 0.f; a.inv_sqrt_bc2 = 1.f;
  if (adamw) {
    const double bc1 = 1.0 - std::pow((double)opt->beta1, (double)opt->step);
    const double bc2 = 1.0 - std::pow((double)opt->beta2, (double)opt->step);
    a.decay_factor = (float)(1.0 - (double)opt->lr * (double)opt->weight_decay);
    a.step_size = (float)((double)opt->lr / bc1);
    a.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const unsigned blocks = (unsigned)((n + 255) / 256);
  const int io = !param_io ? 0 : (io_dtype == HA_BF16 ? 1 : 2);
#define HA_UPD(A, IO) param_update_kernel<A, IO><<<blocks, 256, 0, st>>>(a)
  if (adamw) { if (io == 0) HA_UPD(true, 0); else if (io == 1) HA_UPD(true, 1); else HA_UPD(true, 2); }
  else { if (io == 0) HA_UPD(false, 0); else if (io == 1) HA_UPD(false, 1); else HA_UPD(false, 2); }
#undef HA_UPD
  return hipGetLastError() == hipSuccess ? HA_OK : HA_ERR_DEVICE;
}
