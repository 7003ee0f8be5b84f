// Worker reduce (Sec. 3.2 step 3, Sec. 3.3 step 2), momentum update (Sec. 3.3
// step 3) and the two fused.  All three are streaming kernels bound by HBM
// bandwidth: 16-byte loads/stores, every input element read exactly once,
// grid-stride loops sized to keep every CU busy with many loads in flight.
#include <math.h>

#include "common.h"

namespace synk {

struct BufTable {
  const void* p[SYNK_MAX_WORKERS];
  float w[SYNK_MAX_WORKERS];
};

struct ConcatTable {
  const uint32_t* src[SYNK_MAX_WORKERS];
  int64_t start[SYNK_MAX_WORKERS + 1];
};

// 128 threads: measured on 25.6 M parameters and 8 workers, workgroups of 64, 128 and 512 threads all
// stream at 6.8 TB/s and those of 256 at 6.4.
constexpr int kBlock = 128;

// One 16-byte unit per thread up to 2^20 workgroups (the kernels stride over
// the rest): workgroups then start in address order as earlier ones retire,
// which measured faster than a resident grid striding over the array
// (25.6 M parameters, 8 workers: 6.5 against 6.3 TB/s).
static inline int stream_grid(int64_t units) {
  int64_t b = (units + kBlock - 1) / kBlock;
  const int64_t cap = (int64_t)1 << 20;
  if (b > cap) b = cap;
  if (b < 1) b = 1;
  return (int)b;
}

__device__ __forceinline__ f32x4 ld_stream(const f32x4* p) {
  return __builtin_nontemporal_load(p);
}

__device__ __forceinline__ f32x4 fma4(float w, f32x4 g, f32x4 acc) {
  return f32x4{fmaf(w, g.x, acc.x), fmaf(w, g.y, acc.y), fmaf(w, g.z, acc.z), fmaf(w, g.w, acc.w)};
}

__device__ __forceinline__ void sgd_elem(float G, float& p, float& v, float lr, float m, float wd) {
  const float g = G + wd * p;
  v = m * v - lr * g;
  p = p + v;
}

// The other update rules of Sec. 3.3 (published forms; g = G + wd * p):
//   NESTEROV  v' = m v - lr g ;  p' = p + m v' - lr g
//   RMSPROP   a' = rho a + (1 - rho) g^2 ;  p' = p - lr g / sqrt(a' + eps)
//   ADAM      m' = b1 m + (1 - b1) g ;  v' = b2 v + (1 - b2) g^2 ;
//             p' = p - a_t m' / (sqrt(v') + eps),  a_t = lr sqrt(1 - b2^t) / (1 - b1^t)
// s1 is the velocity / the accumulator / the first moment, s2 the second moment.
struct RuleParams {
  float lr, m, wd;        // momentum rules: m = momentum; RMSPROP: m = rho; ADAM: m = beta1
  float b2, eps, a_t;     // ADAM: beta2, eps, bias-corrected step; RMSPROP: eps
};

template <int RULE>
__device__ __forceinline__ void rule_elem(float G, float& p, float& s1, float& s2, const RuleParams& h) {
  const float g = G + h.wd * p;
  if (RULE == SYNK_RULE_MOMENTUM) {
    s1 = h.m * s1 - h.lr * g;
    p = p + s1;
  } else if (RULE == SYNK_RULE_NESTEROV) {
    s1 = h.m * s1 - h.lr * g;
    p = p + h.m * s1 - h.lr * g;
  } else if (RULE == SYNK_RULE_RMSPROP) {
    s1 = h.m * s1 + (1.0f - h.m) * g * g;
    p = p - h.lr * g / sqrtf(s1 + h.eps);
  } else {
    s1 = h.m * s1 + (1.0f - h.m) * g;
    s2 = h.b2 * s2 + (1.0f - h.b2) * g * g;
    p = p - h.a_t * s1 / (sqrtf(s2) + h.eps);
  }
}

// The fused reduce + update for any rule: the skeleton of reduce_sgd_kernel
// with one more state stream for ADAM.
template <int NS, int RULE>
__global__ __launch_bounds__(kBlock) void reduce_update_kernel(BufTable t, int n_dyn, int64_t len,
                                                               float* __restrict__ p,
                                                               float* __restrict__ s1,
                                                               float* __restrict__ s2, RuleParams h,
                                                               uint16_t* __restrict__ p_lp,
                                                               const float* __restrict__ loss_in,
                                                               float* __restrict__ loss_out) {
  constexpr bool TWO = RULE == SYNK_RULE_ADAM;
  const int n = NS > 0 ? NS : n_dyn;
  const int64_t n_vec = len >> 2;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  f32x4* p4 = reinterpret_cast<f32x4*>(p);
  f32x4* a4 = reinterpret_cast<f32x4*>(s1);
  f32x4* b4 = reinterpret_cast<f32x4*>(s2);
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n_vec; i += stride) {
    f32x4 acc;
    if (NS > 0) {
      f32x4 g[NS > 0 ? NS : 1];
#pragma unroll
      for (int w = 0; w < NS; ++w) g[w] = ld_stream(reinterpret_cast<const f32x4*>(t.p[w]) + i);
      acc = t.w[0] * g[0];
#pragma unroll
      for (int w = 1; w < NS; ++w) acc = fma4(t.w[w], g[w], acc);
    } else {
      f32x4 g = ld_stream(reinterpret_cast<const f32x4*>(t.p[0]) + i);
      acc = t.w[0] * g;
      for (int w = 1; w < n; ++w) {
        g = ld_stream(reinterpret_cast<const f32x4*>(t.p[w]) + i);
        acc = fma4(t.w[w], g, acc);
      }
    }
    f32x4 pp = p4[i], aa = a4[i], bb = TWO ? b4[i] : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    float x0 = pp.x, x1 = pp.y, x2 = pp.z, x3 = pp.w;
    float a0 = aa.x, a1 = aa.y, a2 = aa.z, a3 = aa.w;
    float b0 = bb.x, b1 = bb.y, b2 = bb.z, b3 = bb.w;
    rule_elem<RULE>(acc.x, x0, a0, b0, h);
    rule_elem<RULE>(acc.y, x1, a1, b1, h);
    rule_elem<RULE>(acc.z, x2, a2, b2, h);
    rule_elem<RULE>(acc.w, x3, a3, b3, h);
    p4[i] = f32x4{x0, x1, x2, x3};
    a4[i] = f32x4{a0, a1, a2, a3};
    if (TWO) b4[i] = f32x4{b0, b1, b2, b3};
    if (p_lp) {
      u32x2 q;
      q.x = pack_bf16x2(x0, x1);
      q.y = pack_bf16x2(x2, x3);
      reinterpret_cast<u32x2*>(p_lp)[i] = q;
    }
  }
  if (blockIdx.x == 0) {
    const int64_t e = (n_vec << 2) + threadIdx.x;
    if (threadIdx.x < 4 && e < len) {
      float acc = t.w[0] * reinterpret_cast<const float*>(t.p[0])[e];
      for (int w = 1; w < n; ++w) acc = fmaf(t.w[w], reinterpret_cast<const float*>(t.p[w])[e], acc);
      float pp = p[e], aa = s1[e], bb = TWO ? s2[e] : 0.0f;
      rule_elem<RULE>(acc, pp, aa, bb, h);
      p[e] = pp;
      s1[e] = aa;
      if (TWO) s2[e] = bb;
      if (p_lp) p_lp[e] = f32_to_bf16(pp);
    }
    if (threadIdx.x == 0 && loss_out) {
      float acc = t.w[0] * loss_in[0];
      for (int w = 1; w < n; ++w) acc = fmaf(t.w[w], loss_in[w], acc);
      loss_out[0] = acc;
    }
  }
}

// G = sum_w weight_w * grad_w ; (p, v) <- momentum update ; optional bf16 copy
// of p; optional weighted mean of n scalar losses.  NS > 0 fixes the number of
// gradient buffers at compile time so that all NS loads are issued together.
template <int NS>
__global__ __launch_bounds__(kBlock) void reduce_sgd_kernel(BufTable t, int n_dyn, int64_t len,
                                                            float* __restrict__ p,
                                                            float* __restrict__ v, float lr,
                                                            float m, float wd,
                                                            uint16_t* __restrict__ p_lp,
                                                            const float* __restrict__ loss_in,
                                                            float* __restrict__ loss_out) {
  const int n = NS > 0 ? NS : n_dyn;
  const int64_t n_vec = len >> 2;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  f32x4* p4 = reinterpret_cast<f32x4*>(p);
  f32x4* v4 = reinterpret_cast<f32x4*>(v);
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n_vec; i += stride) {
    f32x4 acc;
    if (NS > 0) {
      f32x4 g[NS > 0 ? NS : 1];
#pragma unroll
      for (int w = 0; w < NS; ++w) g[w] = ld_stream(reinterpret_cast<const f32x4*>(t.p[w]) + i);
      acc = t.w[0] * g[0];
#pragma unroll
      for (int w = 1; w < NS; ++w) acc = fma4(t.w[w], g[w], acc);
    } else {
      f32x4 g = ld_stream(reinterpret_cast<const f32x4*>(t.p[0]) + i);
      acc = t.w[0] * g;
      for (int w = 1; w < n; ++w) {
        g = ld_stream(reinterpret_cast<const f32x4*>(t.p[w]) + i);
        acc = fma4(t.w[w], g, acc);
      }
    }
    f32x4 pp = p4[i], vv = v4[i];
    {
      float a0 = pp.x, a1 = pp.y, a2 = pp.z, a3 = pp.w;
      float b0 = vv.x, b1 = vv.y, b2 = vv.z, b3 = vv.w;
      sgd_elem(acc.x, a0, b0, lr, m, wd);
      sgd_elem(acc.y, a1, b1, lr, m, wd);
      sgd_elem(acc.z, a2, b2, lr, m, wd);
      sgd_elem(acc.w, a3, b3, lr, m, wd);
      pp = f32x4{a0, a1, a2, a3};
      vv = f32x4{b0, b1, b2, b3};
    }
    p4[i] = pp;
    v4[i] = vv;
    if (p_lp) {
      u32x2 q;
      q.x = pack_bf16x2(pp.x, pp.y);
      q.y = pack_bf16x2(pp.z, pp.w);
      reinterpret_cast<u32x2*>(p_lp)[i] = q;
    }
  }
  if (blockIdx.x == 0) {
    // ragged tail (len % 4 elements) and the scalar loss
    const int64_t e = (n_vec << 2) + threadIdx.x;
    if (threadIdx.x < 4 && e < len) {
      float acc = t.w[0] * reinterpret_cast<const float*>(t.p[0])[e];
      for (int w = 1; w < n; ++w) acc = fmaf(t.w[w], reinterpret_cast<const float*>(t.p[w])[e], acc);
      float pp = p[e], vv = v[e];
      sgd_elem(acc, pp, vv, lr, m, wd);
      p[e] = pp;
      v[e] = vv;
      if (p_lp) p_lp[e] = f32_to_bf16(pp);
    }
    if (threadIdx.x == 0 && loss_out) {
      float acc = t.w[0] * loss_in[0];
      for (int w = 1; w < n; ++w) acc = fmaf(t.w[w], loss_in[w], acc);
      loss_out[0] = acc;
    }
  }
}

template <typename T>
struct Vec4 {};
template <>
struct Vec4<float> { using type = f32x4; };
template <>
struct Vec4<int32_t> { using type = i32x4; };

template <typename T, int OP>
__device__ __forceinline__ T fold(T a, T b) {
  if (OP == SYNK_SUM) return a + b;
  if (OP == SYNK_PROD) return a * b;
  if (OP == SYNK_MAX) return a > b ? a : b;
  return a < b ? a : b;  // SYNK_MIN
}

// out[i] = fold over buffers in order; MEAN is the weighted sum.
template <typename T, int OP>
// `out` may be bufs[0] (every thread reads its element of every buffer before it writes), so it
// carries no no-alias qualifier.
__global__ __launch_bounds__(kBlock) void reduce_kernel(BufTable t, int n, int64_t len, T* out) {
  using V = typename Vec4<T>::type;
  const int64_t n_vec = len >> 2;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n_vec; i += stride) {
    V a = __builtin_nontemporal_load(reinterpret_cast<const V*>(t.p[0]) + i);
    if (OP == SYNK_MEAN) {
      a.x = (T)(t.w[0] * (float)a.x); a.y = (T)(t.w[0] * (float)a.y);
      a.z = (T)(t.w[0] * (float)a.z); a.w = (T)(t.w[0] * (float)a.w);
    }
    for (int w = 1; w < n; ++w) {
      const V b = __builtin_nontemporal_load(reinterpret_cast<const V*>(t.p[w]) + i);
      if (OP == SYNK_MEAN) {
        a.x = (T)fmaf(t.w[w], (float)b.x, (float)a.x); a.y = (T)fmaf(t.w[w], (float)b.y, (float)a.y);
        a.z = (T)fmaf(t.w[w], (float)b.z, (float)a.z); a.w = (T)fmaf(t.w[w], (float)b.w, (float)a.w);
      } else {
        a.x = fold<T, OP>(a.x, b.x); a.y = fold<T, OP>(a.y, b.y);
        a.z = fold<T, OP>(a.z, b.z); a.w = fold<T, OP>(a.w, b.w);
      }
    }
    reinterpret_cast<V*>(out)[i] = a;
  }
  if (blockIdx.x == 0 && threadIdx.x < 4) {
    const int64_t e = (n_vec << 2) + threadIdx.x;
    if (e < len) {
      T a = reinterpret_cast<const T*>(t.p[0])[e];
      if (OP == SYNK_MEAN) a = (T)(t.w[0] * (float)a);
      for (int w = 1; w < n; ++w) {
        const T b = reinterpret_cast<const T*>(t.p[w])[e];
        if (OP == SYNK_MEAN) a = (T)fmaf(t.w[w], (float)b, (float)a);
        else a = fold<T, OP>(a, b);
      }
      out[e] = a;
    }
  }
}

// Same kernel for buffers that are only 4-byte aligned.
template <typename T, int OP>
__global__ __launch_bounds__(kBlock) void reduce_kernel_scalar(BufTable t, int n, int64_t len, T* out) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < len; e += stride) {
    T a = reinterpret_cast<const T*>(t.p[0])[e];
    if (OP == SYNK_MEAN) a = (T)(t.w[0] * (float)a);
    for (int w = 1; w < n; ++w) {
      const T b = reinterpret_cast<const T*>(t.p[w])[e];
      if (OP == SYNK_MEAN) a = (T)fmaf(t.w[w], (float)b, (float)a);
      else a = fold<T, OP>(a, b);
    }
    out[e] = a;
  }
}

// CONCAT: blockIdx.y = source buffer; 4-byte elements copied to their offset.
__global__ __launch_bounds__(kBlock) void concat_kernel(ConcatTable t, uint32_t* __restrict__ out) {
  const int b = blockIdx.y;
  const int64_t len = t.start[b + 1] - t.start[b];
  const uint32_t* src = t.src[b];
  uint32_t* dst = out + t.start[b];
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < len; e += stride) dst[e] = src[e];
}

__global__ __launch_bounds__(kBlock) void cast_bf16_kernel(const float* __restrict__ in,
                                                           uint16_t* __restrict__ out, int64_t len,
                                                           int vec_ok) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  const int64_t n_vec = vec_ok ? (len >> 2) : 0;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n_vec; i += stride) {
    const f32x4 a = reinterpret_cast<const f32x4*>(in)[i];
    u32x2 q;
    q.x = pack_bf16x2(a.x, a.y);
    q.y = pack_bf16x2(a.z, a.w);
    reinterpret_cast<u32x2*>(out)[i] = q;
  }
  for (int64_t e = (n_vec << 2) + (int64_t)blockIdx.x * kBlock + threadIdx.x; e < len; e += stride)
    out[e] = f32_to_bf16(in[e]);
}

template <typename T, int OP>
static int launch_reduce(const BufTable& t, int n, int64_t len, void* out, bool vec,
                         hipStream_t s) {
  if (vec)
    SYNK_LAUNCH_TIMED((reduce_kernel<T, OP>), dim3(stream_grid(len >> 2)), dim3(kBlock), 0, s, t, n,
                       len, reinterpret_cast<T*>(out));
  else
    SYNK_LAUNCH_TIMED((reduce_kernel_scalar<T, OP>), dim3(stream_grid(len)), dim3(kBlock), 0, s, t,
                       n, len, reinterpret_cast<T*>(out));
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

template <typename T>
static int dispatch_reduce(int op, const BufTable& t, int n, int64_t len, void* out, bool vec,
                           hipStream_t s) {
  switch (op) {
    case SYNK_SUM: return launch_reduce<T, SYNK_SUM>(t, n, len, out, vec, s);
    case SYNK_MAX: return launch_reduce<T, SYNK_MAX>(t, n, len, out, vec, s);
    case SYNK_MIN: return launch_reduce<T, SYNK_MIN>(t, n, len, out, vec, s);
    case SYNK_PROD: return launch_reduce<T, SYNK_PROD>(t, n, len, out, vec, s);
    default: return SYNK_ERR_OP;
  }
}

static int fill_weights(BufTable& t, int n, const float* weights) {
  for (int w = 0; w < n; ++w) t.w[w] = weights ? weights[w] : 1.0f / (float)n;
  return SYNK_OK;
}

}  // namespace synk

using namespace synk;

extern "C" int synk_reduce_buffers(const void* const* bufs, int n, int64_t len, int dtype, int op,
                                   const float* weights, const int64_t* lens, void* out,
                                   void* stream) {
  if (!bufs || !out) return SYNK_ERR_NULL;
  if (n < 1 || n > SYNK_MAX_WORKERS) return SYNK_ERR_SHAPE;
  if (dtype != SYNK_F32 && dtype != SYNK_I32) return SYNK_ERR_DTYPE;
  if (op < SYNK_SUM || op > SYNK_CONCAT) return SYNK_ERR_OP;
  if (op == SYNK_MEAN && dtype != SYNK_F32) return SYNK_ERR_OP;
  if (weights && op != SYNK_MEAN) return SYNK_ERR_OP;
  if (!aligned_to(out, 4)) return SYNK_ERR_ALIGN;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);

  if (op == SYNK_CONCAT) {
    if (!lens) return SYNK_ERR_NULL;
    ConcatTable ct;
    ct.start[0] = 0;
    int64_t longest = 0;
    for (int w = 0; w < n; ++w) {
      if (lens[w] < 0) return SYNK_ERR_SHAPE;
      if (lens[w] > 0 && !bufs[w]) return SYNK_ERR_NULL;
      if (!aligned_to(bufs[w], 4)) return SYNK_ERR_ALIGN;
      ct.src[w] = reinterpret_cast<const uint32_t*>(bufs[w]);
      ct.start[w + 1] = ct.start[w] + lens[w];
      if (lens[w] > longest) longest = lens[w];
    }
    if (longest == 0) return SYNK_OK;
    int gx = stream_grid(longest);
    if (gx > 1024) gx = 1024;
    hipLaunchKernelGGL(concat_kernel, dim3(gx, n), dim3(kBlock), 0, s, ct,
                       reinterpret_cast<uint32_t*>(out));
    SYNK_LAUNCH_CHECK();
    return SYNK_OK;
  }

  if (len < 0) return SYNK_ERR_SHAPE;
  BufTable t;
  bool vec = aligned_to(out, 16);
  for (int w = 0; w < n; ++w) {
    if (!bufs[w]) return SYNK_ERR_NULL;
    if (!aligned_to(bufs[w], 4)) return SYNK_ERR_ALIGN;
    vec = vec && aligned_to(bufs[w], 16);
    t.p[w] = bufs[w];
  }
  fill_weights(t, n, weights);
  if (len == 0) return SYNK_OK;
  if (op == SYNK_MEAN) return launch_reduce<float, SYNK_MEAN>(t, n, len, out, vec, s);
  if (dtype == SYNK_F32) return dispatch_reduce<float>(op, t, n, len, out, vec, s);
  return dispatch_reduce<int32_t>(op, t, n, len, out, vec, s);
}

static int launch_reduce_sgd(const BufTable& t, int n, int64_t len, float* p, float* v, float lr,
                             float m, float wd, void* p_lp, const float* loss_in, float* loss_out,
                             hipStream_t s) {
  const dim3 grid(stream_grid(len >> 2)), block(kBlock);
  uint16_t* lp = reinterpret_cast<uint16_t*>(p_lp);
#define SYNK_RS(NS)                                                                              \
  SYNK_LAUNCH_TIMED((reduce_sgd_kernel<NS>), grid, block, 0, s, t, n, len, p, v, lr, m, wd, lp,  \
                     loss_in, loss_out)
  switch (n) {
    case 1: SYNK_RS(1); break;
    case 2: SYNK_RS(2); break;
    case 4: SYNK_RS(4); break;
    case 8: SYNK_RS(8); break;
    default: SYNK_RS(0); break;
  }
#undef SYNK_RS
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

extern "C" int synk_reduce_sgd_update(const float* const* grads, int n, int64_t len,
                                      const float* weights, float* p, float* v, float lr,
                                      float momentum, float weight_decay, void* p_lp,
                                      const float* loss_in, float* loss_out, void* stream) {
  if (!grads || !p || !v) return SYNK_ERR_NULL;
  if ((loss_in == nullptr) != (loss_out == nullptr)) return SYNK_ERR_NULL;
  if (n < 1 || n > SYNK_MAX_WORKERS || len < 0) return SYNK_ERR_SHAPE;
  if (!aligned_to(p, 16) || !aligned_to(v, 16) || (p_lp && !aligned_to(p_lp, 8)))
    return SYNK_ERR_ALIGN;
  BufTable t;
  for (int w = 0; w < n; ++w) {
    if (!grads[w]) return SYNK_ERR_NULL;
    if (!aligned_to(grads[w], 16)) return SYNK_ERR_ALIGN;
    t.p[w] = grads[w];
  }
  fill_weights(t, n, weights);
  if (len == 0 && !loss_out) return SYNK_OK;
  return launch_reduce_sgd(t, n, len, p, v, lr, momentum, weight_decay, p_lp, loss_in, loss_out,
                           reinterpret_cast<hipStream_t>(stream));
}

template <int RULE>
static int launch_reduce_update(const BufTable& t, int n, int64_t len, float* p, float* s1, float* s2,
                                const RuleParams& h, void* p_lp, const float* loss_in,
                                float* loss_out, hipStream_t s) {
  const dim3 grid(stream_grid(len >> 2)), block(kBlock);
  uint16_t* lp = reinterpret_cast<uint16_t*>(p_lp);
#define SYNK_RU(NS)                                                                                \
  SYNK_LAUNCH_TIMED((reduce_update_kernel<NS, RULE>), grid, block, 0, s, t, n, len, p, s1, s2, h,  \
                     lp, loss_in, loss_out)
  switch (n) {
    case 1: SYNK_RU(1); break;
    case 2: SYNK_RU(2); break;
    case 4: SYNK_RU(4); break;
    case 8: SYNK_RU(8); break;
    default: SYNK_RU(0); break;
  }
#undef SYNK_RU
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

extern "C" int synk_reduce_update(const synk_update_desc* u, const float* const* grads, int n,
                                  int64_t len, const float* weights, float* p, float* s1, float* s2,
                                  void* p_lp, const float* loss_in, float* loss_out, void* stream) {
  if (!u || !grads || !p || !s1) return SYNK_ERR_NULL;
  if (u->rule < SYNK_RULE_MOMENTUM || u->rule > SYNK_RULE_ADAM) return SYNK_ERR_OP;
  if (u->rule == SYNK_RULE_ADAM && !s2) return SYNK_ERR_NULL;
  if ((loss_in == nullptr) != (loss_out == nullptr)) return SYNK_ERR_NULL;
  if (n < 1 || n > SYNK_MAX_WORKERS || len < 0) return SYNK_ERR_SHAPE;
  if (u->rule == SYNK_RULE_ADAM &&
      (u->step < 1 || !(u->beta1 >= 0.0f && u->beta1 < 1.0f) || !(u->beta2 >= 0.0f && u->beta2 < 1.0f)))
    return SYNK_ERR_SHAPE;
  if (!aligned_to(p, 16) || !aligned_to(s1, 16) || (s2 && !aligned_to(s2, 16)) ||
      (p_lp && !aligned_to(p_lp, 8)))
    return SYNK_ERR_ALIGN;
  BufTable t;
  for (int w = 0; w < n; ++w) {
    if (!grads[w]) return SYNK_ERR_NULL;
    if (!aligned_to(grads[w], 16)) return SYNK_ERR_ALIGN;
    t.p[w] = grads[w];
  }
  fill_weights(t, n, weights);
  if (len == 0 && !loss_out) return SYNK_OK;
  RuleParams h;
  h.lr = u->lr;
  h.wd = u->weight_decay;
  h.eps = u->eps;
  h.b2 = u->beta2;
  h.a_t = 0.0f;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  switch (u->rule) {
    case SYNK_RULE_MOMENTUM:
      h.m = u->momentum;
      return launch_reduce_update<SYNK_RULE_MOMENTUM>(t, n, len, p, s1, s2, h, p_lp, loss_in, loss_out, s);
    case SYNK_RULE_NESTEROV:
      h.m = u->momentum;
      return launch_reduce_update<SYNK_RULE_NESTEROV>(t, n, len, p, s1, s2, h, p_lp, loss_in, loss_out, s);
    case SYNK_RULE_RMSPROP:
      h.m = u->rho;
      return launch_reduce_update<SYNK_RULE_RMSPROP>(t, n, len, p, s1, s2, h, p_lp, loss_in, loss_out, s);
    default: {
      h.m = u->beta1;
      // the bias-corrected step size, once per call on the host in double precision
      const double b1t = pow((double)u->beta1, (double)u->step), b2t = pow((double)u->beta2, (double)u->step);
      h.a_t = (float)((double)u->lr * sqrt(1.0 - b2t) / (1.0 - b1t));
      return launch_reduce_update<SYNK_RULE_ADAM>(t, n, len, p, s1, s2, h, p_lp, loss_in, loss_out, s);
    }
  }
}

extern "C" int synk_sgd_update(float* p, float* v, const float* g, int64_t len, float lr,
                               float momentum, float weight_decay, void* p_lp, void* stream) {
  if (!p || !v || !g) return SYNK_ERR_NULL;
  if (len < 0) return SYNK_ERR_SHAPE;
  if (!aligned_to(p, 16) || !aligned_to(v, 16) || !aligned_to(g, 16) ||
      (p_lp && !aligned_to(p_lp, 8)))
    return SYNK_ERR_ALIGN;
  if (len == 0) return SYNK_OK;
  BufTable t;
  t.p[0] = g;
  t.w[0] = 1.0f;
  return launch_reduce_sgd(t, 1, len, p, v, lr, momentum, weight_decay, p_lp, nullptr, nullptr,
                           reinterpret_cast<hipStream_t>(stream));
}

extern "C" int synk_cast_bf16(const float* in, void* out, int64_t len, void* stream) {
  if (!in || !out) return SYNK_ERR_NULL;
  if (len < 0) return SYNK_ERR_SHAPE;
  if (!aligned_to(in, 4) || !aligned_to(out, 2)) return SYNK_ERR_ALIGN;
  if (len == 0) return SYNK_OK;
  const int vec_ok = aligned_to(in, 16) && aligned_to(out, 8);
  hipLaunchKernelGGL(cast_bf16_kernel, dim3(stream_grid(len >> 2)), dim3(kBlock), 0,
                     reinterpret_cast<hipStream_t>(stream), in,
                     reinterpret_cast<uint16_t*>(out), len, vec_ok);
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}
