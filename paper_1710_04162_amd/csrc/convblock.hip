// A second sliced gradient function (Sec. 3.3 step 1 evaluated as Sec. 3.2 /
// 5.1 describe): one 3x3 convolution + batch-normalisation + ReLU block of the
// kind the scaling study's network is built from (Sec. 6), closed by global
// average pooling, one affine layer and softmax cross-entropy.
//
// One call covers every worker and every slice.  A slice is one call of the
// function (Sec. 5.1), so the batch statistics are per slice; a slice's images
// carry the weight that the aggregation op gives the slice, which makes every
// sum over a worker's images the in-place aggregation of its slice results.
//
// Images are channels-last (a gathered row is H*W*C_in values), so the
// convolution is a product [pixels x 9 C_in] . [9 C_in x C_out] whose left
// operand is never built: for one tap, the row of a pixel is the C_in vector
// of its shifted neighbour (or zero outside the image), which is one
// wave-uniform offset away from the pixel's own address.  Both contractions
// (forward, weight gradient) run on the matrix cores (MFMA 32x32x16 bf16 or
// 32x32x2 fp32, fp32 accumulators) out of LDS; everything between them is
// fp32 streaming work over z.
//
// No floating-point atomics: every sum has a fixed order.
#include <math.h>

#include "common.h"

namespace synk {

typedef uint16_t bf16_t;                                     // raw bfloat16 bits
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));   // MFMA operand type

namespace {

template <typename T> struct EL;
template <> struct EL<float> { static constexpr int V = 4; };    // elements per 16-byte vector
template <> struct EL<bf16_t> { static constexpr int V = 8; };

constexpr int kThreads = 256;
constexpr int kChunkRows = 256;     // pixels of one image handled by one workgroup of the streaming kernels
constexpr int kMaxCout = 512;
constexpr int kMaxClasses = 4096;

struct ConvShape {
  int H, W, cin, cout, classes, HW;
  int n_workers, n_slices, grad_op;
  int n_chunks;      // ceil(HW / kChunkRows)
  int total_images;
  float eps;
};

struct WorkerTable {
  const void* x[SYNK_MAX_WORKERS];
  const int32_t* y[SYNK_MAX_WORKERS];
  float* grad[SYNK_MAX_WORKERS];
  int32_t rows[SYNK_MAX_WORKERS];
  int32_t row_off[SYNK_MAX_WORKERS + 1];   // images held by the workers before w
};

// Offsets into the flat parameter / gradient array.
struct ParamOff {
  int64_t wc, gamma, beta, wf, bf, total;
};
__host__ __device__ inline ParamOff param_off(int cin, int cout, int classes) {
  ParamOff o;
  o.wc = 0;
  o.gamma = (int64_t)9 * cin * cout;
  o.beta = o.gamma + cout;
  o.wf = o.beta + cout;
  o.bf = o.wf + (int64_t)cout * classes;
  o.total = o.bf + classes;
  return o;
}

__device__ __forceinline__ void slice_bounds(int rows, int parts, int s, int* start, int* size) {
  const int base = rows / parts, extra = rows % parts;
  *size = base + (s < extra ? 1 : 0);
  *start = base * s + (s < extra ? s : extra);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 a;
#pragma unroll
  for (int v = 0; v < 16; ++v) a[v] = 0.0f;
  return a;
}

// One 16-byte operand pair -> the MFMAs it feeds.  bf16: 8 contraction steps in
// one instruction.  fp32: lane group g holds steps 4g..4g+3 of an 8-step run;
// instruction j takes element j of both operands (any pairing of steps works
// as long as both operands use the same one).
__device__ __forceinline__ f32x16 mma(bf16_t, u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                 0, 0, 0);
}
__device__ __forceinline__ f32x16 mma(float, u32x4 a, u32x4 b, f32x16 c) {
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
  return c;
}

// ------------------------------------------------------------ weight layout
// wmat[o][k] = (T) Wc[k][o], k = tap*C_in + c: the convolution's right operand
// with its contraction index contiguous, rounded to the compute type.
template <typename T>
__global__ __launch_bounds__(kThreads) void conv_weight_kernel(const float* __restrict__ params, T* __restrict__ wmat,
                                                               int K, int cout) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= (int64_t)K * cout) return;
  const int o = (int)(i / K), k = (int)(i - (int64_t)o * K);
  const float v = params[(int64_t)k * cout + o];
  if (sizeof(T) == 2) reinterpret_cast<uint16_t*>(wmat)[i] = f32_to_bf16(v);
  else reinterpret_cast<float*>(wmat)[i] = v;
}

// ------------------------------------------------------------ forward conv
// z[pixel][o] for a 128-pixel x 64-channel tile of one (worker, slice) unit.
// LDS rows are 8 vectors of 16 bytes (64 bf16 or 32 fp32 contraction steps of
// one tap) plus 16 bytes of padding; two buffers, one barrier per k-tile.
constexpr int kFwdBM = 128, kFwdBN = 64, kLdsRow = 144;

template <typename T>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_fwd_kernel(WorkerTable tab, ConvShape sh,
                                                                  const T* __restrict__ wmat,
                                                                  float* __restrict__ z) {
  constexpr int V = EL<T>::V, BK = 8 * V;
  __shared__ __attribute__((aligned(16))) char smem[2][(kFwdBM + kFwdBN) * kLdsRow];

  const int unit = blockIdx.z;
  const int w = unit / sh.n_slices, s = unit - w * sh.n_slices;
  int img0, nimg;
  slice_bounds(tab.rows[w], sh.n_slices, s, &img0, &nimg);
  const int M = nimg * sh.HW;
  const int m0 = blockIdx.x * kFwdBM;
  if (m0 >= M) return;
  const int n0 = blockIdx.y * kFwdBN;
  const T* __restrict__ xw = reinterpret_cast<const T*>(tab.x[w]) + (int64_t)img0 * sh.HW * sh.cin;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int xi = lane & 31, gk = lane >> 5, wm = wv >> 1, wn = wv & 1;
  const int kv = tid & 7, ur = tid >> 3;   // this thread's vector in a row, and its row within a group of 32

  // left operand: 4 pixel rows per thread; bit 4 = row exists, bits 0..3 = it
  // has a neighbour above / below / left / right
  const T* arow[4];
  uint32_t amask[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int q = m0 + it * 32 + ur;
    arow[it] = xw;
    amask[it] = 0u;
    if (q < M) {
      const int rem = q % sh.HW;
      const int h = rem / sh.W, ww = rem - h * sh.W;
      arow[it] = xw + (int64_t)q * sh.cin;
      amask[it] = 16u | (h > 0 ? 1u : 0u) | (h < sh.H - 1 ? 2u : 0u) | (ww > 0 ? 4u : 0u) | (ww < sh.W - 1 ? 8u : 0u);
    }
  }
  const int K = 9 * sh.cin;
  const T* brow[2];
  bool bok[2];
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int o = n0 + it * 32 + ur;
    bok[it] = o < sh.cout;
    brow[it] = wmat + (int64_t)(bok[it] ? o : 0) * K;
  }

  const int cpt = (sh.cin + BK - 1) / BK;   // k-tiles per tap
  const int n_kt = 9 * cpt;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  u32x4 ra[4], rb[2];

  auto gload = [&](int t) {
    const int tap = t / cpt;
    const int c = (t - tap * cpt) * BK + kv * V;
    const int kh = tap / 3, kw = tap - kh * 3;
    const bool cok = c < sh.cin;
    const uint32_t need = 16u | (kh == 0 ? 1u : 0u) | (kh == 2 ? 2u : 0u) | (kw == 0 ? 4u : 0u) | (kw == 2 ? 8u : 0u);
    const int delta = ((kh - 1) * sh.W + (kw - 1)) * sh.cin + c;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const bool ok = cok && ((amask[it] & need) == need);
      const T* p = ok ? arow[it] + delta : xw;
      const u32x4 v = *reinterpret_cast<const u32x4*>(p);
      ra[it] = ok ? v : zero;
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const bool ok = cok && bok[it];
      const T* p = ok ? brow[it] + tap * sh.cin + c : wmat;
      const u32x4 v = *reinterpret_cast<const u32x4*>(p);
      rb[it] = ok ? v : zero;
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int it = 0; it < 4; ++it)
      *reinterpret_cast<u32x4*>(&smem[buf][(it * 32 + ur) * kLdsRow + kv * 16]) = ra[it];
#pragma unroll
    for (int it = 0; it < 2; ++it)
      *reinterpret_cast<u32x4*>(&smem[buf][(kFwdBM + it * 32 + ur) * kLdsRow + kv * 16]) = rb[it];
  };

  f32x16 acc[2] = {zero16(), zero16()};
  gload(0);
  lstore(0);
  __syncthreads();
  for (int t = 0; t < n_kt; ++t) {
    if (t + 1 < n_kt) gload(t + 1);
    const char* A = smem[t & 1] + (wm * 64 + xi) * kLdsRow + gk * 16;
    const char* B = smem[t & 1] + (kFwdBM + wn * 32 + xi) * kLdsRow + gk * 16;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const u32x4 a0 = *reinterpret_cast<const u32x4*>(A + kk * 32);
      const u32x4 a1 = *reinterpret_cast<const u32x4*>(A + 32 * kLdsRow + kk * 32);
      const u32x4 b = *reinterpret_cast<const u32x4*>(B + kk * 32);
      acc[0] = mma(T(), a0, b, acc[0]);
      acc[1] = mma(T(), a1, b, acc[1]);
    }
    if (t + 1 < n_kt) lstore((t + 1) & 1);
    __syncthreads();
  }

  // accumulator v of lane (xi, gk) is row gk*4 + (v>>2)*8 + (v&3), column xi
  float* __restrict__ zu = z + ((int64_t)(tab.row_off[w] + img0) * sh.HW) * sh.cout;
  const int col = n0 + wn * 32 + xi;
  if (col < sh.cout) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r0 = m0 + wm * 64 + i * 32 + gk * 4;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = r0 + (v >> 2) * 8 + (v & 3);
        if (row < M) zu[(int64_t)row * sh.cout + col] = acc[i][v];
      }
    }
  }
}

// -------------------------------------------------- streaming passes over z
// A workgroup takes up to kChunkRows pixels of one image and all channels:
// thread = (4 consecutive channels, row group); row groups are folded through
// LDS in a fixed order.
struct Chunk {
  int w, unit, img, chunk, nrows, cnt_unit;
  int64_t row0;        // first pixel row in the packed z / dz arrays
  int c4, rg, n_rg;    // this thread's channel quad and row group; number of row groups
  bool active;
};

__device__ __forceinline__ Chunk chunk_of(const WorkerTable& tab, const ConvShape& sh) {
  Chunk c;
  c.img = blockIdx.x / sh.n_chunks;
  c.chunk = blockIdx.x - c.img * sh.n_chunks;
  int w = 0;
  while (w + 1 < sh.n_workers && tab.row_off[w + 1] <= c.img) ++w;
  c.w = w;
  int s;
  int64_t start;
  share_of(tab.rows[w], sh.n_slices, c.img - tab.row_off[w], &s, &start);
  c.unit = w * sh.n_slices + s;
  int s0, sn;
  slice_bounds(tab.rows[w], sh.n_slices, s, &s0, &sn);
  c.cnt_unit = sn * sh.HW;
  const int r0 = c.chunk * kChunkRows;
  c.nrows = min(kChunkRows, sh.HW - r0);
  c.row0 = (int64_t)c.img * sh.HW + r0;
  const int C4 = sh.cout / 4;
  c.n_rg = kThreads / C4;
  c.c4 = threadIdx.x % C4;
  c.rg = threadIdx.x / C4;
  c.active = c.rg < c.n_rg;
  return c;
}

// Sum over row groups of one float4 per thread, for NQ quantities at once:
// red[q][rg][channel].  Returns, for channel ch (ch < cout, called by threads
// ch = tid, tid + 256, ...), the sums in fixed row-group order.
template <int NQ>
__device__ __forceinline__ void fold_store(float* red, const Chunk& c, int cout, const f32x4 (&v)[NQ]) {
  if (c.active) {
#pragma unroll
    for (int q = 0; q < NQ; ++q)
      *reinterpret_cast<f32x4*>(red + ((q * c.n_rg + c.rg) * cout + c.c4 * 4)) = v[q];
  }
}
__device__ __forceinline__ float fold_sum(const float* red, int q, int n_rg, int cout, int ch) {
  float s = 0.0f;
  for (int r = 0; r < n_rg; ++r) s += red[(q * n_rg + r) * cout + ch];
  return s;
}

// Per (image, chunk, channel): mean and centred sum of squares of z, computed
// about the chunk's first row so that nothing cancels.
__global__ __launch_bounds__(kThreads) void bn_stats_chunk_kernel(WorkerTable tab, ConvShape sh,
                                                                  const float* __restrict__ z,
                                                                  float* __restrict__ statp) {
  __shared__ __attribute__((aligned(16))) float red[2 * kThreads * 4];
  const Chunk c = chunk_of(tab, sh);
  f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  if (c.active) {
    const float* p = z + c.row0 * sh.cout + c.c4 * 4;
    const f32x4 k = *reinterpret_cast<const f32x4*>(p);
    for (int r = c.rg; r < c.nrows; r += c.n_rg) {
      const f32x4 d = *reinterpret_cast<const f32x4*>(p + (int64_t)r * sh.cout) - k;
      acc[0] += d;
      acc[1] += d * d;
    }
  }
  fold_store<2>(red, c, sh.cout, acc);
  __syncthreads();
  const float n = (float)c.nrows;
  for (int ch = threadIdx.x; ch < sh.cout; ch += kThreads) {
    const float s1 = fold_sum(red, 0, c.n_rg, sh.cout, ch), s2 = fold_sum(red, 1, c.n_rg, sh.cout, ch);
    const float k = z[c.row0 * sh.cout + ch];
    float* o = statp + ((int64_t)blockIdx.x * sh.cout + ch) * 2;
    o[0] = k + s1 / n;
    o[1] = fmaxf(s2 - s1 * s1 / n, 0.0f);
  }
}

// Per (unit, channel): the chunks' (count, mean, centred sum of squares) are
// merged pairwise in image / chunk order -> mu and 1 / sqrt(var + eps).
__global__ __launch_bounds__(kThreads) void bn_stats_unit_kernel(WorkerTable tab, ConvShape sh,
                                                                 const float* __restrict__ statp,
                                                                 float* __restrict__ mu, float* __restrict__ rstd) {
  const int unit = blockIdx.x;
  const int w = unit / sh.n_slices, s = unit - w * sh.n_slices;
  int img0, nimg;
  slice_bounds(tab.rows[w], sh.n_slices, s, &img0, &nimg);
  img0 += tab.row_off[w];
  for (int ch = threadIdx.x; ch < sh.cout; ch += kThreads) {
    float na = 0.0f, mean = 0.0f, m2 = 0.0f;
    for (int i = 0; i < nimg; ++i) {
      for (int k = 0; k < sh.n_chunks; ++k) {
        const float* p = statp + (((int64_t)(img0 + i) * sh.n_chunks + k) * sh.cout + ch) * 2;
        const float nb = (float)min(kChunkRows, sh.HW - k * kChunkRows);
        const float d = p[0] - mean, nn = na + nb;
        mean += d * (nb / nn);
        m2 += p[1] + d * d * (na * nb / nn);
        na = nn;
      }
    }
    mu[(int64_t)unit * sh.cout + ch] = mean;
    rstd[(int64_t)unit * sh.cout + ch] = nimg > 0 ? 1.0f / sqrtf(m2 / na + sh.eps) : 0.0f;
  }
}

// Per (image, chunk, channel): sum over the chunk's pixels of
// relu(gamma * xhat + beta).
__global__ __launch_bounds__(kThreads) void bn_relu_pool_kernel(WorkerTable tab, ConvShape sh,
                                                                const float* __restrict__ params,
                                                                const float* __restrict__ z,
                                                                const float* __restrict__ mu,
                                                                const float* __restrict__ rstd,
                                                                float* __restrict__ poolp) {
  __shared__ __attribute__((aligned(16))) float red[kThreads * 4];
  const Chunk c = chunk_of(tab, sh);
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  f32x4 acc[1] = {{0.f, 0.f, 0.f, 0.f}};
  if (c.active) {
    f32x4 g, b, m, rs;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      g[e] = params[po.gamma + c.c4 * 4 + e];
      b[e] = params[po.beta + c.c4 * 4 + e];
    }
    m = *reinterpret_cast<const f32x4*>(mu + (int64_t)c.unit * sh.cout + c.c4 * 4);
    rs = *reinterpret_cast<const f32x4*>(rstd + (int64_t)c.unit * sh.cout + c.c4 * 4);
    const float* p = z + c.row0 * sh.cout + c.c4 * 4;
    for (int r = c.rg; r < c.nrows; r += c.n_rg) {
      const f32x4 zz = *reinterpret_cast<const f32x4*>(p + (int64_t)r * sh.cout);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[0][e] += fmaxf(g[e] * ((zz[e] - m[e]) * rs[e]) + b[e], 0.0f);
    }
  }
  fold_store<1>(red, c, sh.cout, acc);
  __syncthreads();
  for (int ch = threadIdx.x; ch < sh.cout; ch += kThreads)
    poolp[(int64_t)blockIdx.x * sh.cout + ch] = fold_sum(red, 0, c.n_rg, sh.cout, ch);
}

// ------------------------------------------------------------------- head
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

// One workgroup per image: pooled features, logits, loss, d loss / d logits
// (scaled by the image's weight in its worker's aggregate) and d loss / d p.
// The image weight is 1/|R_w| for MEAN (slice weight |R_s|/|R_w| times the
// slice mean's 1/|R_s|) and 1/|R_s| for SUM.
__global__ __launch_bounds__(kThreads) void head_image_kernel(WorkerTable tab, ConvShape sh,
                                                              const float* __restrict__ params,
                                                              const float* __restrict__ poolp,
                                                              float* __restrict__ pooled,
                                                              float* __restrict__ dlogits,
                                                              float* __restrict__ dpooled,
                                                              float* __restrict__ row_loss) {
  __shared__ float sp[kMaxCout];
  __shared__ float sl[kMaxClasses];
  __shared__ float sred[8];
  const int img = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int w = 0;
  while (w + 1 < sh.n_workers && tab.row_off[w + 1] <= img) ++w;
  const int j = img - tab.row_off[w];
  int s;
  int64_t start;
  share_of(tab.rows[w], sh.n_slices, j, &s, &start);
  int s0, sn;
  slice_bounds(tab.rows[w], sh.n_slices, s, &s0, &sn);
  const float scale = sh.grad_op == SYNK_MEAN ? 1.0f / (float)tab.rows[w] : 1.0f / (float)sn;
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  const float* __restrict__ Wf = params + po.wf;

  for (int ch = tid; ch < sh.cout; ch += kThreads) {
    float a = 0.0f;
    for (int k = 0; k < sh.n_chunks; ++k) a += poolp[((int64_t)img * sh.n_chunks + k) * sh.cout + ch];
    a /= (float)sh.HW;
    sp[ch] = a;
    pooled[(int64_t)img * sh.cout + ch] = a;
  }
  __syncthreads();

  float mx = -INFINITY;
  for (int k = tid; k < sh.classes; k += kThreads) {
    float a = params[po.bf + k];
    for (int ch = 0; ch < sh.cout; ++ch) a = fmaf(sp[ch], Wf[(int64_t)ch * sh.classes + k], a);
    sl[k] = a;
    mx = fmaxf(mx, a);
  }
  mx = wave_max(mx);
  if (lane == 0) sred[wv] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(sred[0], sred[1]), fmaxf(sred[2], sred[3]));
  float se = 0.0f;
  for (int k = tid; k < sh.classes; k += kThreads) se += expf(sl[k] - mx);
  se = wave_sum(se);
  if (lane == 0) sred[4 + wv] = se;
  __syncthreads();
  se = (sred[4] + sred[5]) + (sred[6] + sred[7]);
  const int y = tab.y[w][j];
  const bool yok = y >= 0 && y < sh.classes;
  if (tid == 0) row_loss[img] = (mx + logf(se) - (yok ? sl[y] : 0.0f)) * scale;
  __syncthreads();   // sl[y] read before sl is overwritten
  const float inv = 1.0f / se;
  for (int k = tid; k < sh.classes; k += kThreads) {
    const float d = (expf(sl[k] - mx) * inv - ((yok && k == y) ? 1.0f : 0.0f)) * scale;
    sl[k] = d;
    dlogits[(int64_t)img * sh.classes + k] = d;
  }
  __syncthreads();
  for (int ch = wv; ch < sh.cout; ch += kThreads / 64) {
    float a = 0.0f;
    for (int k = lane; k < sh.classes; k += 64) a = fmaf(sl[k], Wf[(int64_t)ch * sh.classes + k], a);
    a = wave_sum(a);
    if (lane == 0) dpooled[(int64_t)img * sh.cout + ch] = a;
  }
}

// Per worker and class k: dWf[:, k], dbf[k] over the worker's images in image
// order; workgroup (0, w) also folds the image losses into loss[w].
__global__ __launch_bounds__(kThreads) void head_worker_kernel(WorkerTable tab, ConvShape sh,
                                                               const float* __restrict__ pooled,
                                                               const float* __restrict__ dlogits,
                                                               const float* __restrict__ row_loss,
                                                               float* __restrict__ loss) {
  const int w = blockIdx.y, k = blockIdx.x * kThreads + threadIdx.x;
  const int i0 = tab.row_off[w], n = tab.rows[w];
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  float* __restrict__ g = tab.grad[w];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    float a = 0.0f;
    for (int i = 0; i < n; ++i) a += row_loss[i0 + i];
    loss[w] = a;
  }
  if (k >= sh.classes) return;
  float b = 0.0f;
  for (int i = 0; i < n; ++i) b += dlogits[(int64_t)(i0 + i) * sh.classes + k];
  g[po.bf + k] = b;
  for (int ch = 0; ch < sh.cout; ++ch) {
    float a = 0.0f;
    for (int i = 0; i < n; ++i)
      a = fmaf(pooled[(int64_t)(i0 + i) * sh.cout + ch], dlogits[(int64_t)(i0 + i) * sh.classes + k], a);
    g[po.wf + (int64_t)ch * sh.classes + k] = a;
  }
}

// ------------------------------------------------------ batch-norm backward
// dy = (dp / HW) [gamma*xhat + beta > 0].  Per (image, chunk, channel): sum of
// dy and of dy * xhat.
__global__ __launch_bounds__(kThreads) void bn_bwd_chunk_kernel(WorkerTable tab, ConvShape sh,
                                                                const float* __restrict__ params,
                                                                const float* __restrict__ z,
                                                                const float* __restrict__ mu,
                                                                const float* __restrict__ rstd,
                                                                const float* __restrict__ dpooled,
                                                                float* __restrict__ bwdp) {
  __shared__ __attribute__((aligned(16))) float red[2 * kThreads * 4];
  const Chunk c = chunk_of(tab, sh);
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  if (c.active) {
    f32x4 g, b, m, rs, da;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      g[e] = params[po.gamma + c.c4 * 4 + e];
      b[e] = params[po.beta + c.c4 * 4 + e];
      da[e] = dpooled[(int64_t)c.img * sh.cout + c.c4 * 4 + e] / (float)sh.HW;
    }
    m = *reinterpret_cast<const f32x4*>(mu + (int64_t)c.unit * sh.cout + c.c4 * 4);
    rs = *reinterpret_cast<const f32x4*>(rstd + (int64_t)c.unit * sh.cout + c.c4 * 4);
    const float* p = z + c.row0 * sh.cout + c.c4 * 4;
    for (int r = c.rg; r < c.nrows; r += c.n_rg) {
      const f32x4 zz = *reinterpret_cast<const f32x4*>(p + (int64_t)r * sh.cout);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float xh = (zz[e] - m[e]) * rs[e];
        const float dy = (g[e] * xh + b[e] > 0.0f) ? da[e] : 0.0f;
        acc[0][e] += dy;
        acc[1][e] += dy * xh;
      }
    }
  }
  fold_store<2>(red, c, sh.cout, acc);
  __syncthreads();
  for (int ch = threadIdx.x; ch < sh.cout; ch += kThreads) {
    float* o = bwdp + ((int64_t)blockIdx.x * sh.cout + ch) * 2;
    o[0] = fold_sum(red, 0, c.n_rg, sh.cout, ch);
    o[1] = fold_sum(red, 1, c.n_rg, sh.cout, ch);
  }
}

// Per worker and channel: the slices' sums in slice / image / chunk order ->
// each slice's means (for dz) and the worker's d gamma, d beta.
__global__ __launch_bounds__(kThreads) void bn_bwd_worker_kernel(WorkerTable tab, ConvShape sh,
                                                                 const float* __restrict__ bwdp,
                                                                 float* __restrict__ bmean) {
  const int w = blockIdx.x;
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  float* __restrict__ g = tab.grad[w];
  for (int ch = threadIdx.x; ch < sh.cout; ch += kThreads) {
    float gb = 0.0f, gg = 0.0f;
    for (int s = 0; s < sh.n_slices; ++s) {
      int img0, nimg;
      slice_bounds(tab.rows[w], sh.n_slices, s, &img0, &nimg);
      img0 += tab.row_off[w];
      float sb = 0.0f, sg = 0.0f;
      for (int i = 0; i < nimg; ++i)
        for (int k = 0; k < sh.n_chunks; ++k) {
          const float* p = bwdp + (((int64_t)(img0 + i) * sh.n_chunks + k) * sh.cout + ch) * 2;
          sb += p[0];
          sg += p[1];
        }
      const float cnt = (float)(nimg * sh.HW);
      float* o = bmean + ((int64_t)(w * sh.n_slices + s) * sh.cout + ch) * 2;
      o[0] = nimg > 0 ? sb / cnt : 0.0f;
      o[1] = nimg > 0 ? sg / cnt : 0.0f;
      gb += sb;
      gg += sg;
    }
    g[po.beta + ch] = gb;
    g[po.gamma + ch] = gg;
  }
}

// dz = gamma * rstd * (dy - mean(dy) - xhat * mean(dy * xhat)), stored in the
// compute type for the weight-gradient contraction.
template <typename T>
__global__ __launch_bounds__(kThreads) void bn_bwd_dz_kernel(WorkerTable tab, ConvShape sh,
                                                             const float* __restrict__ params,
                                                             const float* __restrict__ z,
                                                             const float* __restrict__ mu,
                                                             const float* __restrict__ rstd,
                                                             const float* __restrict__ dpooled,
                                                             const float* __restrict__ bmean,
                                                             T* __restrict__ dz) {
  const Chunk c = chunk_of(tab, sh);
  if (!c.active) return;
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  f32x4 g, b, m, rs, da, mb, mg;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    g[e] = params[po.gamma + c.c4 * 4 + e];
    b[e] = params[po.beta + c.c4 * 4 + e];
    da[e] = dpooled[(int64_t)c.img * sh.cout + c.c4 * 4 + e] / (float)sh.HW;
    mb[e] = bmean[((int64_t)c.unit * sh.cout + c.c4 * 4 + e) * 2];
    mg[e] = bmean[((int64_t)c.unit * sh.cout + c.c4 * 4 + e) * 2 + 1];
  }
  m = *reinterpret_cast<const f32x4*>(mu + (int64_t)c.unit * sh.cout + c.c4 * 4);
  rs = *reinterpret_cast<const f32x4*>(rstd + (int64_t)c.unit * sh.cout + c.c4 * 4);
  const int64_t e0 = c.row0 * sh.cout + c.c4 * 4;
  for (int r = c.rg; r < c.nrows; r += c.n_rg) {
    const f32x4 zz = *reinterpret_cast<const f32x4*>(z + e0 + (int64_t)r * sh.cout);
    f32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float xh = (zz[e] - m[e]) * rs[e];
      const float dy = (g[e] * xh + b[e] > 0.0f) ? da[e] : 0.0f;
      o[e] = g[e] * rs[e] * (dy - mb[e] - xh * mg[e]);
    }
    if (sizeof(T) == 2) {
      u32x2 q = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
      *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(dz) + e0 + (int64_t)r * sh.cout) = q;
    } else {
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(dz) + e0 + (int64_t)r * sh.cout) = o;
    }
  }
}

// -------------------------------------------------------- weight gradient
// dWc[tap*C_in + c][o] = sum over a worker's pixels r of X[r shifted by tap][c]
// dz[r][o].  A workgroup owns one tap, a 64 x 64 (c, o) tile and one run of
// pixels; its sum goes to a partial array that conv_dw_fold_kernel adds up in
// run order.  Both operands have the contraction index (the pixel) strided in
// memory: they are laid into LDS pixel-major as loaded (bf16: two pixels
// interleaved per 32-bit word), which is the form the MFMA operands gather
// from.
template <typename T> struct DwGeom;
template <> struct DwGeom<bf16_t> { static constexpr int BR = 64, ROWS_PER_T = 2, LROWS = 32; };
template <> struct DwGeom<float> { static constexpr int BR = 32, ROWS_PER_T = 2, LROWS = 32; };

template <typename T>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_dw_kernel(WorkerTable tab, ConvShape sh,
                                                                 const T* __restrict__ dz,
                                                                 float* __restrict__ dwp, int n_runs,
                                                                 int run_rows) {
  constexpr bool HALF = sizeof(T) == 2;
  constexpr int BR = DwGeom<T>::BR, LROWS = DwGeom<T>::LROWS;
  __shared__ __attribute__((aligned(16))) uint32_t smem[2][2][LROWS * 64];   // [buffer][X | dz][pixel (pair)][64]

  const int w = blockIdx.z, run = blockIdx.y;
  const int ct = (sh.cin + 63) / 64, ot = (sh.cout + 63) / 64;
  const int tap = blockIdx.x / (ct * ot);
  const int rest = blockIdx.x - tap * (ct * ot);
  const int c0 = (rest / ot) * 64, n0 = (rest % ot) * 64;
  const int kh = tap / 3, kw = tap - kh * 3;
  const int M = tab.rows[w] * sh.HW;
  const int r_begin = min(run * run_rows, M), r_end = min(r_begin + run_rows, M);

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int xi = lane & 31, gk = lane >> 5, wm = wv >> 1, wn = wv & 1;

  const T* __restrict__ xw = reinterpret_cast<const T*>(tab.x[w]);
  const T* __restrict__ dw_ = dz + (int64_t)tab.row_off[w] * sh.HW * sh.cout;
  const int delta = ((kh - 1) * sh.W + (kw - 1)) * sh.cin;

  // this thread's vector: bf16: pixel pair tid/8, channels 8*(tid%8); fp32:
  // pixels tid/16 and 16 + tid/16, channels 4*(tid%16)
  constexpr int VPR = HALF ? 8 : 16;            // vectors per 64-channel row
  constexpr int V = EL<T>::V;
  const int uv = tid % VPR, ur = tid / VPR;
  const int rl0 = HALF ? 2 * ur : ur, rl1 = HALF ? 2 * ur + 1 : 16 + ur;   // rows within a step
  const bool xcok = c0 + uv * V < sh.cin, dcok = n0 + uv * V < sh.cout;
  // position (h, w) of the two pixels at the first step, advanced step by step
  int ph[2], pw[2];
  {
    const int q0 = r_begin + rl0, q1 = r_begin + rl1;
    const int e0 = q0 % sh.HW, e1 = q1 % sh.HW;
    ph[0] = e0 / sh.W; pw[0] = e0 - ph[0] * sh.W;
    ph[1] = e1 / sh.W; pw[1] = e1 - ph[1] * sh.W;
  }
  const int adv_h = BR / sh.W, adv_w = BR - adv_h * sh.W;
  const int rl[2] = {rl0, rl1};
  const u32x4 zero = {0u, 0u, 0u, 0u};
  u32x4 rx[2], rd[2];

  auto gload = [&](int r0) {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int q = r0 + rl[e];
      const bool in = q < r_end;
      const bool nb = (kh != 0 || ph[e] > 0) && (kh != 2 || ph[e] < sh.H - 1) && (kw != 0 || pw[e] > 0) &&
                      (kw != 2 || pw[e] < sh.W - 1);
      const bool okx = in && nb && xcok, okd = in && dcok;
      const T* px = okx ? xw + (int64_t)q * sh.cin + delta + c0 + uv * V : xw;
      const T* pd = okd ? dw_ + (int64_t)q * sh.cout + n0 + uv * V : dw_;
      const u32x4 vx = *reinterpret_cast<const u32x4*>(px);
      const u32x4 vd = *reinterpret_cast<const u32x4*>(pd);
      rx[e] = okx ? vx : zero;
      rd[e] = okd ? vd : zero;
      // next step's position
      pw[e] += adv_w;
      ph[e] += adv_h;
      if (pw[e] >= sh.W) { pw[e] -= sh.W; ++ph[e]; }
      while (ph[e] >= sh.H) ph[e] -= sh.H;
    }
  };
  auto interleave = [](const u32x4& a, const u32x4& b, u32x4* lo, u32x4* hi) {
    // word j = (a[j], b[j]) as (low half, high half)
    lo->x = __builtin_amdgcn_perm(b.x, a.x, 0x05040100u); lo->y = __builtin_amdgcn_perm(b.x, a.x, 0x07060302u);
    lo->z = __builtin_amdgcn_perm(b.y, a.y, 0x05040100u); lo->w = __builtin_amdgcn_perm(b.y, a.y, 0x07060302u);
    hi->x = __builtin_amdgcn_perm(b.z, a.z, 0x05040100u); hi->y = __builtin_amdgcn_perm(b.z, a.z, 0x07060302u);
    hi->z = __builtin_amdgcn_perm(b.w, a.w, 0x05040100u); hi->w = __builtin_amdgcn_perm(b.w, a.w, 0x07060302u);
  };
  auto lstore = [&](int buf) {
    if (HALF) {
      u32x4 lo, hi;
      interleave(rx[0], rx[1], &lo, &hi);
      u32x4* d = reinterpret_cast<u32x4*>(&smem[buf][0][ur * 64 + uv * 8]);
      d[0] = lo; d[1] = hi;
      interleave(rd[0], rd[1], &lo, &hi);
      d = reinterpret_cast<u32x4*>(&smem[buf][1][ur * 64 + uv * 8]);
      d[0] = lo; d[1] = hi;
    } else {
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        *reinterpret_cast<u32x4*>(&smem[buf][0][rl[e] * 64 + uv * 4]) = rx[e];
        *reinterpret_cast<u32x4*>(&smem[buf][1][rl[e] * 64 + uv * 4]) = rd[e];
      }
    }
  };

  f32x16 acc = zero16();
  const int n_steps = (r_end - r_begin + BR - 1) / BR;
  if (n_steps > 0) {
    gload(r_begin);
    lstore(0);
  }
  __syncthreads();
  for (int t = 0; t < n_steps; ++t) {
    if (t + 1 < n_steps) gload(r_begin + (t + 1) * BR);
    const uint32_t* Xs = smem[t & 1][0] + wm * 32 + xi;
    const uint32_t* Ds = smem[t & 1][1] + wn * 32 + xi;
    if (HALF) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const uint32_t* pa = Xs + (ks * 8 + gk * 4) * 64;
        const uint32_t* pb = Ds + (ks * 8 + gk * 4) * 64;
        const u32x4 a = {pa[0], pa[64], pa[128], pa[192]};
        const u32x4 b = {pb[0], pb[64], pb[128], pb[192]};
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                      acc, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        const float a = __uint_as_float(Xs[(ks * 2 + gk) * 64]);
        const float b = __uint_as_float(Ds[(ks * 2 + gk) * 64]);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
      }
    }
    if (t + 1 < n_steps) lstore((t + 1) & 1);
    __syncthreads();
  }

  const int K = 9 * sh.cin;
  float* __restrict__ out = dwp + ((int64_t)(w * n_runs + run) * K + (int64_t)tap * sh.cin) * sh.cout;
  const int col = n0 + wn * 32 + xi;
  if (col < sh.cout) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int c = c0 + wm * 32 + gk * 4 + (v >> 2) * 8 + (v & 3);
      if (c < sh.cin) out[(int64_t)c * sh.cout + col] = acc[v];
    }
  }
}

__global__ __launch_bounds__(kThreads) void conv_dw_fold_kernel(WorkerTable tab, const float* __restrict__ dwp,
                                                                int n_runs, int64_t len) {
  const int w = blockIdx.y;
  const int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
  if (i >= len) return;
  const float* p = dwp + (int64_t)w * n_runs * len + i;
  f32x4 a = *reinterpret_cast<const f32x4*>(p);
  for (int r = 1; r < n_runs; ++r) a += *reinterpret_cast<const f32x4*>(p + (int64_t)r * len);
  *reinterpret_cast<f32x4*>(tab.grad[w] + i) = a;
}

// ------------------------------------------------------------------- host
struct Plan {
  ConvShape sh;
  WorkerTable tab;
  int64_t K, P;
  int max_unit_images, max_rows, n_units, n_runs, run_rows;
  size_t elem;
  // workspace offsets in bytes
  size_t o_wmat, o_z, o_dz, o_statp, o_mu, o_rstd, o_poolp, o_pooled, o_dpooled, o_dlogits, o_row_loss, o_bwdp,
      o_bmean, o_dwp, total;
};

int make_plan(const synk_convblock_desc* d, const int64_t* rows, int n_workers, int n_slices, Plan* p) {
  if (!d || !rows) return SYNK_ERR_NULL;
  if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS || n_slices < 1) return SYNK_ERR_SHAPE;
  if (d->height < 1 || d->width < 1 || d->c_in < 8 || d->c_out < 8 || d->classes < 1) return SYNK_ERR_SHAPE;
  if (d->c_in % 8 || d->c_out % 8 || d->c_out > kMaxCout || d->classes > kMaxClasses) return SYNK_ERR_SHAPE;
  if (d->height > 4096 || d->width > 4096 || d->c_in > 4096) return SYNK_ERR_SHAPE;
  if (!(d->eps >= 0.0f)) return SYNK_ERR_SHAPE;
  if (d->compute_dtype != SYNK_F32 && d->compute_dtype != SYNK_BF16) return SYNK_ERR_DTYPE;
  if ((int64_t)n_workers * n_slices > 65535) return SYNK_ERR_SHAPE;
  ConvShape& sh = p->sh;
  sh.H = d->height; sh.W = d->width; sh.cin = d->c_in; sh.cout = d->c_out; sh.classes = d->classes;
  sh.HW = d->height * d->width;
  sh.n_workers = n_workers; sh.n_slices = n_slices; sh.grad_op = 0;
  sh.n_chunks = (sh.HW + kChunkRows - 1) / kChunkRows;
  sh.eps = d->eps;
  int64_t total = 0;
  p->max_rows = 0;
  p->max_unit_images = 0;
  for (int w = 0; w < n_workers; ++w) {
    if (rows[w] < 0) return SYNK_ERR_SHAPE;
    if (total + rows[w] > (int64_t)1 << 30) return SYNK_ERR_SHAPE;
    p->tab.rows[w] = (int32_t)rows[w];
    p->tab.row_off[w] = (int32_t)total;
    total += rows[w];
    if (rows[w] > p->max_rows) p->max_rows = (int)rows[w];
    const int64_t u = (rows[w] + n_slices - 1) / n_slices;
    if (u > p->max_unit_images) p->max_unit_images = (int)u;
  }
  p->tab.row_off[n_workers] = (int32_t)total;
  if (total == 0) return SYNK_ERR_SHAPE;
  // pixel rows, and every element index derived from them, stay below 2^31 per array dimension
  if (total * sh.HW >= ((int64_t)1 << 31) / 4 || total * sh.n_chunks >= ((int64_t)1 << 31)) return SYNK_ERR_SHAPE;
  sh.total_images = (int)total;
  p->n_units = n_workers * n_slices;
  p->K = (int64_t)9 * sh.cin;
  p->P = param_off(sh.cin, sh.cout, sh.classes).total;
  p->elem = d->compute_dtype == SYNK_BF16 ? 2 : 4;

  // runs of the weight gradient: enough workgroups to fill the chip, few enough to keep the partials small
  const int BR = d->compute_dtype == SYNK_BF16 ? DwGeom<bf16_t>::BR : DwGeom<float>::BR;
  const int64_t tiles = (int64_t)9 * ((sh.cin + 63) / 64) * ((sh.cout + 63) / 64);
  const int64_t max_px = (int64_t)p->max_rows * sh.HW;
  int64_t runs = (1024 + tiles * n_workers - 1) / (tiles * n_workers);
  const int64_t max_runs = (max_px + 4 * BR - 1) / (4 * BR);   // at least four steps per run
  if (runs > max_runs) runs = max_runs;
  if (runs > 64) runs = 64;
  if (runs < 1) runs = 1;
  int64_t rr = (max_px + runs - 1) / runs;
  rr = (rr + BR - 1) / BR * BR;
  p->n_runs = (int)runs;
  p->run_rows = (int)rr;

  const int64_t R = total, px = total * sh.HW;
  size_t at = 0;
  auto take = [&](size_t bytes) {
    const size_t o = at;
    at += round_up(bytes, 256);
    return o;
  };
  p->o_wmat = take((size_t)p->K * sh.cout * p->elem);
  p->o_z = take((size_t)px * sh.cout * 4);
  p->o_dz = take((size_t)px * sh.cout * p->elem);
  p->o_statp = take((size_t)R * sh.n_chunks * sh.cout * 2 * 4);
  p->o_mu = take((size_t)p->n_units * sh.cout * 4);
  p->o_rstd = take((size_t)p->n_units * sh.cout * 4);
  p->o_poolp = take((size_t)R * sh.n_chunks * sh.cout * 4);
  p->o_pooled = take((size_t)R * sh.cout * 4);
  p->o_dpooled = take((size_t)R * sh.cout * 4);
  p->o_dlogits = take((size_t)R * sh.classes * 4);
  p->o_row_loss = take((size_t)R * 4);
  p->o_bwdp = take((size_t)R * sh.n_chunks * sh.cout * 2 * 4);
  p->o_bmean = take((size_t)p->n_units * sh.cout * 2 * 4);
  p->o_dwp = take((size_t)n_workers * p->n_runs * p->K * sh.cout * 4);
  p->total = at;
  return SYNK_OK;
}

template <typename T>
int run(const Plan& p, const float* params, float* loss, char* ws, hipStream_t st) {
  const ConvShape& sh = p.sh;
  const WorkerTable& tab = p.tab;
  T* wmat = reinterpret_cast<T*>(ws + p.o_wmat);
  float* z = reinterpret_cast<float*>(ws + p.o_z);
  T* dz = reinterpret_cast<T*>(ws + p.o_dz);
  float* statp = reinterpret_cast<float*>(ws + p.o_statp);
  float* mu = reinterpret_cast<float*>(ws + p.o_mu);
  float* rstd = reinterpret_cast<float*>(ws + p.o_rstd);
  float* poolp = reinterpret_cast<float*>(ws + p.o_poolp);
  float* pooled = reinterpret_cast<float*>(ws + p.o_pooled);
  float* dpooled = reinterpret_cast<float*>(ws + p.o_dpooled);
  float* dlogits = reinterpret_cast<float*>(ws + p.o_dlogits);
  float* row_loss = reinterpret_cast<float*>(ws + p.o_row_loss);
  float* bwdp = reinterpret_cast<float*>(ws + p.o_bwdp);
  float* bmean = reinterpret_cast<float*>(ws + p.o_bmean);
  float* dwp = reinterpret_cast<float*>(ws + p.o_dwp);

  const int64_t wn = p.K * sh.cout;
  hipLaunchKernelGGL(conv_weight_kernel<T>, dim3((unsigned)((wn + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                     params, wmat, (int)p.K, sh.cout);
  SYNK_LAUNCH_CHECK();
  const dim3 gf((unsigned)(((int64_t)p.max_unit_images * sh.HW + kFwdBM - 1) / kFwdBM),
                (unsigned)((sh.cout + kFwdBN - 1) / kFwdBN), (unsigned)p.n_units);
  SYNK_LAUNCH_TIMED(conv3x3_fwd_kernel<T>, gf, dim3(kThreads), 0, st, tab, sh, (const T*)wmat, z);
  SYNK_LAUNCH_CHECK();
  const dim3 gc((unsigned)((int64_t)sh.total_images * sh.n_chunks));
  hipLaunchKernelGGL(bn_stats_chunk_kernel, gc, dim3(kThreads), 0, st, tab, sh, (const float*)z, statp);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_stats_unit_kernel, dim3((unsigned)p.n_units), dim3(kThreads), 0, st, tab, sh,
                     (const float*)statp, mu, rstd);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_relu_pool_kernel, gc, dim3(kThreads), 0, st, tab, sh, params, (const float*)z,
                     (const float*)mu, (const float*)rstd, poolp);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(head_image_kernel, dim3((unsigned)sh.total_images), dim3(kThreads), 0, st, tab, sh, params,
                     (const float*)poolp, pooled, dlogits, dpooled, row_loss);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(head_worker_kernel, dim3((unsigned)((sh.classes + kThreads - 1) / kThreads), (unsigned)sh.n_workers),
                     dim3(kThreads), 0, st, tab, sh, (const float*)pooled, (const float*)dlogits,
                     (const float*)row_loss, loss);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_bwd_chunk_kernel, gc, dim3(kThreads), 0, st, tab, sh, params, (const float*)z,
                     (const float*)mu, (const float*)rstd, (const float*)dpooled, bwdp);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_bwd_worker_kernel, dim3((unsigned)sh.n_workers), dim3(kThreads), 0, st, tab, sh,
                     (const float*)bwdp, bmean);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_bwd_dz_kernel<T>, gc, dim3(kThreads), 0, st, tab, sh, params, (const float*)z,
                     (const float*)mu, (const float*)rstd, (const float*)dpooled, (const float*)bmean, dz);
  SYNK_LAUNCH_CHECK();
  const dim3 gd((unsigned)(9 * ((sh.cin + 63) / 64) * ((sh.cout + 63) / 64)), (unsigned)p.n_runs,
                (unsigned)sh.n_workers);
  hipLaunchKernelGGL(conv3x3_dw_kernel<T>, gd, dim3(kThreads), 0, st, tab, sh, (const T*)dz, dwp, p.n_runs,
                     p.run_rows);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(conv_dw_fold_kernel, dim3((unsigned)((wn / 4 + kThreads - 1) / kThreads), (unsigned)sh.n_workers),
                     dim3(kThreads), 0, st, tab, (const float*)dwp, p.n_runs, wn);
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

}  // namespace
}  // namespace synk

using namespace synk;

extern "C" int synk_convblock_param_count(const synk_convblock_desc* d, int64_t* count) {
  if (!d || !count) return SYNK_ERR_NULL;
  const int64_t one = 1;
  Plan p;
  const int st = make_plan(d, &one, 1, 1, &p);
  if (st != SYNK_OK) return st;
  *count = p.P;
  return SYNK_OK;
}

extern "C" int synk_sliced_grad_conv_workspace_bytes(const synk_convblock_desc* d, const int64_t* rows,
                                                     int n_workers, int n_slices, size_t* bytes) {
  if (!bytes) return SYNK_ERR_NULL;
  Plan p;
  const int st = make_plan(d, rows, n_workers, n_slices, &p);
  if (st != SYNK_OK) return st;
  *bytes = p.total;
  return SYNK_OK;
}

extern "C" int synk_sliced_grad_conv(const synk_convblock_desc* d, const float* params, const void* const* x,
                                     const int32_t* const* y, const int64_t* rows, int n_workers, int n_slices,
                                     int grad_op, float* const* grad, float* loss, void* ws, size_t ws_bytes,
                                     void* stream) {
  if (!d || !params || !x || !y || !rows || !grad || !loss) return SYNK_ERR_NULL;
  Plan p;
  const int st = make_plan(d, rows, n_workers, n_slices, &p);
  if (st != SYNK_OK) return st;
  if (grad_op != SYNK_SUM && grad_op != SYNK_MEAN) return SYNK_ERR_OP;
  p.sh.grad_op = grad_op;
  if (!aligned_to(params, 16)) return SYNK_ERR_ALIGN;
  for (int w = 0; w < n_workers; ++w) {
    if (!grad[w]) return SYNK_ERR_NULL;
    if (!aligned_to(grad[w], 16)) return SYNK_ERR_ALIGN;
    if (rows[w] > 0) {
      if (!x[w] || !y[w]) return SYNK_ERR_NULL;
      if (!aligned_to(x[w], 16)) return SYNK_ERR_ALIGN;
    }
    p.tab.x[w] = x[w];
    p.tab.y[w] = y[w];
    p.tab.grad[w] = grad[w];
  }
  for (int w = n_workers; w < SYNK_MAX_WORKERS; ++w) {
    p.tab.x[w] = nullptr; p.tab.y[w] = nullptr; p.tab.grad[w] = nullptr;
    p.tab.rows[w] = 0; p.tab.row_off[w + 1] = p.tab.row_off[n_workers];
  }
  if (!ws || !aligned_to(ws, 256) || ws_bytes < p.total) return SYNK_ERR_WORKSPACE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (d->compute_dtype == SYNK_BF16) return run<bf16_t>(p, params, loss, reinterpret_cast<char*>(ws), s);
  return run<float>(p, params, loss, reinterpret_cast<char*>(ws), s);
}
