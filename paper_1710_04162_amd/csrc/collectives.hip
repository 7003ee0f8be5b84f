// The collectives over the N worker copies of a variable (Sec. 3.2, the
// part on shared variables, which lists broadcast and all-reduce among its
// collectives; App. A: the parameter average), with the workers emulated as N
// device buffers.  Streaming kernels bound by HBM bandwidth: every source
// element is read once, every destination element written once, 16-byte
// accesses when the buffers allow them.
#include "common.h"

namespace synk {

struct PtrTable {
  void* p[SYNK_MAX_WORKERS];
  float w[SYNK_MAX_WORKERS];
};

struct GatherTable {
  const uint32_t* src[SYNK_MAX_WORKERS];
  uint32_t* dst[SYNK_MAX_WORKERS];
  int64_t start[SYNK_MAX_WORKERS + 1];
};

constexpr int kCBlock = 256;

// Workgroups per launch, measured per kernel at 25.6 M elements and 8 workers:
// the in-place all-reduce is fastest with one unit per thread (4.9 against 4.8
// TB/s at 2048 workgroups), the broadcast at 16384 workgroups (5.5 against 5.0
// at 2048 and 5.1 at one unit per thread), the all-gather at 4096 or more per
// segment (shares of 3,194,629 elements: 213 / 204 / 197 / 191 / 191 us at 512 /
// 1024 / 2048 / 4096 / 16384; shares that are a multiple of 64 elements: 178 us;
// the broadcast of the same bytes: 167 us).
constexpr int64_t kAllReduceGridCap = (int64_t)1 << 20;
constexpr int64_t kBroadcastGridCap = 16384;
constexpr int64_t kAllGatherGridCap = 4096;
static inline int coll_grid(int64_t units, int64_t cap) {
  int64_t b = (units + kCBlock - 1) / kCBlock;
  if (b > cap) b = cap;
  if (b < 1) b = 1;
  return (int)b;
}

// dst_w[i] = src[i] for every worker w.  VEC: 16-byte units, else 4-byte.
// A thread reads a unit once and stores it n times.  One destination per
// workgroup instead (workgroup b serving destination b % n, so that each of the
// 8 XCDs writes one copy and every XCD reads the whole source) took 258-318 us
// against 167 us at 8 x 102 MB: the source would cross the chip eight times.
template <bool VEC>
__global__ __launch_bounds__(kCBlock) void broadcast_kernel(const uint32_t* __restrict__ src, PtrTable t,
                                                            int n, int64_t len) {
  const int64_t stride = (int64_t)gridDim.x * kCBlock;
  const int64_t i0 = (int64_t)blockIdx.x * kCBlock + threadIdx.x;
  if (VEC) {
    const int64_t n_vec = len >> 2;
    for (int64_t i = i0; i < n_vec; i += stride) {
      const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src) + i);
      for (int w = 0; w < n; ++w) reinterpret_cast<u32x4*>(t.p[w])[i] = v;
    }
    for (int64_t e = (n_vec << 2) + i0; e < len; e += stride) {
      const uint32_t v = src[e];
      for (int w = 0; w < n; ++w) reinterpret_cast<uint32_t*>(t.p[w])[e] = v;
    }
  } else {
    for (int64_t e = i0; e < len; e += stride) {
      const uint32_t v = src[e];
      for (int w = 0; w < n; ++w) reinterpret_cast<uint32_t*>(t.p[w])[e] = v;
    }
  }
}

template <typename T, int OP>
__device__ __forceinline__ T fold2(T a, T b, float wb) {
  if (OP == SYNK_SUM) return a + b;
  if (OP == SYNK_PROD) return a * b;
  if (OP == SYNK_MAX) return a > b ? a : b;
  if (OP == SYNK_MIN) return a < b ? a : b;
  return (T)fmaf(wb, (float)b, (float)a);   // SYNK_MEAN: running weighted sum
}

template <typename T>
struct V4 {};
template <>
struct V4<float> { using type = f32x4; };
template <>
struct V4<int32_t> { using type = i32x4; };

// Every buffer receives the fold, in buffer order, of element i of all n
// buffers (in place: a thread reads element i everywhere before it writes it
// anywhere, and no other thread touches element i).  NS > 0 fixes n at compile
// time so that all loads are issued together.
template <typename T, int OP, int NS, bool VEC>
__global__ __launch_bounds__(kCBlock) void all_reduce_kernel(PtrTable t, int n_dyn, int64_t len) {
  using V = typename V4<T>::type;
  const int n = NS > 0 ? NS : n_dyn;
  const int64_t stride = (int64_t)gridDim.x * kCBlock;
  const int64_t i0 = (int64_t)blockIdx.x * kCBlock + threadIdx.x;
  const int64_t n_vec = VEC ? (len >> 2) : 0;
  for (int64_t i = i0; i < n_vec; i += stride) {
    V acc;
    if (NS > 0) {
      V g[NS > 0 ? NS : 1];
#pragma unroll
      for (int w = 0; w < NS; ++w) g[w] = __builtin_nontemporal_load(reinterpret_cast<const V*>(t.p[w]) + i);
      acc = g[0];
      if (OP == SYNK_MEAN) {
        acc.x = (T)(t.w[0] * (float)acc.x); acc.y = (T)(t.w[0] * (float)acc.y);
        acc.z = (T)(t.w[0] * (float)acc.z); acc.w = (T)(t.w[0] * (float)acc.w);
      }
#pragma unroll
      for (int w = 1; w < NS; ++w) {
        acc.x = fold2<T, OP>(acc.x, g[w].x, t.w[w]); acc.y = fold2<T, OP>(acc.y, g[w].y, t.w[w]);
        acc.z = fold2<T, OP>(acc.z, g[w].z, t.w[w]); acc.w = fold2<T, OP>(acc.w, g[w].w, t.w[w]);
      }
    } else {
      acc = reinterpret_cast<const V*>(t.p[0])[i];
      if (OP == SYNK_MEAN) {
        acc.x = (T)(t.w[0] * (float)acc.x); acc.y = (T)(t.w[0] * (float)acc.y);
        acc.z = (T)(t.w[0] * (float)acc.z); acc.w = (T)(t.w[0] * (float)acc.w);
      }
      for (int w = 1; w < n; ++w) {
        const V g = reinterpret_cast<const V*>(t.p[w])[i];
        acc.x = fold2<T, OP>(acc.x, g.x, t.w[w]); acc.y = fold2<T, OP>(acc.y, g.y, t.w[w]);
        acc.z = fold2<T, OP>(acc.z, g.z, t.w[w]); acc.w = fold2<T, OP>(acc.w, g.w, t.w[w]);
      }
    }
    for (int w = 0; w < n; ++w) reinterpret_cast<V*>(t.p[w])[i] = acc;
  }
  for (int64_t e = (n_vec << 2) + i0; e < len; e += stride) {
    T acc = reinterpret_cast<const T*>(t.p[0])[e];
    if (OP == SYNK_MEAN) acc = (T)(t.w[0] * (float)acc);
    for (int w = 1; w < n; ++w) acc = fold2<T, OP>(acc, reinterpret_cast<const T*>(t.p[w])[e], t.w[w]);
    for (int w = 0; w < n; ++w) reinterpret_cast<T*>(t.p[w])[e] = acc;
  }
}

// Body of a source that starts R elements past a 16-byte boundary: destination vector i is elements
// R .. R+3 of the aligned source vectors i and i+1.
template <int R>
__device__ __forceinline__ void gather_body_shifted(const u32x4* __restrict__ al, const GatherTable& t, int n,
                                                    int64_t dst_off, int64_t n_vec, int64_t i0, int64_t stride) {
  for (int64_t i = i0; i < n_vec; i += stride) {
    const u32x4 lo = __builtin_nontemporal_load(al + i), hi = __builtin_nontemporal_load(al + i + 1);
    u32x4 v;
    if (R == 1) v = u32x4{lo.y, lo.z, lo.w, hi.x};
    else if (R == 2) v = u32x4{lo.z, lo.w, hi.x, hi.y};
    else v = u32x4{lo.w, hi.x, hi.y, hi.z};
    for (int w = 0; w < n; ++w) *reinterpret_cast<u32x4*>(t.dst[w] + dst_off + (i << 2)) = v;
  }
}

// blockIdx.y = source worker b: its lens[b] elements go to offset start[b] of
// every destination.  VEC (every destination base 16-byte aligned): the
// segment is cut where the destination offset becomes a multiple of four
// elements and the body is written with 16-byte stores.  The source may sit at
// any 4-byte offset against that grid (shards of 3,194,629 elements do): a body
// vector is then put together from the two aligned 16-byte source vectors that
// hold it (neighbouring threads ask for the same lines, so memory is still read
// once), and the first and last body vector, whose aligned neighbours may lie
// outside the source, go with the head and tail in 4-byte units.
template <bool VEC>
__global__ __launch_bounds__(kCBlock) void all_gather_kernel(GatherTable t, int n) {
  const int b = blockIdx.y;
  const int64_t len = t.start[b + 1] - t.start[b];
  const uint32_t* src = t.src[b];
  const int64_t off = t.start[b];
  const int64_t stride = (int64_t)gridDim.x * kCBlock;
  const int64_t i0 = (int64_t)blockIdx.x * kCBlock + threadIdx.x;
  int64_t head = VEC ? ((64 - (off & 63)) & 63) : len;   // to a 256-byte boundary of the destinations
  if (head > len) head = len;
  int64_t n_vec = (len - head) >> 2;
  // elements by which the source of the body is past a 16-byte boundary (uniform for the source)
  const int r = VEC ? (int)((reinterpret_cast<uintptr_t>(src + head) >> 2) & 3) : 0;
  if (VEC && r != 0) {
    if (n_vec >= 2) {
      head += 4;
      n_vec -= 2;
    } else {
      n_vec = 0;
    }
  }
  if (VEC) {
    if (r == 0) {
      for (int64_t i = i0; i < n_vec; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + head) + i);
        for (int w = 0; w < n; ++w) *reinterpret_cast<u32x4*>(t.dst[w] + off + head + (i << 2)) = v;
      }
    } else {
      const u32x4* al = reinterpret_cast<const u32x4*>(src + head - r);   // inside the source: head >= 4 > r
      if (r == 1) gather_body_shifted<1>(al, t, n, off + head, n_vec, i0, stride);
      else if (r == 2) gather_body_shifted<2>(al, t, n, off + head, n_vec, i0, stride);
      else gather_body_shifted<3>(al, t, n, off + head, n_vec, i0, stride);
    }
  }
  // head and tail (or everything, without VEC) in 4-byte units
  const int64_t tail0 = head + (n_vec << 2);
  const int64_t rest = head + (len - tail0);
  for (int64_t k = i0; k < rest; k += stride) {
    const int64_t e = k < head ? k : tail0 + (k - head);
    const uint32_t v = src[e];
    for (int w = 0; w < n; ++w) t.dst[w][off + e] = v;
  }
}

template <typename T, int OP, bool VEC>
static int launch_all_reduce_n(const PtrTable& t, int n, int64_t len, hipStream_t s) {
  const dim3 grid(coll_grid(VEC ? (len >> 2) + 1 : len, kAllReduceGridCap)), block(kCBlock);
#define SYNK_AR(NS) SYNK_LAUNCH_TIMED((all_reduce_kernel<T, OP, NS, VEC>), grid, block, 0, s, t, n, len)
  switch (n) {
    case 2: SYNK_AR(2); break;
    case 4: SYNK_AR(4); break;
    case 8: SYNK_AR(8); break;
    default: SYNK_AR(0); break;
  }
#undef SYNK_AR
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

template <typename T, int OP>
static int launch_all_reduce(const PtrTable& t, int n, int64_t len, bool vec, hipStream_t s) {
  return vec ? launch_all_reduce_n<T, OP, true>(t, n, len, s) : launch_all_reduce_n<T, OP, false>(t, n, len, s);
}

template <typename T>
static int dispatch_all_reduce(int op, const PtrTable& t, int n, int64_t len, bool vec, hipStream_t s) {
  switch (op) {
    case SYNK_SUM: return launch_all_reduce<T, SYNK_SUM>(t, n, len, vec, s);
    case SYNK_MAX: return launch_all_reduce<T, SYNK_MAX>(t, n, len, vec, s);
    case SYNK_MIN: return launch_all_reduce<T, SYNK_MIN>(t, n, len, vec, s);
    case SYNK_PROD: return launch_all_reduce<T, SYNK_PROD>(t, n, len, vec, s);
    default: return SYNK_ERR_OP;
  }
}

}  // namespace synk

using namespace synk;

extern "C" int synk_broadcast(const void* src, void* const* dsts, int n, int64_t len, int dtype,
                              void* stream) {
  if (!src || !dsts) return SYNK_ERR_NULL;
  if (n < 1 || n > SYNK_MAX_WORKERS || len < 0) return SYNK_ERR_SHAPE;
  if (dtype != SYNK_F32 && dtype != SYNK_I32) return SYNK_ERR_DTYPE;
  if (!aligned_to(src, 4)) return SYNK_ERR_ALIGN;
  PtrTable t;
  bool vec = aligned_to(src, 16);
  for (int w = 0; w < n; ++w) {
    if (!dsts[w]) return SYNK_ERR_NULL;
    if (!aligned_to(dsts[w], 4)) return SYNK_ERR_ALIGN;
    vec = vec && aligned_to(dsts[w], 16);
    t.p[w] = dsts[w];
    t.w[w] = 0.0f;
  }
  if (len == 0) return SYNK_OK;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const uint32_t* sp = reinterpret_cast<const uint32_t*>(src);
  if (vec)
    SYNK_LAUNCH_TIMED((broadcast_kernel<true>), dim3(coll_grid((len >> 2) + 1, kBroadcastGridCap)), dim3(kCBlock), 0, s, sp, t, n, len);
  else
    SYNK_LAUNCH_TIMED((broadcast_kernel<false>), dim3(coll_grid(len, kBroadcastGridCap)), dim3(kCBlock), 0, s, sp, t, n, len);
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

extern "C" int synk_all_reduce(void* const* bufs, int n, int64_t len, int dtype, int op,
                               const float* weights, void* stream) {
  if (!bufs) return SYNK_ERR_NULL;
  if (n < 1 || n > SYNK_MAX_WORKERS || len < 0) return SYNK_ERR_SHAPE;
  if (dtype != SYNK_F32 && dtype != SYNK_I32) return SYNK_ERR_DTYPE;
  if (op < SYNK_SUM || op > SYNK_PROD) return SYNK_ERR_OP;          // CONCAT: use synk_all_gather
  if (op == SYNK_MEAN && dtype != SYNK_F32) return SYNK_ERR_OP;
  if (weights && op != SYNK_MEAN) return SYNK_ERR_OP;
  PtrTable t;
  bool vec = true;
  for (int w = 0; w < n; ++w) {
    if (!bufs[w]) return SYNK_ERR_NULL;
    if (!aligned_to(bufs[w], 4)) return SYNK_ERR_ALIGN;
    for (int q = 0; q < w; ++q)
      if (bufs[q] == bufs[w]) return SYNK_ERR_SHAPE;               // the N copies must be distinct buffers
    vec = vec && aligned_to(bufs[w], 16);
    t.p[w] = bufs[w];
    t.w[w] = weights ? weights[w] : 1.0f / (float)n;
  }
  if (len == 0) return SYNK_OK;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (op == SYNK_MEAN) return launch_all_reduce<float, SYNK_MEAN>(t, n, len, vec, s);
  if (dtype == SYNK_F32) return dispatch_all_reduce<float>(op, t, n, len, vec, s);
  return dispatch_all_reduce<int32_t>(op, t, n, len, vec, s);
}

extern "C" int synk_all_gather(const void* const* srcs, const int64_t* lens, int n, int dtype,
                               void* const* dsts, void* stream) {
  if (!srcs || !lens || !dsts) return SYNK_ERR_NULL;
  if (n < 1 || n > SYNK_MAX_WORKERS) return SYNK_ERR_SHAPE;
  if (dtype != SYNK_F32 && dtype != SYNK_I32) return SYNK_ERR_DTYPE;
  GatherTable t;
  t.start[0] = 0;
  int64_t longest = 0;
  for (int w = 0; w < n; ++w) {
    if (lens[w] < 0) return SYNK_ERR_SHAPE;
    if (lens[w] > 0 && !srcs[w]) return SYNK_ERR_NULL;
    if (!aligned_to(srcs[w], 4)) return SYNK_ERR_ALIGN;
    t.src[w] = reinterpret_cast<const uint32_t*>(srcs[w]);
    t.start[w + 1] = t.start[w] + lens[w];
    if (lens[w] > longest) longest = lens[w];
  }
  if (t.start[n] == 0) return SYNK_OK;
  for (int w = 0; w < n; ++w) {
    if (!dsts[w]) return SYNK_ERR_NULL;
    if (!aligned_to(dsts[w], 4)) return SYNK_ERR_ALIGN;
    t.dst[w] = reinterpret_cast<uint32_t*>(dsts[w]);
  }
  bool vec = true;
  for (int w = 0; w < n; ++w) vec = vec && aligned_to(dsts[w], 16);
  int gx = coll_grid(vec ? (longest >> 2) + 1 : longest, kAllGatherGridCap);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (vec) SYNK_LAUNCH_TIMED((all_gather_kernel<true>), dim3(gx, n), dim3(kCBlock), 0, s, t, n);
  else SYNK_LAUNCH_TIMED((all_gather_kernel<false>), dim3(gx, n), dim3(kCBlock), 0, s, t, n);
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}
