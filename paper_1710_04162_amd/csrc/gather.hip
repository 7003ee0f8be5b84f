// Input indexing (Sec. 5.2) fused with the scatter of the index list over
// workers (Sec. 3.2 step 1): batch row j = data[idx[j]] lands, densely packed,
// in the buffer of the worker whose share holds j.  Pure data movement, bound
// by HBM bandwidth: one workgroup per (batch row, row chunk), every load and
// store coalesced across the wavefront.
#include "common.h"

namespace synk {

struct DstTable {
  void* dst[SYNK_MAX_WORKERS];
  int32_t* lab[SYNK_MAX_WORKERS];
};

constexpr int kGBlock = 256;

struct RowRef {
  int64_t src_row;   // idx[j], or -1 when out of range
  int worker;
  int64_t local;     // row inside the worker's buffer
  const void* base;  // the array the row is read from
  const int32_t* labels;
};

// Where batch row j comes from: a list entry, or start + j * step (slice form).
struct IdxSrc {
  const int32_t* idx;   // device int32[n_idx]; NULL = slice form
  int64_t start, step;
};

// Resident shares: worker w indexes its own array with its own list; batch
// row j belongs to the worker whose run [off[w], off[w+1]) of the concatenated
// lists holds it.
struct ResTable {
  const void* data[SYNK_MAX_WORKERS];
  const int32_t* idx[SYNK_MAX_WORKERS];
  const int32_t* lab[SYNK_MAX_WORKERS];
  int32_t n_rows[SYNK_MAX_WORKERS];
  int32_t off[SYNK_MAX_WORKERS + 1];
};
template <bool RES>
struct ResArg {};
template <>
struct ResArg<true> {
  ResTable t;
};

template <bool RES>
__device__ __forceinline__ RowRef locate(const IdxSrc& ix, const ResArg<RES>& ra, const void* data,
                                         const int32_t* labels, int64_t n_idx, int n_workers,
                                         int64_t n_rows, int64_t j, uint32_t* err_word) {
  RowRef r;
  int64_t src;
  if constexpr (RES) {
    int w = 0;
    while (w + 1 < n_workers && j >= ra.t.off[w + 1]) ++w;   // block-uniform, at most 63 steps
    r.worker = w;
    r.local = j - ra.t.off[w];
    src = ra.t.idx[w][r.local];
    r.base = ra.t.data[w];
    r.labels = ra.t.lab[w];
    n_rows = ra.t.n_rows[w];
  } else {
    src = ix.idx ? (int64_t)ix.idx[j] : ix.start + j * ix.step;
    int64_t start;
    share_of(n_idx, n_workers, j, &r.worker, &start);
    r.local = j - start;
    r.base = data;
    r.labels = labels;
  }
  r.src_row = (src >= 0 && src < n_rows) ? src : -1;
  if (r.src_row < 0 && err_word && threadIdx.x == 0 && blockIdx.y == 0) atomicOr(err_word, 1u);
  return r;
}

__device__ __forceinline__ void copy_label(const DstTable& t, const RowRef& r) {
  if (r.labels && blockIdx.y == 0 && threadIdx.x == 0) t.lab[r.worker][r.local] = r.labels[r.src_row];
}

// Bit-exact copy in units of V (16, 4 or 1 bytes).  grid = (n_idx, chunks).
template <bool RES, typename V>
__global__ __launch_bounds__(kGBlock) void gather_copy_kernel(
    const V* __restrict__ data, int64_t n_rows, int64_t row_units, IdxSrc idx, ResArg<RES> ra,
    int64_t n_idx, DstTable t, int n_workers, const int32_t* __restrict__ labels,
    uint32_t* err_word, int units_per_block) {
  const int64_t j = blockIdx.x;
  const RowRef r = locate<RES>(idx, ra, data, labels, n_idx, n_workers, n_rows, j, err_word);
  if (r.src_row < 0) return;
  copy_label(t, r);
  const V* src = reinterpret_cast<const V*>(r.base) + r.src_row * row_units;
  V* dst = reinterpret_cast<V*>(t.dst[r.worker]) + r.local * row_units;
  const int64_t u0 = (int64_t)blockIdx.y * units_per_block;
  int64_t u1 = u0 + units_per_block;
  if (u1 > row_units) u1 = row_units;
  // four loads in flight per thread: a unit past the end re-reads the last one and is dropped
  for (int64_t u = u0 + threadIdx.x; u < u1; u += 4 * kGBlock) {
    V v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t uu = u + k * kGBlock;
      v[k] = src[uu < u1 ? uu : u1 - 1];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (u + k * kGBlock < u1) dst[u + k * kGBlock] = v[k];
  }
}

// float32 -> bfloat16 (nearest-even).  VEC: 4 floats in, 8 bytes out per lane.
template <bool RES, bool VEC>
__global__ __launch_bounds__(kGBlock) void gather_bf16_kernel(
    const float* __restrict__ data, int64_t n_rows, int64_t row_elems,
    IdxSrc idx, ResArg<RES> ra, int64_t n_idx, DstTable t, int n_workers,
    const int32_t* __restrict__ labels, uint32_t* err_word, int units_per_block) {
  const int64_t j = blockIdx.x;
  const RowRef r = locate<RES>(idx, ra, data, labels, n_idx, n_workers, n_rows, j, err_word);
  if (r.src_row < 0) return;
  copy_label(t, r);
  const float* src = reinterpret_cast<const float*>(r.base) + r.src_row * row_elems;
  uint16_t* dst = reinterpret_cast<uint16_t*>(t.dst[r.worker]) + r.local * row_elems;
  const int64_t units = VEC ? (row_elems >> 2) : row_elems;
  const int64_t u0 = (int64_t)blockIdx.y * units_per_block;
  int64_t u1 = u0 + units_per_block;
  if (u1 > units) u1 = units;
  if (VEC) {
    // four loads in flight per thread: a unit past the end re-reads the last one and is dropped
    for (int64_t u = u0 + threadIdx.x; u < u1; u += 4 * kGBlock) {
      f32x4 a[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int64_t uu = u + k * kGBlock;
        a[k] = reinterpret_cast<const f32x4*>(src)[uu < u1 ? uu : u1 - 1];
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (u + k * kGBlock < u1) {
          u32x2 q;
          q.x = pack_bf16x2(a[k].x, a[k].y);
          q.y = pack_bf16x2(a[k].z, a[k].w);
          reinterpret_cast<u32x2*>(dst)[u + k * kGBlock] = q;
        }
      }
    }
  } else {
    for (int64_t u = u0 + threadIdx.x; u < u1; u += kGBlock) dst[u] = f32_to_bf16(src[u]);
  }
}

// uint8 -> float32 through a per-channel table held in LDS.  VEC: each lane
// loads 4 pixels (one dword) and stores one 16-byte vector, so both the load
// and the store of a wavefront are contiguous.  The channel of a unit is
// tracked incrementally (units only move forwards), never divided out.
constexpr int kLBlock = 1024;

template <bool RES, bool VEC>
__global__ __launch_bounds__(kLBlock) void gather_u8_lut_kernel(
    const uint8_t* __restrict__ data, int64_t n_rows, int row_elems, int plane,
    IdxSrc idx, ResArg<RES> ra, int64_t n_idx, DstTable t, int n_workers,
    const float* __restrict__ lut, int channels, const int32_t* __restrict__ labels,
    uint32_t* err_word, int units_per_block) {
  __shared__ float s_lut[SYNK_MAX_CHANNELS * 256];
  const int64_t j = blockIdx.x;
  const RowRef r = locate<RES>(idx, ra, data, labels, n_idx, n_workers, n_rows, j, err_word);
  if (r.src_row < 0) return;   // uniform per block: before the barrier is fine
  for (int i = threadIdx.x; i < channels * 256; i += kLBlock) s_lut[i] = lut[i];
  __syncthreads();
  copy_label(t, r);
  const uint8_t* src = reinterpret_cast<const uint8_t*>(r.base) + r.src_row * (int64_t)row_elems;
  float* dst = reinterpret_cast<float*>(t.dst[r.worker]) + r.local * (int64_t)row_elems;
  const int units = VEC ? (row_elems >> 2) : row_elems;
  const int plane_u = VEC ? (plane >> 2) : plane;     // units per channel plane
  const int u0 = blockIdx.y * units_per_block;
  int u1 = u0 + units_per_block;
  if (u1 > units) u1 = units;
  int u = u0 + threadIdx.x;
  int c = u / plane_u;                  // one division per thread
  int bound = (c + 1) * plane_u;        // first unit of the next channel
  if (VEC) {
    constexpr int UNROLL = 4;
    for (; u + (UNROLL - 1) * kLBlock < u1; u += UNROLL * kLBlock) {
      uint32_t px[UNROLL];
#pragma unroll
      for (int k = 0; k < UNROLL; ++k)
        px[k] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(src) + u + k * kLBlock);
#pragma unroll
      for (int k = 0; k < UNROLL; ++k) {
        const int uu = u + k * kLBlock;
        while (uu >= bound) { ++c; bound += plane_u; }
        const float* l = s_lut + c * 256;
        f32x4 o;
        o.x = l[px[k] & 0xffu];
        o.y = l[(px[k] >> 8) & 0xffu];
        o.z = l[(px[k] >> 16) & 0xffu];
        o.w = l[px[k] >> 24];
        reinterpret_cast<f32x4*>(dst)[uu] = o;
      }
    }
    for (; u < u1; u += kLBlock) {
      while (u >= bound) { ++c; bound += plane_u; }
      const uint32_t px = reinterpret_cast<const uint32_t*>(src)[u];
      const float* l = s_lut + c * 256;
      f32x4 o;
      o.x = l[px & 0xffu];
      o.y = l[(px >> 8) & 0xffu];
      o.z = l[(px >> 16) & 0xffu];
      o.w = l[px >> 24];
      reinterpret_cast<f32x4*>(dst)[u] = o;
    }
  } else {
    for (; u < u1; u += kLBlock) {
      while (u >= bound) { ++c; bound += plane_u; }
      dst[u] = s_lut[c * 256 + src[u]];
    }
  }
}

struct LutArgs {
  double v[2 * SYNK_MAX_CHANNELS];
};

__global__ void norm_lut_kernel_args(float* __restrict__ lut, int channels, LutArgs a) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < channels * 256) {
    const int c = i >> 8;
    lut[i] = (float)(((double)(i & 255) - a.v[c]) / a.v[SYNK_MAX_CHANNELS + c]);
  }
}

__global__ void clear_word_kernel(uint32_t* w) { *w = 0u; }

static int chunking(int64_t units, int* units_per_block, int* chunks) {
  // one batch of four units per thread per block (short-lived workgroups stream faster than
  // ones that loop: 14.3 against 15.7 us on 64 rows of 200,704 floats); at least one block per row
  int64_t upb = (int64_t)kGBlock * 4;
  if (units < upb) upb = (units + kGBlock - 1) / kGBlock * kGBlock;
  if (upb < kGBlock) upb = kGBlock;
  while ((units + upb - 1) / upb > 65535 && upb < ((int64_t)1 << 30)) upb *= 2;   // grid.y limit: longer loops instead
  *units_per_block = (int)upb;
  const int64_t c = (units + upb - 1) / upb;
  if (c > 65535) return SYNK_ERR_UNSUPPORTED;
  *chunks = c < 1 ? 1 : (int)c;
  return SYNK_OK;
}

}  // namespace synk

using namespace synk;

extern "C" size_t synk_gather_workspace_bytes(void) { return 256; }

// The gather behind every entry point.  res != NULL: resident shares (worker
// w reads res->data[w] with res->idx[w]; counts[w] rows each, n_idx their sum;
// data, n_rows, idx and labels are then unused).
static int gather_impl(const void* data, int64_t n_rows, int64_t row_elems, int src_dtype,
                       IdxSrc idx, int64_t n_idx, void* const* dst, int n_workers,
                       int dst_dtype, const float* lut, int channels,
                       const int32_t* labels, int32_t* const* dst_labels, uint32_t flags,
                       void* ws, size_t ws_bytes, void* stream, const ResTable* res = nullptr,
                       const int64_t* counts = nullptr) {
  if ((!res && !data) || !dst) return SYNK_ERR_NULL;
  const bool want_labels = res ? (dst_labels != nullptr) : (labels != nullptr);
  if (labels && !dst_labels) return SYNK_ERR_NULL;
  if (n_rows < 0 || row_elems <= 0 || n_idx < 0) return SYNK_ERR_SHAPE;
  if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS) return SYNK_ERR_SHAPE;
  if (n_idx > 0x7fffffffLL) return SYNK_ERR_SHAPE;   // grid.x limit
  if (src_dtype < SYNK_U8 || src_dtype > SYNK_BF16 || dst_dtype < SYNK_U8 || dst_dtype > SYNK_BF16)
    return SYNK_ERR_DTYPE;
  enum { COPY, TO_BF16, U8_LUT } mode;
  if (dst_dtype == src_dtype) mode = COPY;
  else if (src_dtype == SYNK_F32 && dst_dtype == SYNK_BF16) mode = TO_BF16;
  else if (src_dtype == SYNK_U8 && dst_dtype == SYNK_F32) mode = U8_LUT;
  else return SYNK_ERR_DTYPE;
  if (mode == U8_LUT) {
    if (!lut) return SYNK_ERR_NULL;
    if (channels < 1 || channels > SYNK_MAX_CHANNELS || row_elems % channels != 0)
      return SYNK_ERR_SHAPE;
    if (row_elems > 0x7fffffffLL - (1 << 20)) return SYNK_ERR_UNSUPPORTED;   // 32-bit unit arithmetic
  }
  static const int kElemBytes[4] = {1, 4, 4, 2};
  const int src_b = kElemBytes[src_dtype], dst_b = kElemBytes[dst_dtype];
  // alignment that every array rows are read from has
  auto src_aligned = [&](size_t a) {
    if (!res) return aligned_to(data, a);
    for (int w = 0; w < n_workers; ++w)
      if (counts[w] > 0 && !aligned_to(res->data[w], a)) return false;
    return true;
  };
  if (!src_aligned(src_b)) return SYNK_ERR_ALIGN;
  uint32_t* err_word = nullptr;
  if (flags & SYNK_FLAG_CHECK_INDEX) {
    if (!ws || ws_bytes < synk_gather_workspace_bytes() || !aligned_to(ws, 256))
      return SYNK_ERR_WORKSPACE;
    err_word = reinterpret_cast<uint32_t*>(ws);
  }
  DstTable t;
  bool dst16 = true, dst8 = true, dst4 = true;
  for (int w = 0; w < n_workers; ++w) {
    int64_t s, n;
    share(n_idx, n_workers, w, &s, &n);
    if (counts) n = counts[w];
    if (n > 0 && (!dst[w] || (want_labels && !dst_labels[w]))) return SYNK_ERR_NULL;
    if (n > 0 && !aligned_to(dst[w], dst_b)) return SYNK_ERR_ALIGN;
    if (n > 0) {
      dst16 = dst16 && aligned_to(dst[w], 16);
      dst8 = dst8 && aligned_to(dst[w], 8);
      dst4 = dst4 && aligned_to(dst[w], 4);
    }
    t.dst[w] = dst[w];
    t.lab[w] = want_labels ? dst_labels[w] : nullptr;
  }
  // Every check that can refuse the call is made before the first launch.
  int upb = 0, chunks = 0, unit = 1, plane = 0;
  bool vec = false;
  int64_t row_units = 0;
  if (n_idx > 0) {
    if (mode == COPY) {
      const int64_t row_bytes = row_elems * src_b;
      if (row_bytes % 16 == 0 && src_aligned(16) && dst16) unit = 16;
      else if (row_bytes % 4 == 0 && src_aligned(4) && dst4) unit = 4;
      row_units = row_bytes / unit;
      if (int rc = chunking(row_units, &upb, &chunks)) return rc;
    } else if (mode == TO_BF16) {
      vec = row_elems % 4 == 0 && src_aligned(16) && dst8;
      if (int rc = chunking(vec ? row_elems / 4 : row_elems, &upb, &chunks)) return rc;
    } else {
      plane = (int)(row_elems / channels);
      vec = plane % 4 == 0 && src_aligned(4) && dst16;
      const int64_t units = vec ? row_elems / 4 : row_elems;
      upb = kLBlock * 4;                                   // 4 units per thread: one unrolled batch
      const int64_t nch = (units + upb - 1) / upb;
      if (nch > 65535) return SYNK_ERR_UNSUPPORTED;
      chunks = (int)nch;
    }
  }
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (err_word) {
    hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, s, err_word);
    SYNK_LAUNCH_CHECK();
  }
  if (n_idx == 0) return SYNK_OK;

  const dim3 gb(kGBlock), lb(kLBlock);
  const dim3 grid((unsigned)n_idx, chunks);
  if (mode == COPY) {
#define SYNK_COPY(V, RES, RA)                                                                        \
  SYNK_LAUNCH_TIMED((gather_copy_kernel<RES, V>), grid, gb, 0, s, reinterpret_cast<const V*>(data),  \
                     n_rows, row_units, idx, RA, n_idx, t, n_workers, labels, err_word, upb)
    if (res) {
      if (unit == 16) SYNK_COPY(u32x4, true, ResArg<true>{*res});
      else if (unit == 4) SYNK_COPY(uint32_t, true, ResArg<true>{*res});
      else SYNK_COPY(uint8_t, true, ResArg<true>{*res});
    } else {
      if (unit == 16) SYNK_COPY(u32x4, false, ResArg<false>{});
      else if (unit == 4) SYNK_COPY(uint32_t, false, ResArg<false>{});
      else SYNK_COPY(uint8_t, false, ResArg<false>{});
    }
#undef SYNK_COPY
  } else if (mode == TO_BF16) {
#define SYNK_BF(VEC, RES, RA)                                                                            \
  SYNK_LAUNCH_TIMED((gather_bf16_kernel<RES, VEC>), grid, gb, 0, s, reinterpret_cast<const float*>(data),  \
                     n_rows, row_elems, idx, RA, n_idx, t, n_workers, labels, err_word, upb)
    if (res) {
      if (vec) SYNK_BF(true, true, ResArg<true>{*res});
      else SYNK_BF(false, true, ResArg<true>{*res});
    } else {
      if (vec) SYNK_BF(true, false, ResArg<false>{});
      else SYNK_BF(false, false, ResArg<false>{});
    }
#undef SYNK_BF
  } else {
#define SYNK_LUT(VEC, RES, RA)                                                                   \
  SYNK_LAUNCH_TIMED((gather_u8_lut_kernel<RES, VEC>), grid, lb, 0, s,                            \
                     reinterpret_cast<const uint8_t*>(data), n_rows, (int)row_elems, plane, idx, \
                     RA, n_idx, t, n_workers, lut, channels, labels, err_word, upb)
    if (res) {
      if (vec) SYNK_LUT(true, true, ResArg<true>{*res});
      else SYNK_LUT(false, true, ResArg<true>{*res});
    } else {
      if (vec) SYNK_LUT(true, false, ResArg<false>{});
      else SYNK_LUT(false, false, ResArg<false>{});
    }
#undef SYNK_LUT
  }
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

extern "C" int synk_gather_rows(const void* data, int64_t n_rows, int64_t row_elems, int src_dtype,
                                const int32_t* idx, int64_t n_idx, void* const* dst, int n_workers,
                                int dst_dtype, const float* lut, int channels,
                                const int32_t* labels, int32_t* const* dst_labels, uint32_t flags,
                                void* ws, size_t ws_bytes, void* stream) {
  if (!idx && n_idx > 0) return SYNK_ERR_NULL;
  return gather_impl(data, n_rows, row_elems, src_dtype, IdxSrc{idx, 0, 0}, n_idx, dst, n_workers, dst_dtype,
                     lut, channels, labels, dst_labels, flags, ws, ws_bytes, stream);
}

extern "C" int synk_gather_slice(const void* data, int64_t n_rows, int64_t row_elems, int src_dtype,
                                 int64_t start, int64_t stop, int64_t step, void* const* dst,
                                 int n_workers, int dst_dtype, const float* lut, int channels,
                                 const int32_t* labels, int32_t* const* dst_labels, void* stream) {
  if (step < 1) return SYNK_ERR_SHAPE;
  if (n_rows < 0) return SYNK_ERR_SHAPE;
  if (start < 0 || stop < start || stop > n_rows) return SYNK_ERR_INDEX;
  const int64_t n_idx = (stop - start + step - 1) / step;
  return gather_impl(data, n_rows, row_elems, src_dtype, IdxSrc{nullptr, start, step}, n_idx, dst, n_workers,
                     dst_dtype, lut, channels, labels, dst_labels, 0u, nullptr, 0, stream);
}

extern "C" int synk_scatter_rows(const void* data, int64_t n_rows, int64_t row_elems, int dtype,
                                 void* const* dst, int n_workers, const int32_t* labels,
                                 int32_t* const* dst_labels, void* stream) {
  return synk_gather_slice(data, n_rows, row_elems, dtype, 0, n_rows, 1, dst, n_workers, dtype, nullptr, 0,
                           labels, dst_labels, stream);
}

extern "C" int synk_gather_resident(const void* const* shares, const int64_t* share_rows, int64_t row_elems,
                                    int src_dtype, const int32_t* const* idx, const int64_t* n_idx,
                                    void* const* dst, int n_workers, int dst_dtype, const float* lut,
                                    int channels, const int32_t* const* labels,
                                    int32_t* const* dst_labels, uint32_t flags, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (!shares || !share_rows || !idx || !n_idx || !dst) return SYNK_ERR_NULL;
  if (labels && !dst_labels) return SYNK_ERR_NULL;
  if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS) return SYNK_ERR_SHAPE;
  ResTable rt;
  int64_t total = 0;
  for (int w = 0; w < n_workers; ++w) {
    if (n_idx[w] < 0 || share_rows[w] < 0 || share_rows[w] > 0x7fffffffLL) return SYNK_ERR_SHAPE;
    if (n_idx[w] > 0 && (!shares[w] || !idx[w])) return SYNK_ERR_NULL;
    if (n_idx[w] > 0 && labels && !labels[w]) return SYNK_ERR_NULL;
    rt.data[w] = shares[w];
    rt.idx[w] = idx[w];
    rt.lab[w] = labels ? labels[w] : nullptr;
    rt.n_rows[w] = (int32_t)share_rows[w];
    rt.off[w] = (int32_t)total;
    total += n_idx[w];
    if (total > 0x7fffffffLL) return SYNK_ERR_SHAPE;
  }
  for (int w = n_workers; w <= SYNK_MAX_WORKERS; ++w) rt.off[w] = (int32_t)total;
  return gather_impl(nullptr, 0, row_elems, src_dtype, IdxSrc{nullptr, 0, 0}, total, dst, n_workers, dst_dtype,
                     lut, channels, nullptr, labels ? dst_labels : nullptr, flags, ws, ws_bytes, stream, &rt,
                     n_idx);
}

extern "C" int synk_build_norm_lut(const float* mean, const float* std, int channels, float* lut,
                                   void* stream) {
  if (!mean || !std || !lut) return SYNK_ERR_NULL;
  if (channels < 1 || channels > SYNK_MAX_CHANNELS) return SYNK_ERR_SHAPE;
  if (!aligned_to(lut, 4)) return SYNK_ERR_ALIGN;
  LutArgs a;
  for (int c = 0; c < SYNK_MAX_CHANNELS; ++c) {
    a.v[c] = c < channels ? (double)mean[c] : 0.0;
    a.v[SYNK_MAX_CHANNELS + c] = c < channels ? (double)std[c] : 1.0;
    if (c < channels && std[c] == 0.0f) return SYNK_ERR_SHAPE;
  }
  hipLaunchKernelGGL(norm_lut_kernel_args, dim3(channels), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(stream), lut, channels, a);
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

extern "C" int synk_poll_error(void* ws, void* stream) {
  if (!ws) return SYNK_ERR_NULL;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  uint32_t word = 0;
  SYNK_HIP_TRY(hipMemcpyAsync(&word, ws, sizeof(word), hipMemcpyDeviceToHost, s));
  SYNK_HIP_TRY(hipStreamSynchronize(s));
  if (word) {
    hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, s, reinterpret_cast<uint32_t*>(ws));
    SYNK_LAUNCH_CHECK();
    return SYNK_ERR_INDEX;
  }
  return SYNK_OK;
}
