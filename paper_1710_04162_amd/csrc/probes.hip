// Measured peaks of the part, for the rooflines the benchmark reports: what the
// matrix cores deliver from registers alone, what plain 16-byte stores and loads
// reach, how fast a CU takes operand tiles from L2 straight into LDS, and what one
// wavefront hides behind its own MFMAs.  Timing
// kernels only: they compute nothing of the method.  Every access stays inside
// the caller's buffer (checked on the host).
#include "common.h"

namespace synk {

typedef __bf16 bf16x8p __attribute__((ext_vector_type(8)));

// 4 independent accumulator chains of 32x32x16 bf16 MFMAs, operands in registers.
__global__ __launch_bounds__(512) void probe_mfma_kernel(float* __restrict__ sink, int iters) {
  bf16x8p a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.001f * (float)(threadIdx.x + i));
    b[i] = (__bf16)(0.002f * (float)((int)threadIdx.x - i));
  }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop alive; never true in practice
}

// one 16-byte store per thread, in address order
__global__ __launch_bounds__(256) void probe_fill_kernel(f32x4* __restrict__ dst, int64_t units) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < units) dst[i] = f32x4{1.0f, 2.0f, 3.0f, 4.0f};
}

// eight 16-byte loads per thread, all issued before the first use; a workgroup reads 32 KB in address order
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, uint32_t* __restrict__ sink) {
  const u32x4* p = src + (int64_t)blockIdx.x * 2048 + threadIdx.x;
  u32x4 q[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) q[k] = __builtin_nontemporal_load(p + k * 256);
  u32x4 x = q[0];
#pragma unroll
  for (int k = 1; k < 8; ++k) x ^= q[k];
  if ((x.x ^ x.y ^ x.z ^ x.w) == 0x9e3779b9u) sink[0] = 1u;   // keeps the loads alive; the caller's data never gives this
}

// Every workgroup (8 wavefronts) streams tiles of 128 rows x 128 bytes (row pitch `pitch`) straight into a
// ring of four 16 KB LDS stages, advancing 128 bytes along the rows per step: the access shape of an
// operand tile of the whole-tile GEMM core.  All workgroups read the same window, so after the first pass
// the loads are L2 hits.
__global__ __launch_bounds__(512) void probe_fetch_kernel(const char* __restrict__ src, int64_t pitch, int steps) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[4 * 16384];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned lds0 = __builtin_amdgcn_readfirstlane(
      (unsigned)(size_t)((__attribute__((address_space(3))) void*)lds) + wave * 1024);
  const char* p[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) p[j] = src + (int64_t)(8 * (wave + 8 * j) + (lane >> 3)) * pitch + (lane & 7) * 16;
  for (int s = 0; s < steps; ++s) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      unsigned saved_m0;   // M0 is the compiler's register: put back before the statement ends
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %1, off\n\ts_nop 0\n\ts_mov_b32 m0, %0"
                   : "=&s"(saved_m0)
                   : "v"(p[j]), "s"(lds0 + (s & 3) * 16384 + 8 * j * 1024)
                   : "memory");
      p[j] += 128;
    }
    if ((s & 3) == 3) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

// What a lone wavefront hides behind its own MFMAs: 256 workgroups of 4 wavefronts (one per SIMD),
// each looping over two independent 32x32x16 bf16 MFMAs with NV vector-ALU additions or NL 4-byte LDS
// reads after each of them.  The time of a launch over 2 * iters is the time per MFMA.
template <int NV, int NL>
__global__ __launch_bounds__(256) void probe_beside_kernel(float* __restrict__ sink, int iters) {
  __shared__ uint32_t lds[4096];
  const int tid = threadIdx.x;
  for (int i = tid; i < 4096; i += 256) lds[i] = (uint32_t)i;
  __syncthreads();
  // two sums that differ (operands and start), so that neither can stand in for the other
  bf16x8p a, b, a1, b1;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.001f * (float)(tid + i));
    b[i] = (__bf16)(0.002f * (float)(tid - i));
    a1[i] = (__bf16)(0.003f * (float)(tid + 2 * i));
    b1[i] = (__bf16)(0.001f * (float)(3 * i - tid));
  }
  f32x16 c0 = {0}, c1 = {0};
  c1[0] = 1.0f;
  uint32_t x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = (uint32_t)(tid + i);
  const uint32_t one = 1u;
  auto others = [&]() {
#pragma unroll
    for (int i = 0; i < NV; ++i) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x[i & 7]) : "v"(one));
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      uint32_t r;
      asm volatile("ds_read_b32 %0, %1" : "=v"(r) : "v"((uint32_t)(tid * 4 + i * 1024)) : "memory");
      asm volatile("" ::"v"(r));
    }
  };
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    others();
    __builtin_amdgcn_sched_barrier(0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, c1, 0, 0, 0);
    others();
    __builtin_amdgcn_sched_barrier(0);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i];
  uint32_t xs = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) xs ^= x[i];
  if (s == 12345.678f) sink[0] = s + (float)xs;   // keeps the loop alive; never true in practice
}

}  // namespace synk

using namespace synk;

extern "C" int synk_probe_launch(int probe, void* buf, size_t buf_bytes, int iters, double* work, void* stream) {
  if (!buf || !work) return SYNK_ERR_NULL;
  if (iters < 1 || !aligned_to(buf, 16)) return SYNK_ERR_SHAPE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (probe == SYNK_PROBE_MFMA_BF16) {
    if (buf_bytes < 4) return SYNK_ERR_WORKSPACE;
    const int blocks = 2 * kNumCU;   // 16 wavefronts a CU
    SYNK_LAUNCH_TIMED(probe_mfma_kernel, dim3(blocks), dim3(512), 0, s, reinterpret_cast<float*>(buf), iters);
    *work = (double)blocks * 8.0 * (double)iters * 4.0 * 32768.0;          // flops
  } else if (probe == SYNK_PROBE_FILL) {
    const int64_t units = (int64_t)(buf_bytes / 16);
    if (units < 1 || units > (int64_t)0x7fffffff * 256) return SYNK_ERR_SHAPE;
    SYNK_LAUNCH_TIMED(probe_fill_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s,
                      reinterpret_cast<f32x4*>(buf), units);
    *work = (double)units * 16.0;                                          // bytes stored
  } else if (probe == SYNK_PROBE_LDS_FETCH) {
    // window: 128 rows at a pitch of 6 KB (the wide configuration's row), iters steps of 128 bytes along them
    const int64_t pitch = 6144;
    if (iters > 48 || buf_bytes < (size_t)(128 * pitch)) return SYNK_ERR_WORKSPACE;
    SYNK_LAUNCH_TIMED(probe_fetch_kernel, dim3(kNumCU), dim3(512), 0, s, reinterpret_cast<const char*>(buf), pitch, iters);
    *work = (double)kNumCU * (double)iters * 16384.0;                      // bytes brought into LDS
  } else if (probe == SYNK_PROBE_READ) {
    const int64_t blocks = (int64_t)(buf_bytes / 32768);
    if (blocks < 1 || blocks > 0x7fffffff) return SYNK_ERR_SHAPE;
    SYNK_LAUNCH_TIMED(probe_read_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                      reinterpret_cast<const u32x4*>(buf), reinterpret_cast<uint32_t*>(buf));
    *work = (double)blocks * 32768.0;                                      // bytes loaded
  } else if (probe >= SYNK_PROBE_MFMA_BESIDE_VALU && probe < SYNK_PROBE_MFMA_BESIDE_LDS + 16) {
    if (buf_bytes < 4) return SYNK_ERR_WORKSPACE;
    float* sink = reinterpret_cast<float*>(buf);
    const dim3 grid(kNumCU), block(256);
#define SYNK_BESIDE(NV, NL) SYNK_LAUNCH_TIMED((probe_beside_kernel<NV, NL>), grid, block, 0, s, sink, iters)
    switch (probe) {
      case SYNK_PROBE_MFMA_BESIDE_VALU + 0: SYNK_BESIDE(0, 0); break;
      case SYNK_PROBE_MFMA_BESIDE_VALU + 1: SYNK_BESIDE(1, 0); break;
      case SYNK_PROBE_MFMA_BESIDE_VALU + 2: SYNK_BESIDE(2, 0); break;
      case SYNK_PROBE_MFMA_BESIDE_VALU + 4: SYNK_BESIDE(4, 0); break;
      case SYNK_PROBE_MFMA_BESIDE_VALU + 6: SYNK_BESIDE(6, 0); break;
      case SYNK_PROBE_MFMA_BESIDE_VALU + 8: SYNK_BESIDE(8, 0); break;
      case SYNK_PROBE_MFMA_BESIDE_VALU + 12: SYNK_BESIDE(12, 0); break;
      case SYNK_PROBE_MFMA_BESIDE_LDS + 1: SYNK_BESIDE(0, 1); break;
      case SYNK_PROBE_MFMA_BESIDE_LDS + 2: SYNK_BESIDE(0, 2); break;
      case SYNK_PROBE_MFMA_BESIDE_LDS + 4: SYNK_BESIDE(0, 4); break;
      default: return SYNK_ERR_UNSUPPORTED;
    }
#undef SYNK_BESIDE
    *work = (double)kNumCU * 4.0 * (double)iters * 2.0 * 32768.0;         // flops
  } else {
    return SYNK_ERR_UNSUPPORTED;
  }
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}
