// Measurement helpers: what the GPU reaches on HBM reads and on bf16 MFMAs (see xy_attn.h).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "xy_probe.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <bool ONCE>      // ONCE: loads with the non-temporal hint, as the bandwidth-bound units of the attention kernel issue them
__device__ __forceinline__ uint4 load16(const uint4* p) {
  if (ONCE) {
    const unsigned* w = reinterpret_cast<const unsigned*>(p);
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(w));
    return uint4{v[0], v[1], v[2], v[3]};
  }
  return *p;
}

template <bool ONCE>
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                          unsigned* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  unsigned acc = 0;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {          // four loads in flight per thread
    const uint4 a = load16<ONCE>(src + i), b = load16<ONCE>(src + i + stride), c = load16<ONCE>(src + i + 2 * stride),
                d = load16<ONCE>(src + i + 3 * stride);
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const uint4 a = load16<ONCE>(src + i);
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9e3779b9u) atomicXor(sink, acc);           // practically never: keeps the loads alive
}

__global__ __launch_bounds__(512) void mfma_kernel(int iters, unsigned* __restrict__ sink) {
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.001f * (threadIdx.x + i));
    b[i] = (__bf16)(0.5f - 0.01f * i);
  }
  f32x16 acc[4];
  for (int j = 0; j < 4; ++j)
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  for (int it = 0; it < iters; ++it)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j & 3], 0, 0, 0);
  float s = 0.f;
  for (int j = 0; j < 4; ++j) s += acc[j][0] + acc[j][15];
  if (s == 123.456f) atomicXor(sink, 1u);
}

// One wavefront per SIMD issues iters x 32 MFMAs with the instructions of MIX between them and reports the
// cycles it took.  96 KB of LDS per workgroup keep a second workgroup off the CU.
template <int MIX>
__global__ __launch_bounds__(256) void issue_mix_kernel(int iters, unsigned long long* __restrict__ cycles,
                                                        unsigned* __restrict__ sink) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[96 * 1024];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < (int)sizeof(lds) / 4; i += 256) reinterpret_cast<float*>(lds)[i] = (float)i;
  __syncthreads();
  float x[16];
  for (int i = 0; i < 16; ++i) x[i] = lane * 0.001f + i;
  f32x16 acc[8];
  for (int i = 0; i < 8; ++i)
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(lane * 0.001f + i);
    b[i] = (__bf16)(0.5f - i);
  }
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  f32x4 frag[8];
  for (int i = 0; i < 8; ++i) frag[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  const unsigned addr = (unsigned)(size_t)((__attribute__((address_space(3))) unsigned char*)lds) + wave * 16384 + lane * 16;
  int sc = 0;
  const long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i % 8]) : "v"(a), "v"(b));
      auto fma = [&](const int n) {
#pragma unroll
        for (int j = 0; j < n; ++j)
          asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[(i * 5 + j) & 15]) : "v"(x[(i + j + 7) & 15]), "v"(1.0f));
      };
      if (MIX == XY_MIX_EVEN_4) fma(4);
      if (MIX == XY_MIX_UNEVEN_8_0 && (i & 1) == 0) fma(8);
      if (MIX == XY_MIX_DOT2) asm volatile("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(x[i & 15]) : "v"(x[(i + 7) & 15]), "v"(x[(i + 3) & 15]));
      if (MIX == XY_MIX_SCALAR_2) {
        fma(3);
        asm volatile("s_add_u32 %0, %0, 1\n\ts_add_u32 %0, %0, 1" : "+s"(sc) : : "scc");
      }
      if (MIX == XY_MIX_ATTENTION) {
        asm volatile("v_exp_f32 %0, %0" : "+v"(x[i & 15]));
        fma(2);
        if ((i & 3) != 3)
          asm volatile("ds_read_b128 %0, %1 offset:1024" : "=v"(frag[(i & 3) + 4 * ((i >> 2) & 1)]) : "v"(addr) : "memory");
        else
          asm volatile("s_waitcnt lgkmcnt(3)" : "+v"(frag[0]), "+v"(frag[1]), "+v"(frag[2]), "+v"(frag[3]), "+v"(frag[4]), "+v"(frag[5]), "+v"(frag[6]), "+v"(frag[7]) : : "memory");
      }
    }
  }
  const long long t1 = clock64();
  float s = (float)sc;
  for (int i = 0; i < 16; ++i) s += x[i];
  for (int i = 0; i < 8; ++i) s += acc[i][0] + frag[i][0];
  if (s == 123.456f) atomicXor(sink, 1u);
  if (lane == 0) cycles[blockIdx.x * 4 + wave] = (unsigned long long)(t1 - t0);
}

}  // namespace

extern "C" int xy_probe_issue_mix(int32_t mix, int32_t iters, void* cycles, void* sink, void* hip_stream) {
  if (iters < 1 || !cycles || !sink || ((uintptr_t)cycles & 7)) return XY_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned long long* out = static_cast<unsigned long long*>(cycles);
  unsigned* sk = static_cast<unsigned*>(sink);
  switch (mix) {
    case XY_MIX_NONE: hipLaunchKernelGGL(issue_mix_kernel<XY_MIX_NONE>, dim3(256), dim3(256), 0, st, iters, out, sk); break;
    case XY_MIX_EVEN_4: hipLaunchKernelGGL(issue_mix_kernel<XY_MIX_EVEN_4>, dim3(256), dim3(256), 0, st, iters, out, sk); break;
    case XY_MIX_UNEVEN_8_0: hipLaunchKernelGGL(issue_mix_kernel<XY_MIX_UNEVEN_8_0>, dim3(256), dim3(256), 0, st, iters, out, sk); break;
    case XY_MIX_DOT2: hipLaunchKernelGGL(issue_mix_kernel<XY_MIX_DOT2>, dim3(256), dim3(256), 0, st, iters, out, sk); break;
    case XY_MIX_SCALAR_2: hipLaunchKernelGGL(issue_mix_kernel<XY_MIX_SCALAR_2>, dim3(256), dim3(256), 0, st, iters, out, sk); break;
    case XY_MIX_ATTENTION: hipLaunchKernelGGL(issue_mix_kernel<XY_MIX_ATTENTION>, dim3(256), dim3(256), 0, st, iters, out, sk); break;
    default: return XY_ERR_ARG;
  }
  return hipGetLastError() == hipSuccess ? XY_OK : XY_ERR_HIP;
}

extern "C" int xy_probe_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink || (bytes & 15) || ((uintptr_t)src & 15)) return XY_ERR_ARG;
  if (bytes == 0) return XY_OK;
  hipLaunchKernelGGL(stream_read_kernel<false>, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(src), bytes / 16, static_cast<unsigned*>(sink));
  return hipGetLastError() == hipSuccess ? XY_OK : XY_ERR_HIP;
}

extern "C" int xy_probe_stream_read_once(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink || (bytes & 15) || ((uintptr_t)src & 15)) return XY_ERR_ARG;
  if (bytes == 0) return XY_OK;
  hipLaunchKernelGGL(stream_read_kernel<true>, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(src), bytes / 16, static_cast<unsigned*>(sink));
  return hipGetLastError() == hipSuccess ? XY_OK : XY_ERR_HIP;
}

extern "C" int xy_probe_mfma(int32_t iters, void* sink, void* hip_stream) {
  if (iters < 1 || !sink) return XY_ERR_ARG;
  hipLaunchKernelGGL(mfma_kernel, dim3(256), dim3(512), 0, static_cast<hipStream_t>(hip_stream), iters,
                     static_cast<unsigned*>(sink));
  return hipGetLastError() == hipSuccess ? XY_OK : XY_ERR_HIP;
}
