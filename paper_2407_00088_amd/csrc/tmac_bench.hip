// Measurement helpers: a plain streaming-read kernel, the "what can a read-only kernel reach on
// this chip" reference that the benchmark prints next to the lookup kernels, and a probe of the
// LDS lookup rate, a probe of the vector-instruction issue rate, and an empty kernel; none takes part in the mpGEMM path (they are built into a
// library of their own, libtmac_bench.so).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "tmac_bench.h"

namespace tmac_bench {

typedef uint32_t ru32x4 __attribute__((ext_vector_type(4)));

// Every thread reads PER_THREAD 16-byte pieces, one per "wave row" of the block's span, so that a
// wavefront always reads 1 KB contiguous; all loads are issued before the first use.
template <int PER_THREAD, bool NONTEMPORAL>
__global__ __launch_bounds__(256) void stream_read_kernel(const ru32x4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
  const size_t base = (size_t)blockIdx.x * (256 * PER_THREAD) + threadIdx.x;
  ru32x4 v[PER_THREAD];
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i) {
    const size_t j = base + (size_t)i * 256;
    const size_t jc = j < n16 ? j : n16 - 1;
    v[i] = NONTEMPORAL ? __builtin_nontemporal_load(src + jc) : src[jc];
  }
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  // data-dependent store that practically never happens keeps the loads alive
  if (acc == 0x9E3779B9u) sink[blockIdx.x & 63] = acc;
}

// Measurement helper: the lookup rate of LDS alone.  A workgroup holds 32 KB of tables laid out as
// the batched kernels keep them (256-byte tables of sixteen 16-byte entries: eight activation
// rows side by side) and every lane reads entries at data-dependent offsets, sixteen reads in
// flight, with the address arithmetic of those kernels (one byte permute per read) and nothing
// done with the values.  One read of a wavefront serves 64 lanes x 8 rows = 512 lookups.
typedef __attribute__((address_space(3))) ru32x4 probe_lds_u32x4;
__global__ __launch_bounds__(256) void lds_lookup_probe_kernel(int rounds, uint32_t* __restrict__ sink) {
  __shared__ __attribute__((aligned(2048))) char tab[32768];
  for (int i = threadIdx.x; i < 32768 / 16; i += 256)
    reinterpret_cast<ru32x4*>(tab)[i] = ru32x4{(uint32_t)i, (uint32_t)i * 3u, (uint32_t)i * 5u, (uint32_t)i * 7u};
  __syncthreads();
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)tab);
  uint32_t x = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
  uint32_t keep = 0;
  for (int r = 0; r < rounds; ++r) {
    x = x * 1664525u + 1013904223u;                       // two index dwords (two bit planes): eight 4-bit indices each
    const uint32_t x2 = x * 22695477u + 1u;
    const uint32_t cbase = lds0 + (uint32_t)(r & 15) * 2048u;  // the chunk's eight tables
    const uint32_t off[4] = {(x << 4) & 0xF0F0F0F0u, x & 0xF0F0F0F0u, (x2 << 4) & 0xF0F0F0F0u, x2 & 0xF0F0F0F0u};
    ru32x4 e[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      // address = {0, cbase byte 2, cbase byte 1, one byte of the offsets}; table j % 8 of the chunk
      const uint32_t a = __builtin_amdgcn_perm(off[2 * (j >> 3) + (j & 1)], cbase, 0x0C020100u + 4u + (uint32_t)((j >> 1) & 3));
      e[j] = *reinterpret_cast<probe_lds_u32x4*>(a + (j & 7) * 256);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) asm volatile("" ::"v"(e[j]));  // the values are "used": no instruction
    keep += x >> 31;
  }
  if (keep == 0xFFFFFFFFu) sink[blockIdx.x & 63] = keep;  // practically never; keeps the loop alive
}

__global__ void empty_kernel() {}

// Measurement helper: how fast a SIMD issues the vector instructions the register-table lookups are
// made of.  Every lane runs `iters` x 64 instructions of one kind on eight independent registers
// (KIND 0: v_and_b32, 1: v_perm_b32, 2: v_dot2c_f32_f16), or `iters` x 8 times the lookup sequence
// of one index dword (KIND 3: 17 instructions: rotation, two masks, two sign XORs, four lookup
// permutes, four re-interleave permutes, four dot products, in the order the compiler emits them).
// The caller picks the number of workgroups of 256 lanes, i.e. wavefronts per SIMD.
template <int KIND>
__global__ __launch_bounds__(256) void valu_rate_probe_kernel(int iters, uint32_t* __restrict__ sink) {
  uint32_t a[8];
  float f[8];
  const uint32_t t = threadIdx.x * 2654435761u + blockIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = t + (uint32_t)i * 0x01020304u; f[i] = (float)i; }
  const uint32_t lo0 = t ^ 0x55aa55aau, lo1 = t * 3u, hi0 = t * 5u, hi1 = t * 7u;
  uint32_t c78 = 0x80808080u, c1 = 0x05010400u, c2 = 0x07030602u;
  asm volatile("" : "+s"(c78), "+s"(c1), "+s"(c2));
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      if constexpr (KIND == 3) {
        uint32_t x = a[r], s, l, h, p, q, xr;
        asm volatile(
            "v_and_b32 %1, 0x7070707, %0\n v_perm_b32 %2, %8, %7, %1\n v_perm_b32 %3, %10, %9, %1\n"
            "v_bitop3_b32 %3, %3, %0, %11 bitop3:0x78\n v_perm_b32 %4, %3, %2, %12\n v_perm_b32 %5, %3, %2, %13\n"
            "v_dot2c_f32_f16 %14, %4, %16\n v_dot2c_f32_f16 %14, %5, %17\n"
            "v_alignbit_b32 %6, %0, %0, 4\n"
            "v_and_b32 %1, 0x7070707, %6\n v_perm_b32 %2, %8, %7, %1\n v_perm_b32 %3, %10, %9, %1\n"
            "v_bitop3_b32 %3, %3, %6, %11 bitop3:0x78\n v_perm_b32 %4, %3, %2, %12\n v_perm_b32 %5, %3, %2, %13\n"
            "v_dot2c_f32_f16 %15, %4, %16\n v_dot2c_f32_f16 %15, %5, %17\n"
            : "+v"(x), "=&v"(s), "=&v"(l), "=&v"(h), "=&v"(p), "=&v"(q), "=&v"(xr)
            : "v"(lo0), "v"(lo1), "v"(hi0), "v"(hi1), "s"(c78), "s"(c1), "s"(c2), "v"(f[r]), "v"(f[(r + 1) & 7]), "v"(lo0),
              "v"(hi1));
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if constexpr (KIND == 0) asm volatile("v_and_b32 %0, %0, %1" : "+v"(a[i]) : "v"(lo1));
          else if constexpr (KIND == 1) asm volatile("v_perm_b32 %0, %1, %0, %2" : "+v"(a[i]) : "v"(lo0), "v"(lo1));
          else asm volatile("v_dot2c_f32_f16 %0, %1, %2" : "+v"(f[i]) : "v"(lo1), "v"(lo0));
        }
      }
    }
  }
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) acc ^= a[i] ^ __float_as_uint(f[i]);
  if (acc == 0x12345678u) sink[blockIdx.x & 63] = acc;  // practically never; keeps the loop alive
}

}  // namespace tmac_bench

using namespace tmac_bench;

extern "C" int tmac_bench_lds_lookup_probe(int32_t workgroups, int32_t rounds, void* sink_dev, void* stream) {
  if (!sink_dev || workgroups <= 0 || rounds <= 0 || rounds > (1 << 24)) return 1;
  uint32_t* sink = static_cast<uint32_t*>(sink_dev);
  int r = rounds;
  void* args[] = {&r, &sink};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(lds_lookup_probe_kernel), dim3((unsigned)workgroups),
                                       dim3(256), args, 0, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) {
    return 4;
  }
  return 0;
}

extern "C" int tmac_bench_stream_read(const void* src_dev, size_t bytes, void* sink_dev, int32_t per_thread,
                                        int32_t nontemporal, void* stream) {
  if (!src_dev || !sink_dev || bytes < 16 || (reinterpret_cast<uintptr_t>(src_dev) & 15u)) return 1;
  const size_t n16 = bytes / 16;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const ru32x4* src = static_cast<const ru32x4*>(src_dev);
  uint32_t* sink = static_cast<uint32_t*>(sink_dev);
  void* args[] = {&src, const_cast<size_t*>(&n16), &sink};
  const void* fn = nullptr;
  int pt = per_thread;
  switch (per_thread * 2 + (nontemporal ? 1 : 0)) {
    case 2: fn = reinterpret_cast<const void*>(stream_read_kernel<1, false>); break;
    case 3: fn = reinterpret_cast<const void*>(stream_read_kernel<1, true>); break;
    case 8: fn = reinterpret_cast<const void*>(stream_read_kernel<4, false>); break;
    case 9: fn = reinterpret_cast<const void*>(stream_read_kernel<4, true>); break;
    case 16: fn = reinterpret_cast<const void*>(stream_read_kernel<8, false>); break;
    case 17: fn = reinterpret_cast<const void*>(stream_read_kernel<8, true>); break;
    default: return 1;
  }
  const size_t per_block = (size_t)256 * pt;
  const size_t blocks = (n16 + per_block - 1) / per_block;
  if (blocks > 0x7fffffffu) return 2;
  const hipError_t e = hipLaunchKernel(fn, dim3((unsigned)blocks), dim3(256), args, 0, st);
  if (e != hipSuccess) {
    return 4;
  }
  return 0;
}

extern "C" int tmac_bench_valu_rate_probe(int32_t kind, int32_t workgroups, int32_t iters, void* sink_dev, void* stream) {
  if (!sink_dev || workgroups <= 0 || iters <= 0 || iters > (1 << 24) || kind < 0 || kind > 3) return 1;
  uint32_t* sink = static_cast<uint32_t*>(sink_dev);
  int it = iters;
  void* args[] = {&it, &sink};
  const void* fn = kind == 0   ? reinterpret_cast<const void*>(valu_rate_probe_kernel<0>)
                   : kind == 1 ? reinterpret_cast<const void*>(valu_rate_probe_kernel<1>)
                   : kind == 2 ? reinterpret_cast<const void*>(valu_rate_probe_kernel<2>)
                               : reinterpret_cast<const void*>(valu_rate_probe_kernel<3>);
  const hipError_t e = hipLaunchKernel(fn, dim3((unsigned)workgroups), dim3(256), args, 0, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? 0 : 4;
}

extern "C" int tmac_bench_empty_kernel(void* stream) {
  void* args[] = {nullptr};  // no parameters
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(empty_kernel), dim3(1), dim3(64), args, 0,
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? 0 : 4;
}
