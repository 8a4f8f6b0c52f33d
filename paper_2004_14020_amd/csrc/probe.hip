// Plain streaming kernels of known size, for measurement only: ceilings to set the reduce kernels
// against, and kernels whose HBM traffic is known exactly, to check what the profiler's counters
// report.  No descriptor tables: workgroup b handles run b of every buffer.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "caramel.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
#define PROBE_GLOBAL __attribute__((address_space(1)))
typedef PROBE_GLOBAL u32x4* gvec_ptr;

struct Buffers {
  uint64_t p[16];
};

// READ: every vector of every buffer is loaded (the sum is stored only if it is a value no input
// produces, i.e. never, so the loads stay).  WRITE: every vector is stored.  UPDATE: every
// vector of all W buffers is loaded, the W values are added, and the sum is stored to all W
// buffers -- the reduce kernel's traffic without its tables.  COPY: buffer 0 to buffer 1.
template <int W, int MODE>
__global__ void __launch_bounds__(1024)
k_probe(Buffers b, uint64_t n_vec, uint32_t run_vecs) {
  const uint64_t first = uint64_t(blockIdx.x) * run_vecs;
  const uint64_t last = first + run_vecs < n_vec ? first + run_vecs : n_vec;
  for (uint64_t v = first + threadIdx.x; v < last; v += blockDim.x) {
    if constexpr (MODE == CARAMEL_PROBE_WRITE) {
      const u32x4 y = {uint32_t(v), 1u, 2u, 3u};
#pragma unroll
      for (int w = 0; w < W; ++w) __builtin_nontemporal_store(y, reinterpret_cast<gvec_ptr>(b.p[w]) + v);
    } else if constexpr (MODE == CARAMEL_PROBE_COPY) {
      __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<gvec_ptr>(b.p[0]) + v),
                                  reinterpret_cast<gvec_ptr>(b.p[1]) + v);
    } else {
      u32x4 x[W];
#pragma unroll
      for (int w = 0; w < W; ++w) x[w] = __builtin_nontemporal_load(reinterpret_cast<gvec_ptr>(b.p[w]) + v);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (MODE == CARAMEL_PROBE_READ) {
        u32x4 acc = x[0];
#pragma unroll
        for (int w = 1; w < W; ++w) acc = acc ^ x[w];
        if (acc.x == 0x7FC12345u && acc.y == 0x7FC54321u && acc.z == acc.w)
          __builtin_nontemporal_store(acc, reinterpret_cast<gvec_ptr>(b.p[0]) + v);
      } else {
        f32x4 acc = __builtin_bit_cast(f32x4, x[0]);
#pragma unroll
        for (int w = 1; w < W; ++w) acc = acc + __builtin_bit_cast(f32x4, x[w]);
        const u32x4 y = __builtin_bit_cast(u32x4, acc * (1.0f / W));
#pragma unroll
        for (int w = 0; w < W; ++w) __builtin_nontemporal_store(y, reinterpret_cast<gvec_ptr>(b.p[w]) + v);
      }
    }
  }
}

template <int W>
hipError_t launch(uint32_t mode, const Buffers& b, uint64_t n_vec, uint32_t run_vecs, uint32_t block, hipStream_t s) {
  const dim3 grid(uint32_t((n_vec + run_vecs - 1) / run_vecs));
  switch (mode) {
    case CARAMEL_PROBE_READ: hipLaunchKernelGGL((k_probe<W, CARAMEL_PROBE_READ>), grid, dim3(block), 0, s, b, n_vec, run_vecs); break;
    case CARAMEL_PROBE_WRITE: hipLaunchKernelGGL((k_probe<W, CARAMEL_PROBE_WRITE>), grid, dim3(block), 0, s, b, n_vec, run_vecs); break;
    case CARAMEL_PROBE_UPDATE: hipLaunchKernelGGL((k_probe<W, CARAMEL_PROBE_UPDATE>), grid, dim3(block), 0, s, b, n_vec, run_vecs); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

extern "C" int caramel_stream_probe(uint32_t mode, void* const* buffers, uint32_t n_buffers, uint64_t bytes,
                                    uint32_t run_bytes, uint32_t block, void* stream) {
  if (!buffers || bytes == 0 || bytes % 16 || run_bytes == 0 || run_bytes % 16) return CARAMEL_EINVAL;
  if (block != 256 && block != 512 && block != 1024) return CARAMEL_EINVAL;
  const uint64_t n_vec = bytes / 16;
  if ((n_vec + run_bytes / 16 - 1) / (run_bytes / 16) > 0x7FFFFFFFull) return CARAMEL_EINVAL;
  Buffers b{};
  if (n_buffers > 16) return CARAMEL_EINVAL;
  for (uint32_t w = 0; w < n_buffers; ++w) {
    if (!buffers[w] || reinterpret_cast<uint64_t>(buffers[w]) % 16) return CARAMEL_EINVAL;
    b.p[w] = reinterpret_cast<uint64_t>(buffers[w]);
  }
  hipStream_t s = hipStream_t(stream);
  hipError_t e = hipErrorInvalidValue;
  if (mode == CARAMEL_PROBE_COPY) {
    if (n_buffers != 2) return CARAMEL_EINVAL;
    const dim3 grid(uint32_t((n_vec + run_bytes / 16 - 1) / (run_bytes / 16)));
    hipLaunchKernelGGL((k_probe<2, CARAMEL_PROBE_COPY>), grid, dim3(block), 0, s, b, n_vec, run_bytes / 16);
    e = hipGetLastError();
  } else {
    switch (n_buffers) {
      case 1: e = launch<1>(mode, b, n_vec, run_bytes / 16, block, s); break;
      case 2: e = launch<2>(mode, b, n_vec, run_bytes / 16, block, s); break;
      case 4: e = launch<4>(mode, b, n_vec, run_bytes / 16, block, s); break;
      case 8: e = launch<8>(mode, b, n_vec, run_bytes / 16, block, s); break;
      case 16: e = launch<16>(mode, b, n_vec, run_bytes / 16, block, s); break;
      default: return CARAMEL_EINVAL;
    }
  }
  return e == hipSuccess ? CARAMEL_OK : CARAMEL_EHIP;
}
