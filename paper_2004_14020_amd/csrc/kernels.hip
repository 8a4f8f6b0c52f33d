// gfx950 kernels of the aggregation path.  Everything here is bandwidth work: 128-bit
// coalesced loads and stores, no matrix cores.
//
//  k_ring_reduce   ring reduce-scatter arithmetic, 1/W scaling and all-gather (paper
//                  sections 2 and 4.4: partial sums travel round the ring and are added to
//                  at each worker; the owner's result is then copied to every worker).
//                  A workgroup handles one tile, which lies inside one ring segment, so the
//                  chain of workers  first, first+1, ...  is the same for all lanes and the
//                  W base pointers live in scalar registers.
//  k_copy          pack / unpack of batched parameters (section 4.2) through an offset table,
//                  one workgroup per run of at most 16 KiB.
#include "kernels.hpp"

#include <type_traits>

namespace caramel {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// Pointers built from table entries are declared as global-memory pointers so that loads and
// stores use the global (scalar base + lane offset) form rather than the generic one.
#define CARAMEL_GLOBAL __attribute__((address_space(1)))
typedef CARAMEL_GLOBAL u32x4* gvec_ptr;
typedef CARAMEL_GLOBAL float* gf32_ptr;
typedef CARAMEL_GLOBAL uint16_t* gu16_ptr;
typedef CARAMEL_GLOBAL uint32_t* gu32_ptr;

constexpr int kCopyBlock = 1024;  // pack / unpack workgroup
constexpr int kMaxBlock = 1024;  // ring-reduce workgroups are 256, 512 or 1024 lanes

template <bool NT>
__device__ __forceinline__ u32x4 ld(gvec_ptr p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT>
__device__ __forceinline__ void st(gvec_ptr p, u32x4 v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// scalar base + 32-bit lane byte offset
__device__ __forceinline__ gvec_ptr at(gvec_ptr base, uint32_t byte_off) {
  return reinterpret_cast<gvec_ptr>(reinterpret_cast<CARAMEL_GLOBAL char*>(base) + byte_off);
}

__device__ __forceinline__ f32x4 bits_to_f32(u32x4 v) { return __builtin_bit_cast(f32x4, v); }
__device__ __forceinline__ u32x4 f32_to_bits(f32x4 v) { return __builtin_bit_cast(u32x4, v); }

// fp32 -> bf16, round to nearest, ties to even; NaN stays a (quiet) NaN.
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t b = __float_as_uint(f);
  const uint32_t r = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
  return (f != f) ? ((b >> 16) | 0x40u) : r;
}

// Running ring sum of one 16-byte vector.  F32: four lanes.  BF16: eight values, kept as the
// even-indexed (low halves) and odd-indexed (high halves) quartets, widened exactly.
template <bool BF16>
struct Chain {
  f32x4 a, b;
  __device__ __forceinline__ void start(u32x4 x) {
    if constexpr (BF16) {
      a = bits_to_f32(x << 16);
      b = bits_to_f32(x & 0xFFFF0000u);
    } else {
      a = bits_to_f32(x);
    }
  }
  __device__ __forceinline__ void add(u32x4 x) {
    if constexpr (BF16) {
      a = a + bits_to_f32(x << 16);
      b = b + bits_to_f32(x & 0xFFFF0000u);
    } else {
      a = a + bits_to_f32(x);
    }
  }
  // this partial sum + another one
  __device__ __forceinline__ void merge(const Chain& o) {
    a = a + o.a;
    if constexpr (BF16) b = b + o.b;
  }
  // becomes `o` in the lanes where `c` holds (a select on the bits: no arithmetic)
  __device__ __forceinline__ void take_if(bool c, const Chain& o) {
    a.x = c ? o.a.x : a.x;
    a.y = c ? o.a.y : a.y;
    a.z = c ? o.a.z : a.z;
    a.w = c ? o.a.w : a.w;
    if constexpr (BF16) {
      b.x = c ? o.b.x : b.x;
      b.y = c ? o.b.y : b.y;
      b.z = c ? o.b.z : b.z;
      b.w = c ? o.b.w : b.w;
    }
  }
  __device__ __forceinline__ u32x4 finish(float inv_w) {
    if constexpr (BF16) {
      const f32x4 ya = a * inv_w, yb = b * inv_w;
      u32x4 r;
      r.x = bf16_rne(ya.x) | (bf16_rne(yb.x) << 16);
      r.y = bf16_rne(ya.y) | (bf16_rne(yb.y) << 16);
      r.z = bf16_rne(ya.z) | (bf16_rne(yb.z) << 16);
      r.w = bf16_rne(ya.w) | (bf16_rne(yb.w) << 16);
      return r;
    } else {
      return f32_to_bits(a * inv_w);
    }
  }
};

// Sum of the W vectors x[0..W-1] in the order of the pattern, scaled and converted back.
// Chain: ((x0 + x1) + x2) + ...   Tree: neighbours first, then pairs of pairs, ...
template <int W, bool BF16, bool TREE>
__device__ __forceinline__ u32x4 combine(const u32x4 (&x)[W], float inv_w) {
  if constexpr (!TREE) {
    Chain<BF16> c;
    c.start(x[0]);
#pragma unroll
    for (int k = 1; k < W; ++k) c.add(x[k]);
    return c.finish(inv_w);
  } else {
    Chain<BF16> part[W];
#pragma unroll
    for (int k = 0; k < W; ++k) part[k].start(x[k]);
#pragma unroll
    for (int s = 1; s < W; s *= 2)
#pragma unroll
      for (int i = 0; i + s < W; i += 2 * s) {
        part[i].a = part[i].a + part[i + s].a;
        if constexpr (BF16) part[i].b = part[i].b + part[i + s].b;
      }
    return part[0].finish(inv_w);
  }
}

// Same for one scalar element per worker.
template <int W, bool TREE>
__device__ __forceinline__ float combine_scalar(float (&v)[W], float inv_w) {
  if constexpr (!TREE) {
    float acc = v[0];
#pragma unroll
    for (int k = 1; k < W; ++k) acc = acc + v[k];
    return acc * inv_w;
  } else {
#pragma unroll
    for (int s = 1; s < W; s *= 2)
#pragma unroll
      for (int i = 0; i + s < W; i += 2 * s) v[i] = v[i] + v[i + s];
    return v[0] * inv_w;
  }
}

__device__ __forceinline__ float widen(uint16_t h) { return __uint_as_float(uint32_t(h) << 16); }

// ------------------------------------------------------------------------------------------
// W known at compile time: all W loads of a vector (times U vectors) are issued before the
// first add, so each lane keeps W*U 128-bit requests in flight.
template <int W, int U, bool BF16, bool NT, bool TREE>
__global__ void __launch_bounds__(kMaxBlock)
k_ring_reduce(const ReduceTile* __restrict__ tiles, const uint64_t* __restrict__ rows, uint32_t begin,
              uint32_t count, float inv_w) {
  constexpr uint32_t VE = BF16 ? 8 : 4;
  for (uint32_t ti = blockIdx.x; ti < count; ti += gridDim.x) {
    const ReduceTile tl = tiles[begin + ti];
    gvec_ptr p[W];
#pragma unroll
    for (int k = 0; k < W; ++k) {
      uint32_t w = tl.first + k;
      if (w >= uint32_t(W)) w -= W;
      p[k] = reinterpret_cast<gvec_ptr>(rows[size_t(tl.row) * W + w]) + tl.vec_off;
    }
    const uint32_t nvec = tl.n_elems / VE;
    const uint32_t B = blockDim.x;
    uint32_t v = threadIdx.x;
    // lane offsets are 32-bit byte offsets from the scalar bases (a tile spans < 2^24 bytes)
    for (; v + (U - 1) * B < nvec; v += U * B) {
      u32x4 x[U][W];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < W; ++k) x[u][k] = ld<NT>(at(p[k], (v + u * B) * 16u));
      __builtin_amdgcn_sched_barrier(0);  // keep all loads ahead of the arithmetic
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const u32x4 y = combine<W, BF16, TREE>(x[u], inv_w);
#pragma unroll
        for (int k = 0; k < W; ++k) st<NT>(at(p[k], (v + u * B) * 16u), y);
      }
    }
    for (; v < nvec; v += B) {
      u32x4 x[W];
#pragma unroll
      for (int k = 0; k < W; ++k) x[k] = ld<NT>(at(p[k], v * 16u));
      __builtin_amdgcn_sched_barrier(0);
      const u32x4 y = combine<W, BF16, TREE>(x, inv_w);
#pragma unroll
      for (int k = 0; k < W; ++k) st<NT>(at(p[k], v * 16u), y);
    }
    // a run that ends a tensor may stop inside a vector: finish it element by element
    const uint32_t rem = tl.n_elems - nvec * VE;
    if (threadIdx.x < rem) {
      const uint32_t e = nvec * VE + threadIdx.x;
      float v[W];
      if constexpr (BF16) {
#pragma unroll
        for (int k = 0; k < W; ++k) v[k] = widen(reinterpret_cast<gu16_ptr>(p[k])[e]);
        const uint16_t y = uint16_t(bf16_rne(combine_scalar<W, TREE>(v, inv_w)));
#pragma unroll
        for (int k = 0; k < W; ++k) reinterpret_cast<gu16_ptr>(p[k])[e] = y;
      } else {
#pragma unroll
        for (int k = 0; k < W; ++k) v[k] = reinterpret_cast<gf32_ptr>(p[k])[e];
        const float y = combine_scalar<W, TREE>(v, inv_w);
#pragma unroll
        for (int k = 0; k < W; ++k) reinterpret_cast<gf32_ptr>(p[k])[e] = y;
      }
    }
  }
}

// One stream-major pass over U vectors of this lane (B apart, starting at v): the chain is walked
// one worker at a time, with the loads of the next D - 1 workers in flight while the current
// worker's values are added.  (D = 2 everywhere: looking further ahead for short tiles, which
// have fewer vectors per lane, measured no faster.)
// RAGGED: the last of the U vectors may lie at or beyond nvec; such a lane reads the tile's last
// vector instead (no divergence among the loads) and stores nothing for it.
// TREE: the values are added as the balanced pairwise tree of the halving-doubling order instead of
// a chain: worker k's value is merged with the open partial sums the way a binary counter carries
// (one level per trailing one bit of k), which needs log2(W) partial sums per vector.
template <int W, int U, int D, bool BF16, bool NT, bool RAGGED, bool TREE = false>
__device__ __forceinline__ void sm_walk(const gvec_ptr (&p)[W], uint32_t v, uint32_t B, uint32_t nvec, float inv_w) {
  static_assert(D >= 2 && D <= W, "look-ahead between 2 and W workers");
  static_assert(!TREE || (W & (W - 1)) == 0, "the tree needs a power of two");
  constexpr int LEVELS = W >= 16 ? 4 : (W >= 8 ? 3 : (W >= 4 ? 2 : 1));
  u32x4 buf[D][U];
  Chain<BF16> acc[U];
  Chain<BF16> lvl[TREE ? LEVELS : 1][U];
  const bool last_ok = !RAGGED || v + (U - 1) * B < nvec;
  auto off = [&](int u) -> uint32_t {
    if (RAGGED && u == U - 1) return (last_ok ? v + (U - 1) * B : nvec - 1) * 16u;
    return (v + u * B) * 16u;
  };
#pragma unroll
  for (int k = 0; k < D - 1; ++k)
#pragma unroll
    for (int u = 0; u < U; ++u) buf[k][u] = ld<NT>(at(p[k], off(u)));
#pragma unroll
  for (int k = 0; k < W; ++k) {
    if (k + D - 1 < W) {
#pragma unroll
      for (int u = 0; u < U; ++u) buf[(k + D - 1) % D][u] = ld<NT>(at(p[k + D - 1], off(u)));
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (!TREE) {
        if (k == 0) acc[u].start(buf[k % D][u]);
        else acc[u].add(buf[k % D][u]);
      } else {
        acc[u].start(buf[k % D][u]);
        int j = 0;
#pragma unroll
        for (int m = k; m & 1; m >>= 1) {
          lvl[j][u].merge(acc[u]);  // the earlier partial sum + the later one
          acc[u] = lvl[j][u];
          ++j;
        }
        if (k + 1 < W) lvl[j][u] = acc[u];
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  u32x4 y[U];
#pragma unroll
  for (int u = 0; u < U; ++u) y[u] = acc[u].finish(inv_w);
  constexpr int SURE = RAGGED ? U - 1 : U;  // vectors that are stored by every lane
#pragma unroll
  for (int k = 0; k < W; ++k)
#pragma unroll
    for (int u = 0; u < SURE; ++u) st<NT>(at(p[k], off(u)), y[u]);
  if constexpr (RAGGED) {
    if (last_ok) {
#pragma unroll
      for (int k = 0; k < W; ++k) st<NT>(at(p[k], off(U - 1)), y[U - 1]);
    }
  }
}

// Stream-major variant for large tiles (chain orders only).  A lane handles U vectors, but
// instead of fetching all W workers' values at once it walks the chain one worker at a time,
// with the next worker's U loads in flight while the current ones are added.  A 1024-lane
// workgroup thus requests 1024*U*16 contiguous bytes of one replica before it moves on to the
// next replica, which the memory system serves better than many short interleaved runs.
template <int W, int U, bool BF16, bool NT>
__global__ void __launch_bounds__(kMaxBlock)
k_ring_reduce_sm(const ReduceTile* __restrict__ tiles, const uint64_t* __restrict__ rows, uint32_t begin,
                 uint32_t count, float inv_w) {
  constexpr uint32_t VE = BF16 ? 8 : 4;
  for (uint32_t ti = blockIdx.x; ti < count; ti += gridDim.x) {
    const ReduceTile tl = tiles[begin + ti];
    gvec_ptr p[W];
#pragma unroll
    for (int k = 0; k < W; ++k) {
      uint32_t w = tl.first + k;
      if (w >= uint32_t(W)) w -= W;
      p[k] = reinterpret_cast<gvec_ptr>(rows[size_t(tl.row) * W + w]) + tl.vec_off;
    }
    const uint32_t nvec = tl.n_elems / VE;
    const uint32_t B = blockDim.x;
    uint32_t v = threadIdx.x;
    const uint32_t whole = nvec / (U * B) * (U * B);  // the same for all lanes
    for (; v < whole; v += U * B) {
      u32x4 cur[U], nxt[U];
      Chain<BF16> acc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) cur[u] = ld<NT>(at(p[0], (v + u * B) * 16u));
#pragma unroll
      for (int k = 1; k < W; ++k) {
#pragma unroll
        for (int u = 0; u < U; ++u) nxt[u] = ld<NT>(at(p[k], (v + u * B) * 16u));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (k == 1) acc[u].start(cur[u]);
          else acc[u].add(cur[u]);
          cur[u] = nxt[u];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      u32x4 y[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        acc[u].add(cur[u]);
        y[u] = acc[u].finish(inv_w);
      }
#pragma unroll
      for (int k = 0; k < W; ++k)
#pragma unroll
        for (int u = 0; u < U; ++u) st<NT>(at(p[k], (v + u * B) * 16u), y[u]);
    }
    // what is left (fewer than U*B vectors: up to U rows of B lanes, the last row possibly
    // ragged) is walked the same way in one go
    const uint32_t rows_left = (nvec - whole + B - 1) / B;
    if (rows_left == 1) {
      // at most one vector per lane: nothing to walk, fetch all workers' values at once
      if (v < nvec) {
        u32x4 x[W];
#pragma unroll
        for (int k = 0; k < W; ++k) x[k] = ld<NT>(at(p[k], v * 16u));
        __builtin_amdgcn_sched_barrier(0);
        const u32x4 y = combine<W, BF16, false>(x, inv_w);
#pragma unroll
        for (int k = 0; k < W; ++k) st<NT>(at(p[k], v * 16u), y);
      }
    }
    if (rows_left == 2) sm_walk<W, 2, 2, BF16, NT, true>(p, v, B, nvec, inv_w);
    if constexpr (U >= 4) {
      if (rows_left == 3) sm_walk<W, 3, 2, BF16, NT, true>(p, v, B, nvec, inv_w);
      if (rows_left == 4) sm_walk<W, 4, 2, BF16, NT, true>(p, v, B, nvec, inv_w);
    }
    if constexpr (U >= 8) {
      if (rows_left == 5) sm_walk<W, 5, 2, BF16, NT, true>(p, v, B, nvec, inv_w);
      if (rows_left == 6) sm_walk<W, 6, 2, BF16, NT, true>(p, v, B, nvec, inv_w);
      if (rows_left == 7) sm_walk<W, 7, 2, BF16, NT, true>(p, v, B, nvec, inv_w);
      if (rows_left == 8) sm_walk<W, 8, 2, BF16, NT, true>(p, v, B, nvec, inv_w);
    }
    const uint32_t rem = tl.n_elems - nvec * VE;
    if (threadIdx.x < rem) {
      const uint32_t e = nvec * VE + threadIdx.x;
      float val[W];
      if constexpr (BF16) {
#pragma unroll
        for (int k = 0; k < W; ++k) val[k] = widen(reinterpret_cast<gu16_ptr>(p[k])[e]);
        const uint16_t y = uint16_t(bf16_rne(combine_scalar<W, false>(val, inv_w)));
#pragma unroll
        for (int k = 0; k < W; ++k) reinterpret_cast<gu16_ptr>(p[k])[e] = y;
      } else {
#pragma unroll
        for (int k = 0; k < W; ++k) val[k] = reinterpret_cast<gf32_ptr>(p[k])[e];
        const float y = combine_scalar<W, false>(val, inv_w);
#pragma unroll
        for (int k = 0; k < W; ++k) reinterpret_cast<gf32_ptr>(p[k])[e] = y;
      }
    }
  }
}

// Stream-major kernel for the halving-doubling order (W a power of two up to 16): the same walk,
// one replica after the other, with the values added as the balanced tree.  The tree does not
// depend on the segment, so the workers are read in the order 0 .. W-1.
template <int W, int U, bool BF16, bool NT>
__global__ void __launch_bounds__(kMaxBlock)
k_ring_reduce_smt(const ReduceTile* __restrict__ tiles, const uint64_t* __restrict__ rows, uint32_t begin,
                  uint32_t count, float inv_w) {
  constexpr uint32_t VE = BF16 ? 8 : 4;
  for (uint32_t ti = blockIdx.x; ti < count; ti += gridDim.x) {
    const ReduceTile tl = tiles[begin + ti];
    gvec_ptr p[W];
#pragma unroll
    for (int k = 0; k < W; ++k) p[k] = reinterpret_cast<gvec_ptr>(rows[size_t(tl.row) * W + k]) + tl.vec_off;
    const uint32_t nvec = tl.n_elems / VE;
    const uint32_t B = blockDim.x;
    const uint32_t whole = nvec / (U * B) * (U * B);  // the same for all lanes
    uint32_t v = threadIdx.x;
#pragma unroll 1
    // (the walk with a guarded last row, although every row is whole here: the compiler keeps
    // fewer values live in that form and does not spill)
    for (; v < whole; v += U * B) sm_walk<W, U, 2, BF16, NT, true, true>(p, v, B, nvec, inv_w);
    const uint32_t rows_left = (nvec - whole + B - 1) / B;
    if (rows_left == 1) {
      if (v < nvec) {
        u32x4 x[W];
#pragma unroll
        for (int k = 0; k < W; ++k) x[k] = ld<NT>(at(p[k], v * 16u));
        __builtin_amdgcn_sched_barrier(0);
        const u32x4 y = combine<W, BF16, true>(x, inv_w);
#pragma unroll
        for (int k = 0; k < W; ++k) st<NT>(at(p[k], v * 16u), y);
      }
    }
    if (rows_left == 2) sm_walk<W, 2, 2, BF16, NT, true, true>(p, v, B, nvec, inv_w);
    if constexpr (U >= 4) {
      if (rows_left == 3) sm_walk<W, 3, 2, BF16, NT, true, true>(p, v, B, nvec, inv_w);
      if (rows_left == 4) sm_walk<W, 4, 2, BF16, NT, true, true>(p, v, B, nvec, inv_w);
    }
    const uint32_t rem = tl.n_elems - nvec * VE;
    if (threadIdx.x < rem) {
      const uint32_t e = nvec * VE + threadIdx.x;
      float val[W];
      if constexpr (BF16) {
#pragma unroll
        for (int k = 0; k < W; ++k) val[k] = widen(reinterpret_cast<gu16_ptr>(p[k])[e]);
        const uint16_t y = uint16_t(bf16_rne(combine_scalar<W, true>(val, inv_w)));
#pragma unroll
        for (int k = 0; k < W; ++k) reinterpret_cast<gu16_ptr>(p[k])[e] = y;
      } else {
#pragma unroll
        for (int k = 0; k < W; ++k) val[k] = reinterpret_cast<gf32_ptr>(p[k])[e];
        const float y = combine_scalar<W, true>(val, inv_w);
#pragma unroll
        for (int k = 0; k < W; ++k) reinterpret_cast<gf32_ptr>(p[k])[e] = y;
      }
    }
  }
}

// Any W: the chain is walked one worker at a time, like the stream-major kernel: the next
// worker's base pointer (a scalar load) and its vectors are requested while the current ones are
// added.  What is left of a tile after whole groups of U*B vectors (up to U rows of B lanes, the
// last row possibly ragged) is walked in one go with that many vectors per lane; a lane beyond
// the end of a ragged row reads the tile's last vector instead and stores nothing for it.
template <bool BF16, bool NT, int U>
__global__ void __launch_bounds__(kMaxBlock)
k_ring_reduce_any(const ReduceTile* __restrict__ tiles, const uint64_t* __restrict__ rows, uint32_t begin,
                  uint32_t count, uint32_t W, float inv_w) {
  constexpr uint32_t VE = BF16 ? 8 : 4;
  for (uint32_t ti = blockIdx.x; ti < count; ti += gridDim.x) {
    const ReduceTile tl = tiles[begin + ti];
    const uint64_t* row = rows + size_t(tl.row) * W;
    const uint32_t nvec = tl.n_elems / VE;
    const uint32_t B = blockDim.x;
    const uint32_t late_from = tl.split / VE;  // used for split tiles only
    // One pass of the chain over N vectors of this lane, B apart, starting at v.
    // SPLIT (a tile across a segment boundary, W >= 2): the workers are visited in the tile's
    // order and then the first one once more, W + 1 steps; the lanes before the boundary add the
    // values of steps 0 .. W-1, the late lanes (whose sums start one worker later) those of steps
    // 1 .. W.  A lane asks for no data in the step it sits out, so nothing is fetched twice and
    // the whole workgroup still reads one replica at a time.
    auto chain = [&](uint32_t v, auto n_tag, auto ragged_tag, auto split_tag) {
      constexpr int N = decltype(n_tag)::value;
      constexpr bool RAGGED = decltype(ragged_tag)::value;
      constexpr bool SPLIT = decltype(split_tag)::value;
      Chain<BF16> acc[N];
      u32x4 cur[N], nxt[N];
      const bool last_ok = !RAGGED || v + (N - 1) * B < nvec;
      uint32_t off[N];
      bool late[N];
#pragma unroll
      for (int u = 0; u < N; ++u) {
        off[u] = (v + u * B) * 16u;
        late[u] = SPLIT && v + u * B >= late_from;
      }
      if (RAGGED && !last_ok) off[N - 1] = (nvec - 1) * 16u;
      uint32_t w = tl.first;
      gvec_ptr base = reinterpret_cast<gvec_ptr>(row[w]) + tl.vec_off;
#pragma unroll
      for (int u = 0; u < N; ++u) {
        cur[u] = u32x4{0u, 0u, 0u, 0u};
        if (!late[u]) cur[u] = ld<NT>(at(base, off[u]));
      }
      const uint32_t steps = SPLIT ? W + 1 : W;
      for (uint32_t k = 1; k < steps; ++k) {
        w = (w + 1 == W) ? 0 : w + 1;
        base = reinterpret_cast<gvec_ptr>(row[w]) + tl.vec_off;
        if (SPLIT && k == W) {
          // back at the first worker: only the late lanes still need its value
#pragma unroll
          for (int u = 0; u < N; ++u) {
            nxt[u] = cur[u];
            if (late[u]) nxt[u] = ld<NT>(at(base, off[u]));
          }
        } else {
#pragma unroll
          for (int u = 0; u < N; ++u) nxt[u] = ld<NT>(at(base, off[u]));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < N; ++u) {
          // cur holds the values of step k - 1
          if (k == 1) {
            acc[u].start(cur[u]);  // (a late lane starts over at the next step)
          } else if (SPLIT && k == 2) {
            Chain<BF16> fresh;
            fresh.start(cur[u]);
            acc[u].add(cur[u]);
            acc[u].take_if(late[u], fresh);
          } else {
            acc[u].add(cur[u]);
          }
          cur[u] = nxt[u];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      u32x4 y[N];
#pragma unroll
      for (int u = 0; u < N; ++u) {
        if constexpr (SPLIT) {
          Chain<BF16> more = acc[u];
          more.add(cur[u]);
          acc[u].take_if(late[u], more);
        } else {
          if (W == 1) acc[u].start(cur[u]);
          else acc[u].add(cur[u]);
        }
        y[u] = acc[u].finish(inv_w);
      }
      for (uint32_t k = 0; k < W; ++k) {
        base = reinterpret_cast<gvec_ptr>(row[k]) + tl.vec_off;
#pragma unroll
        for (int u = 0; u < N; ++u)
          if (!RAGGED || u < N - 1 || last_ok) st<NT>(at(base, off[u]), y[u]);
      }
    };
    const uint32_t whole = nvec / (U * B) * (U * B);  // the same for all lanes
    uint32_t v = threadIdx.x;
    const uint32_t rows_left = (nvec - whole + B - 1) / B;
    static_assert(U == 4, "the dispatches below list the row counts of U = 4");
    if (tl.split) {
      for (; v < whole; v += U * B) chain(v, std::integral_constant<int, U>{}, std::false_type{}, std::true_type{});
      if (rows_left == 1) chain(v, std::integral_constant<int, 1>{}, std::true_type{}, std::true_type{});
      if (rows_left == 2) chain(v, std::integral_constant<int, 2>{}, std::true_type{}, std::true_type{});
      if (rows_left == 3) chain(v, std::integral_constant<int, 3>{}, std::true_type{}, std::true_type{});
      if (rows_left == 4) chain(v, std::integral_constant<int, 4>{}, std::true_type{}, std::true_type{});
    } else {
      for (; v < whole; v += U * B) chain(v, std::integral_constant<int, U>{}, std::false_type{}, std::false_type{});
      if (rows_left == 1 && v < nvec) {
        // at most one vector per lane: nothing to walk; fetch the workers' values eight at a time
        Chain<BF16> acc;
        for (uint32_t k0 = 0; k0 < W; k0 += 8) {
          u32x4 x[8];
#pragma unroll
          for (uint32_t i = 0; i < 8; ++i)
            if (k0 + i < W) {
              uint32_t w = tl.first + k0 + i;
              if (w >= W) w -= W;
              x[i] = ld<NT>(at(reinterpret_cast<gvec_ptr>(row[w]) + tl.vec_off, v * 16u));
            }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (uint32_t i = 0; i < 8; ++i)
            if (k0 + i < W) {
              if (k0 + i == 0) acc.start(x[i]);
              else acc.add(x[i]);
            }
        }
        const u32x4 y = acc.finish(inv_w);
        for (uint32_t k = 0; k < W; ++k) st<NT>(at(reinterpret_cast<gvec_ptr>(row[k]) + tl.vec_off, v * 16u), y);
      }
      if (rows_left == 2) chain(v, std::integral_constant<int, 2>{}, std::true_type{}, std::false_type{});
      if (rows_left == 3) chain(v, std::integral_constant<int, 3>{}, std::true_type{}, std::false_type{});
      if (rows_left == 4) chain(v, std::integral_constant<int, 4>{}, std::true_type{}, std::false_type{});
    }
    const uint32_t rem = tl.n_elems - nvec * VE;
    if (threadIdx.x < rem) {
      const size_t e = size_t(tl.vec_off) * VE + nvec * VE + threadIdx.x;
      // an element behind the boundary of a split tile starts one worker later
      uint32_t w = tl.first + ((tl.split && nvec * VE + threadIdx.x >= tl.split) ? 1u : 0u);
      if (w >= W) w -= W;
      if constexpr (BF16) {
        float acc = widen(reinterpret_cast<gu16_ptr>(row[w])[e]);
        for (uint32_t k = 1; k < W; ++k) {
          w = (w + 1 == W) ? 0 : w + 1;
          acc = acc + widen(reinterpret_cast<gu16_ptr>(row[w])[e]);
        }
        const uint16_t y = uint16_t(bf16_rne(acc * inv_w));
        for (uint32_t k = 0; k < W; ++k) reinterpret_cast<gu16_ptr>(row[k])[e] = y;
      } else {
        float acc = reinterpret_cast<gf32_ptr>(row[w])[e];
        for (uint32_t k = 1; k < W; ++k) {
          w = (w + 1 == W) ? 0 : w + 1;
          acc = acc + reinterpret_cast<gf32_ptr>(row[w])[e];
        }
        const float y = acc * inv_w;
        for (uint32_t k = 0; k < W; ++k) reinterpret_cast<gf32_ptr>(row[k])[e] = y;
      }
    }
  }
}

// Balanced pairwise tree (halving-doubling order) for W = 32 or 64.  The workers are taken eight
// at a time: their eight vectors are added as a three-level tree, and the partial sums of the
// blocks are merged the way a binary counter carries (block j closes as many levels as j + 1 has
// trailing zeros), which is the same tree  ((x0+x1)+(x2+x3)) + ...  up to its root.
template <bool BF16, bool NT>
__global__ void __launch_bounds__(kMaxBlock)
k_ring_reduce_tree_any(const ReduceTile* __restrict__ tiles, const uint64_t* __restrict__ rows, uint32_t begin,
                       uint32_t count, uint32_t W, float inv_w) {
  constexpr uint32_t VE = BF16 ? 8 : 4;
  constexpr int kBlk = 8;       // workers per block
  constexpr int kMaxBlocks = 8;  // W <= 64
  for (uint32_t ti = blockIdx.x; ti < count; ti += gridDim.x) {
    const ReduceTile tl = tiles[begin + ti];
    const uint64_t* row = rows + size_t(tl.row) * W;
    const uint32_t nvec = tl.n_elems / VE;
    const uint32_t n_blocks = W / kBlk;
    for (uint32_t v = threadIdx.x; v < nvec; v += blockDim.x) {
      Chain<BF16> part[4];  // open partial sums of 8, 16, 32 workers (and the root of 64)
      u32x4 y = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < kMaxBlocks; ++j) {
        if (uint32_t(j) < n_blocks) {
          u32x4 x[kBlk];
#pragma unroll
          for (int i = 0; i < kBlk; ++i)
            x[i] = ld<NT>(at(reinterpret_cast<gvec_ptr>(row[j * kBlk + i]) + tl.vec_off, v * 16u));
          __builtin_amdgcn_sched_barrier(0);
          Chain<BF16> t[kBlk];
#pragma unroll
          for (int i = 0; i < kBlk; ++i) t[i].start(x[i]);
#pragma unroll
          for (int s = 1; s < kBlk; s *= 2)
#pragma unroll
            for (int i = 0; i + s < kBlk; i += 2 * s) t[i].merge(t[i + s]);
          // carry: j + 1 = ...1000 closes one level per trailing zero
          int lvl = 0;
#pragma unroll
          for (int m = j + 1; (m & 1) == 0; m >>= 1) {
            part[lvl].merge(t[0]);
            t[0] = part[lvl];
            ++lvl;
          }
          part[lvl] = t[0];
          if (uint32_t(j) + 1 == n_blocks) y = t[0].finish(inv_w);
        }
      }
      for (uint32_t k = 0; k < W; ++k) st<NT>(at(reinterpret_cast<gvec_ptr>(row[k]) + tl.vec_off, v * 16u), y);
    }
    const uint32_t rem = tl.n_elems - nvec * VE;
    if (threadIdx.x < rem) {
      // ragged end of a tensor, one element per lane: the same tree on scalars
      const size_t e = size_t(tl.vec_off) * VE + nvec * VE + threadIdx.x;
      float part[4];
      float y = 0.f;
#pragma unroll
      for (int j = 0; j < kMaxBlocks; ++j) {
        if (uint32_t(j) < n_blocks) {
          float t[kBlk];
#pragma unroll
          for (int i = 0; i < kBlk; ++i) {
            if constexpr (BF16) t[i] = widen(reinterpret_cast<gu16_ptr>(row[j * kBlk + i])[e]);
            else t[i] = reinterpret_cast<gf32_ptr>(row[j * kBlk + i])[e];
          }
#pragma unroll
          for (int s = 1; s < kBlk; s *= 2)
#pragma unroll
            for (int i = 0; i + s < kBlk; i += 2 * s) t[i] = t[i] + t[i + s];
          int lvl = 0;
#pragma unroll
          for (int m = j + 1; (m & 1) == 0; m >>= 1) {
            t[0] = part[lvl] + t[0];
            ++lvl;
          }
          part[lvl] = t[0];
          if (uint32_t(j) + 1 == n_blocks) y = t[0] * inv_w;
        }
      }
      if constexpr (BF16) {
        const uint16_t o = uint16_t(bf16_rne(y));
        for (uint32_t k = 0; k < W; ++k) reinterpret_cast<gu16_ptr>(row[k])[e] = o;
      } else {
        for (uint32_t k = 0; k < W; ++k) reinterpret_cast<gf32_ptr>(row[k])[e] = y;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// pack / unpack: one 1024-lane workgroup per copy tile (at most 1024 vectors of one member, so a
// lane moves one vector and one load instruction of the workgroup covers 16 contiguous KiB),
// grid.y = worker.  A tiny member leaves most lanes idle; measured against one wavefront per 8 KiB
// run, which keeps every lane busy, this is 2 to 7 points of peak faster where it matters and
// equal where the members are small.
template <typename E, bool UNPACK, bool NT>
__global__ void __launch_bounds__(kCopyBlock)
k_copy(const CopyTile* __restrict__ tiles, const uint64_t* __restrict__ rows, uint32_t begin, uint32_t count,
       uint32_t W, uint32_t fused_row) {
  constexpr uint32_t VE = 16 / sizeof(E);
  const uint32_t lane = threadIdx.x;
  const CopyTile t = tiles[begin + blockIdx.x];
  const uint32_t w = blockIdx.y;
  gvec_ptr tp = reinterpret_cast<gvec_ptr>(rows[size_t(t.row) * W + w]) + t.t_vec_off;
  gvec_ptr fp = reinterpret_cast<gvec_ptr>(rows[size_t(fused_row) * W + w]) + t.f_vec_off;
  const uint32_t nvec = t.n_elems / VE;
  gvec_ptr src = UNPACK ? fp : tp;
  gvec_ptr dst = UNPACK ? tp : fp;
  for (uint32_t v = lane; v < nvec; v += kCopyBlock) st<NT>(dst + v, ld<NT>(src + v));
  // ragged end of a member, and (pack only) the +0.0 padding up to the next member
  CARAMEL_GLOBAL E* se = reinterpret_cast<CARAMEL_GLOBAL E*>(src);
  CARAMEL_GLOBAL E* de = reinterpret_cast<CARAMEL_GLOBAL E*>(dst);
  const uint32_t end = UNPACK ? t.n_elems : t.n_elems + t.n_zero;
  for (uint32_t e = nvec * VE + lane; e < end; e += kCopyBlock) de[e] = (e < t.n_elems) ? se[e] : E(0);
}

template <int W, int U>
hipError_t launch_w(const ReduceArgs& a, dim3 grid, float inv_w, hipStream_t s) {
#define CARAMEL_GO(BF, NT, TR) \
  hipLaunchKernelGGL((k_ring_reduce<W, U, BF, NT, TR>), grid, dim3(a.block), 0, s, a.tiles, a.rows, a.begin, a.count, inv_w)
#define CARAMEL_GO2(BF, NT) \
  do { if (a.tree) CARAMEL_GO(BF, NT, true); else CARAMEL_GO(BF, NT, false); } while (0)
  if (a.bf16) {
    if (a.nontemporal) CARAMEL_GO2(true, true); else CARAMEL_GO2(true, false);
  } else {
    if (a.nontemporal) CARAMEL_GO2(false, true); else CARAMEL_GO2(false, false);
  }
#undef CARAMEL_GO2
#undef CARAMEL_GO
  return hipGetLastError();
}

template <int W, int U>
hipError_t launch_sm(const ReduceArgs& a, dim3 grid, float inv_w, hipStream_t s) {
#define CARAMEL_SM(BF, NT) \
  hipLaunchKernelGGL((k_ring_reduce_sm<W, U, BF, NT>), grid, dim3(a.block), 0, s, a.tiles, a.rows, a.begin, a.count, inv_w)
  if constexpr (U >= 8) {
    // eight vectors per lane fit the register file for fp32 only (launch_u sends bf16 elsewhere)
    if (a.bf16) return hipErrorInvalidValue;
    if (a.nontemporal) CARAMEL_SM(false, true); else CARAMEL_SM(false, false);
  } else if (a.bf16) {
    if (a.nontemporal) CARAMEL_SM(true, true); else CARAMEL_SM(true, false);
  } else {
    if (a.nontemporal) CARAMEL_SM(false, true); else CARAMEL_SM(false, false);
  }
#undef CARAMEL_SM
  return hipGetLastError();
}

// fp32: four vectors per lane; bf16 (twice the partial sums per vector): two, i.e. a long tile in
// two passes
template <int W>
hipError_t launch_smt(const ReduceArgs& a, dim3 grid, float inv_w, hipStream_t s) {
#define CARAMEL_SMT(U, BF, NT) \
  hipLaunchKernelGGL((k_ring_reduce_smt<W, U, BF, NT>), grid, dim3(a.block), 0, s, a.tiles, a.rows, a.begin, a.count, inv_w)
  if (a.bf16) {
    if (a.nontemporal) CARAMEL_SMT(2, true, true); else CARAMEL_SMT(2, true, false);
  } else if (a.stream_major >= 4) {
    if (a.nontemporal) CARAMEL_SMT(4, false, true); else CARAMEL_SMT(4, false, false);
  } else {
    if (a.nontemporal) CARAMEL_SMT(2, false, true); else CARAMEL_SMT(2, false, false);
  }
#undef CARAMEL_SMT
  return hipGetLastError();
}

template <int W>
hipError_t launch_u(const ReduceArgs& a, dim3 grid, float inv_w, hipStream_t s) {
  if (a.stream_major && a.tree) return launch_smt<W>(a, grid, inv_w, s);
  if (a.stream_major && !a.tree) {
    if constexpr (W <= 8) {
      if (a.stream_major >= 8 && !a.bf16) return launch_sm<W, 8>(a, grid, inv_w, s);
    }
    if (a.stream_major >= 4) return launch_sm<W, 4>(a, grid, inv_w, s);
    return launch_sm<W, 2>(a, grid, inv_w, s);
  }
  // W * U vectors per lane must fit the register budget of a 1024-lane workgroup
  constexpr uint32_t kMaxU = W <= 4 ? 4 : (W <= 8 ? 2 : 1);
  uint32_t u = a.unroll ? a.unroll : kMaxU;
  if (u > kMaxU) u = kMaxU;
  if constexpr (kMaxU >= 4) if (u >= 4) return launch_w<W, 4>(a, grid, inv_w, s);
  if constexpr (kMaxU >= 2) if (u >= 2) return launch_w<W, 2>(a, grid, inv_w, s);
  return launch_w<W, 1>(a, grid, inv_w, s);
}

}  // namespace

hipError_t launch_ring_reduce(const ReduceArgs& a, hipStream_t s) {
  if (a.count == 0) return hipSuccess;
  if (a.block != 256 && a.block != 512 && a.block != 1024) return hipErrorInvalidValue;
  uint32_t g = a.count;
  if (a.max_grid && g > a.max_grid) g = a.max_grid;
  const dim3 grid(g);
  const float inv_w = 1.0f / float(a.world);
  switch (a.world) {
    case 2: return launch_u<2>(a, grid, inv_w, s);
    case 4: return launch_u<4>(a, grid, inv_w, s);
    case 8: return launch_u<8>(a, grid, inv_w, s);
    case 16: return launch_u<16>(a, grid, inv_w, s);
    default: break;
  }
  if (a.tree && a.world != 1) {  // a tree over one worker is the chain
    if (a.world != 32 && a.world != 64) return hipErrorInvalidValue;
#define CARAMEL_TREE(BF, NT) \
  hipLaunchKernelGGL((k_ring_reduce_tree_any<BF, NT>), grid, dim3(a.block), 0, s, a.tiles, a.rows, a.begin, a.count, a.world, inv_w)
    if (a.bf16) {
      if (a.nontemporal) CARAMEL_TREE(true, true); else CARAMEL_TREE(true, false);
    } else {
      if (a.nontemporal) CARAMEL_TREE(false, true); else CARAMEL_TREE(false, false);
    }
#undef CARAMEL_TREE
    return hipGetLastError();
  }
#define CARAMEL_ANY(BF, NT) \
  hipLaunchKernelGGL((k_ring_reduce_any<BF, NT, 4>), grid, dim3(a.block), 0, s, a.tiles, a.rows, a.begin, a.count, a.world, inv_w)
  if (a.bf16) {
    if (a.nontemporal) CARAMEL_ANY(true, true); else CARAMEL_ANY(true, false);
  } else {
    if (a.nontemporal) CARAMEL_ANY(false, true); else CARAMEL_ANY(false, false);
  }
#undef CARAMEL_ANY
  return hipGetLastError();
}

// the kernel for any world size does; the ones specialised for 2, 4, 8 and 16 workers do not
bool reduce_handles_split_tiles(uint32_t world) {
  return world != 2 && world != 4 && world != 8 && world != 16;
}

hipError_t launch_copy(const CopyArgs& a, hipStream_t s) {
  if (a.count == 0) return hipSuccess;
  const dim3 grid(a.count, a.world);
#define CARAMEL_CP(E, UN) \
  do { \
    if (a.nontemporal) \
      hipLaunchKernelGGL((k_copy<E, UN, true>), grid, dim3(kCopyBlock), 0, s, a.tiles, a.rows, a.begin, a.count, a.world, a.fused_row); \
    else \
      hipLaunchKernelGGL((k_copy<E, UN, false>), grid, dim3(kCopyBlock), 0, s, a.tiles, a.rows, a.begin, a.count, a.world, a.fused_row); \
  } while (0)
  if (a.bf16) {
    if (a.unpack) CARAMEL_CP(uint16_t, true); else CARAMEL_CP(uint16_t, false);
  } else {
    if (a.unpack) CARAMEL_CP(uint32_t, true); else CARAMEL_CP(uint32_t, false);
  }
#undef CARAMEL_CP
  return hipGetLastError();
}

}  // namespace caramel
