// Rotary positional embedding, rotate-half form (the paper's language-model case study,
// Sec. 4 "Case study"): y[i] = x[i] cos[i] + rot(x)[i] sin[i] per head vector.
//
// A pure streaming kernel: every element of the tensors is read once and written once,
// the tables are small and stay in cache (all heads of a position share one row).  In the
// paper's taxonomy (Sec. 3.2): d_mem = 1 (coalesced 16-byte accesses), d_algo = 1 (one
// fused pass), d_sync = 0.  A work item is one 16-byte chunk of a head vector's first half
// together with its partner chunk in the second half, so a lane owns whole rotation pairs
// and the kernel may run in place.  A workgroup takes a few consecutive positions of one
// batch; its items run over (position, tensor, head, chunk) with the chunk fastest, which
// makes the lanes of a wave walk through memory contiguously when the heads of a position
// are adjacent in memory.
#pragma once

#include "common.hpp"

namespace mi355gemm {

struct RopeTensorArgs {
  const void* x; void* y;
  int64_t xb, xh, xs;          // element strides of x: batch, head, position
  int64_t yb, yh, ys;
  int heads;
};

struct RopeArgs {
  RopeTensorArgs t[2];
  const void* cos; const void* sin;
  int64_t table_stride_b;
  int64_t positions;           // batch * seq
  int seq, head_dim;
  int n_tensors;
  int pos_per_block;           // positions a workgroup handles
  int chunks;                  // work items per head vector
  int items0, items_pos;       // work items per position: first tensor, all tensors
};

template <typename T> struct Vec8;           // eight elements of the storage type
template <> struct Vec8<bf16_t> {
  u32x4_t v;
  __device__ __forceinline__ void load(const bf16_t* p) { v = __builtin_nontemporal_load((const u32x4_t*)p); }
  __device__ __forceinline__ void load_cached(const bf16_t* p) { v = *(const u32x4_t*)p; }
  __device__ __forceinline__ void store(bf16_t* p) const { __builtin_nontemporal_store(v, (u32x4_t*)p); }
  __device__ __forceinline__ float get(int e) const {
    const uint32_t w = v[e >> 1];
    return __builtin_bit_cast(float, (e & 1) ? (w & 0xffff0000u) : (w << 16));
  }
  __device__ __forceinline__ void set2(int e, float a, float b) { v[e >> 1] = pack2<bf16_t>(a, b); }
  __device__ __forceinline__ Vec8 from_lane_xor(int mask) const {
    Vec8 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = (uint32_t)__shfl_xor((int)v[i], mask, 64);
    return r;
  }
};
template <> struct Vec8<f16_t> {
  u32x4_t v;
  __device__ __forceinline__ void load(const f16_t* p) { v = __builtin_nontemporal_load((const u32x4_t*)p); }
  __device__ __forceinline__ void load_cached(const f16_t* p) { v = *(const u32x4_t*)p; }
  __device__ __forceinline__ void store(f16_t* p) const { __builtin_nontemporal_store(v, (u32x4_t*)p); }
  __device__ __forceinline__ float get(int e) const {
    const uint32_t w = v[e >> 1];
    const uint16_t h = (e & 1) ? (uint16_t)(w >> 16) : (uint16_t)(w & 0xffffu);
    return (float)__builtin_bit_cast(f16_t, h);
  }
  __device__ __forceinline__ void set2(int e, float a, float b) { v[e >> 1] = pack2<f16_t>(a, b); }
  __device__ __forceinline__ Vec8 from_lane_xor(int mask) const {
    Vec8 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = (uint32_t)__shfl_xor((int)v[i], mask, 64);
    return r;
  }
};
template <> struct Vec8<float> {
  f32x4_t lo, hi;
  __device__ __forceinline__ void load(const float* p) {
    lo = __builtin_nontemporal_load((const f32x4_t*)p);
    hi = __builtin_nontemporal_load((const f32x4_t*)p + 1);
  }
  __device__ __forceinline__ void load_cached(const float* p) {
    lo = *(const f32x4_t*)p;
    hi = *((const f32x4_t*)p + 1);
  }
  __device__ __forceinline__ void store(float* p) const {
    __builtin_nontemporal_store(lo, (f32x4_t*)p);
    __builtin_nontemporal_store(hi, (f32x4_t*)p + 1);
  }
  __device__ __forceinline__ float get(int e) const { return e < 4 ? lo[e] : hi[e - 4]; }
  __device__ __forceinline__ void set2(int e, float a, float b) {
    if (e < 4) { lo[e] = a; lo[e + 1] = b; } else { hi[e - 4] = a; hi[e - 3] = b; }
  }
  __device__ __forceinline__ Vec8 from_lane_xor(int mask) const {
    Vec8 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) { r.lo[i] = __shfl_xor(lo[i], mask, 64); r.hi[i] = __shfl_xor(hi[i], mask, 64); }
    return r;
  }
};

// The fast kernel: 16-byte accesses, and a group of G lanes (G a multiple of the chunks per
// head vector, so that a lane's chunk never changes) takes one position and walks over the
// heads of every tensor.  A lane therefore loads its table entries once and re-uses them for
// all the heads it visits: the tables' share of the load traffic drops from twice the
// tensors' to a fraction of it, while the G lanes still touch G*16 contiguous bytes (per
// half) when the heads of a position are adjacent in memory.  The head loop requests U head
// vectors before it writes any (the tensors may be rotated in place, so loads cannot be
// hoisted over stores by the compiler).
template <typename T, typename TT, int G>
__global__ __launch_bounds__(256) void rope_group_kernel(RopeArgs p) {
  constexpr int U = 4;
  const int64_t pos = ((int64_t)blockIdx.x * 256 + threadIdx.x) / G;
  if (pos >= p.positions) return;
  const int lg = threadIdx.x % G;
  const int c = lg % p.chunks;                 // chunks divides G
  const int h0 = lg / p.chunks, hstep = G / p.chunks;
  const int half = p.head_dim / 2;
  const int b = (int)(pos / p.seq);
  const int s = (int)(pos - (int64_t)b * p.seq);
  const TT* ct = (const TT*)p.cos + (int64_t)b * p.table_stride_b + (int64_t)s * p.head_dim + c * 8;
  const TT* st = (const TT*)p.sin + (int64_t)b * p.table_stride_b + (int64_t)s * p.head_dim + c * 8;
  Vec8<TT> c1, c2, s1, s2;
  c1.load_cached(ct); c2.load_cached(ct + half);
  s1.load_cached(st); s2.load_cached(st + half);
  for (int ti = 0; ti < p.n_tensors; ++ti) {
    const RopeTensorArgs& t = p.t[ti];
    const T* x = (const T*)t.x + (int64_t)b * t.xb + (int64_t)s * t.xs + c * 8;
    T* y = (T*)t.y + (int64_t)b * t.yb + (int64_t)s * t.ys + c * 8;
    for (int h = h0; h < t.heads; h += U * hstep) {
      Vec8<T> x1[U], x2[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int hh = h + u * hstep;
        if (hh < t.heads) { x1[u].load(x + (int64_t)hh * t.xh); x2[u].load(x + (int64_t)hh * t.xh + half); }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int hh = h + u * hstep;
        if (hh >= t.heads) break;
        Vec8<T> y1, y2;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          float o1[2], o2[2];
#pragma unroll
          for (int v = 0; v < 2; ++v) {
            const float a = x1[u].get(e + v), w = x2[u].get(e + v);
            o1[v] = fmaf(a, c1.get(e + v), -(w * s1.get(e + v)));     // x[i] cos[i] - x[i + D/2] sin[i]
            o2[v] = fmaf(w, c2.get(e + v), a * s2.get(e + v));        // x[i + D/2] cos[..] + x[i] sin[..]
          }
          y1.set2(e, o1[0], o1[1]);
          y2.set2(e, o2[0], o2[1]);
        }
        y1.store(y + (int64_t)hh * t.yh);
        y2.store(y + (int64_t)hh * t.yh + half);
      }
    }
  }
}

// The fastest kernel, for head vectors whose half is a power-of-two number of 16-byte chunks
// (head_dim 16, 32, 64, 128, ...): a lane owns ONE chunk of the whole head vector, so the G
// lanes of a group read and write G*16 contiguous bytes per instruction (whole cache lines
// even when a half is only 64 bytes), and fetches the partner chunk (the other half, same
// offset) from the lane `chunks` away with a cross-lane exchange.  Partner lanes visit the
// same head of the same position, so they are always active together.
template <typename T, typename TT, int G>
__global__ __launch_bounds__(256) void rope_exchange_kernel(RopeArgs p) {
  constexpr int U = 4;
  const int64_t pos = ((int64_t)blockIdx.x * 256 + threadIdx.x) / G;
  if (pos >= p.positions) return;
  const int lg = threadIdx.x % G;
  const int per_head = 2 * p.chunks;           // lanes per head vector; divides G
  const int cc = lg % per_head;                // chunk of the whole vector
  const int h0 = lg / per_head, hstep = G / per_head;
  const bool first_half = cc < p.chunks;
  const int b = (int)(pos / p.seq);
  const int s = (int)(pos - (int64_t)b * p.seq);
  Vec8<TT> cv, sv;
  cv.load_cached((const TT*)p.cos + (int64_t)b * p.table_stride_b + (int64_t)s * p.head_dim + cc * 8);
  sv.load_cached((const TT*)p.sin + (int64_t)b * p.table_stride_b + (int64_t)s * p.head_dim + cc * 8);
  float sg[8];                                  // rot(x) = -partner in the first half, +partner in the second
#pragma unroll
  for (int e = 0; e < 8; ++e) sg[e] = first_half ? -sv.get(e) : sv.get(e);
  for (int ti = 0; ti < p.n_tensors; ++ti) {
    const RopeTensorArgs& t = p.t[ti];
    const T* x = (const T*)t.x + (int64_t)b * t.xb + (int64_t)s * t.xs + cc * 8;
    T* y = (T*)t.y + (int64_t)b * t.yb + (int64_t)s * t.ys + cc * 8;
    for (int h = h0; h < t.heads; h += U * hstep) {
      Vec8<T> xv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int hh = h + u * hstep;
        if (hh < t.heads) xv[u].load(x + (int64_t)hh * t.xh);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int hh = h + u * hstep;
        if (hh >= t.heads) break;
        const Vec8<T> pv = xv[u].from_lane_xor(p.chunks);
        Vec8<T> yv;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const float o0 = fmaf(xv[u].get(e), cv.get(e), pv.get(e) * sg[e]);
          const float o1 = fmaf(xv[u].get(e + 1), cv.get(e + 1), pv.get(e + 1) * sg[e + 1]);
          yv.set2(e, o0, o1);
        }
        yv.store(y + (int64_t)hh * t.yh);
      }
    }
  }
}

// The general kernel.
// VEC = 8: a work item is 8 + 8 elements moved with 16-byte accesses (needs head_dim % 16 == 0
// and 16-byte aligned rows); VEC = 1: one pair per work item, any even head_dim.
template <typename T, typename TT, int VEC>
__global__ __launch_bounds__(256) void rope_kernel(RopeArgs p) {
  const int64_t pos0 = (int64_t)blockIdx.x * p.pos_per_block;
  const int n_pos = (int)min((int64_t)p.pos_per_block, p.positions - pos0);
  const int total = n_pos * p.items_pos;
  const int half = p.head_dim / 2;
  for (int j = threadIdx.x; j < total; j += 256) {
    const int lp = j / p.items_pos;               // position within the workgroup's share
    int r = j - lp * p.items_pos;
    const int ti = r >= p.items0 ? 1 : 0;          // which tensor
    if (ti) r -= p.items0;
    const int h = r / p.chunks;
    const int c = r - h * p.chunks;
    const int64_t pos = pos0 + lp;
    const int64_t b = pos / p.seq;
    const int64_t s = pos - b * p.seq;
    const RopeTensorArgs& t = p.t[ti];
    const T* x = (const T*)t.x + b * t.xb + (int64_t)h * t.xh + s * t.xs + c * VEC;
    T* y = (T*)t.y + b * t.yb + (int64_t)h * t.yh + s * t.ys + c * VEC;
    const TT* ct = (const TT*)p.cos + b * p.table_stride_b + s * p.head_dim + c * VEC;
    const TT* st = (const TT*)p.sin + b * p.table_stride_b + s * p.head_dim + c * VEC;
    if constexpr (VEC == 8) {
      Vec8<T> x1, x2, y1, y2;
      Vec8<TT> c1, c2, s1, s2;
      x1.load(x); x2.load(x + half);
      c1.load_cached(ct); c2.load_cached(ct + half);
      s1.load_cached(st); s2.load_cached(st + half);
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        float o1[2], o2[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const float a = x1.get(e + u), w = x2.get(e + u);
          o1[u] = fmaf(a, c1.get(e + u), -(w * s1.get(e + u)));     // x[i] cos[i] - x[i + D/2] sin[i]
          o2[u] = fmaf(w, c2.get(e + u), a * s2.get(e + u));        // x[i + D/2] cos[..] + x[i] sin[..]
        }
        y1.set2(e, o1[0], o1[1]);
        y2.set2(e, o2[0], o2[1]);
      }
      y1.store(y); y2.store(y + half);
    } else {
      const float a = to_float<T>(x[0]), w = to_float<T>(x[half]);
      const float o1 = fmaf(a, to_float<TT>(ct[0]), -(w * to_float<TT>(st[0])));
      const float o2 = fmaf(w, to_float<TT>(ct[half]), a * to_float<TT>(st[half]));
      y[0] = from_float<T>(o1);
      y[half] = from_float<T>(o2);
    }
  }
}

}  // namespace mi355gemm
