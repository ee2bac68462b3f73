// Small device kernels of the library besides the grouped GEMM (gfx950 only; included by
// exec.hip): the replica sum and the replica broadcast of Table 1, the pass that adds up the
// partial tiles of K-split macro-tiles, and the matrix-pipe rate probe.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"

namespace dmm {

// ------------------------------------------------------------------ device tables (replica sum)

struct RedTile {         // one C tile for the replica sum
  float *out;
  int64_t ldo;
  int64_t part_begin;    // index into the parts arrays (nparts entries)
  int32_t rows, cols;
};

struct RedItem {
  int32_t tile;
  int32_t row0, nrows;
  int32_t pad;
};

typedef float floatx4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ replica sum

// out = ((p0 + p1) + p2) + ...  for a block of rows of one C tile (reduce_replicas, Table 1).
// HBM-bound: (nparts + 1) * 4 bytes per element.  float4 path when every pointer and
// leading dimension allows it.
constexpr int RED_NT = 256;
// Elements of C one workgroup sums: one trip of its 256 threads x 4 float4 columns.  Measured on
// 16 tiles of 2048 x 2048 with two replicas: 4 K elements 6.4 TB/s, 16 K 5.8, 64 K 5.5, 1 K 6.3.
constexpr int RED_ELEMS = 4096;

__global__ __launch_bounds__(RED_NT) void reduce_replicas_kernel(const RedItem *__restrict__ items,
                                                                 const RedTile *__restrict__ tiles,
                                                                 const float *const *__restrict__ parts,
                                                                 const int64_t *__restrict__ part_ld,
                                                                 int nparts, int vec_ok) {
  const RedItem it = items[blockIdx.x];
  const RedTile t = tiles[it.tile];
  const float *const *pp = parts + t.part_begin;
  const int64_t *pl = part_ld + t.part_begin;
  if (vec_ok) {
    // Four independent float4 columns of work per thread and trip, all loads issued before the
    // first add: (4 nparts) 16-byte loads in flight per thread keep HBM busy at modest occupancy.
    const int c4 = t.cols >> 2;
    const int total = it.nrows * c4;
    constexpr int U = 4;
    for (int base = threadIdx.x; base < total; base += U * RED_NT) {
      floatx4 s[U];
      int64_t oo[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = base + u * RED_NT;
        ok[u] = idx < total;
        const int r = it.row0 + (ok[u] ? idx / c4 : 0), c = ok[u] ? (idx % c4) << 2 : 0;
        oo[u] = (int64_t)r * t.ldo + c;
        if (ok[u]) s[u] = __builtin_nontemporal_load((const floatx4 *)(pp[0] + (int64_t)r * pl[0] + c));
      }
      for (int q = 1; q < nparts; ++q) {
        floatx4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int idx = base + u * RED_NT;
          const int r = it.row0 + (ok[u] ? idx / c4 : 0), c = ok[u] ? (idx % c4) << 2 : 0;
          if (ok[u]) v[u] = __builtin_nontemporal_load((const floatx4 *)(pp[q] + (int64_t)r * pl[q] + c));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (ok[u]) {
            s[u].x = s[u].x + v[u].x;
            s[u].y = s[u].y + v[u].y;
            s[u].z = s[u].z + v[u].z;
            s[u].w = s[u].w + v[u].w;
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) __builtin_nontemporal_store(s[u], (floatx4 *)(t.out + oo[u]));
    }
  } else {
    const int total = it.nrows * t.cols;
    for (int idx = threadIdx.x; idx < total; idx += RED_NT) {
      const int r = it.row0 + idx / t.cols, c = idx % t.cols;
      float s = pp[0][(int64_t)r * pl[0] + c];
      for (int q = 1; q < nparts; ++q) s = s + pp[q][(int64_t)r * pl[q] + c];
      t.out[(int64_t)r * t.ldo + c] = s;
    }
  }
}

// Every replica's tile except the origin's becomes a copy of the origin's (broadcast_replica,
// Table 1).  Same work items and tables as the replica sum, `out` being the origin's tile.
// HBM-bound: nparts * 4 bytes per element (one read, nparts - 1 writes).
__global__ __launch_bounds__(RED_NT) void broadcast_replica_kernel(const RedItem *__restrict__ items,
                                                                   const RedTile *__restrict__ tiles,
                                                                   float *const *__restrict__ parts,
                                                                   const int64_t *__restrict__ part_ld, int nparts,
                                                                   int vec_ok) {
  const RedItem it = items[blockIdx.x];
  const RedTile t = tiles[it.tile];
  float *const *pp = parts + t.part_begin;
  const int64_t *pl = part_ld + t.part_begin;
  if (vec_ok) {
    const int c4 = t.cols >> 2;
    const int total = it.nrows * c4;
    for (int idx = threadIdx.x; idx < total; idx += RED_NT) {
      const int r = it.row0 + idx / c4, c = (idx % c4) << 2;
      const floatx4 v = __builtin_nontemporal_load((const floatx4 *)(t.out + (int64_t)r * t.ldo + c));
      for (int q = 0; q < nparts; ++q)
        if (pp[q] != t.out) __builtin_nontemporal_store(v, (floatx4 *)(pp[q] + (int64_t)r * pl[q] + c));
    }
  } else {
    const int total = it.nrows * t.cols;
    for (int idx = threadIdx.x; idx < total; idx += RED_NT) {
      const int r = it.row0 + idx / t.cols, c = idx % t.cols;
      const float v = t.out[(int64_t)r * t.ldo + c];
      for (int q = 0; q < nparts; ++q)
        if (pp[q] != t.out) pp[q][(int64_t)r * pl[q] + c] = v;
    }
  }
}

// ------------------------------------------------------------------ K-split of the last round

// When the number of macro-tiles is not a multiple of the number of CUs, the last round of
// workgroups leaves CUs idle.  The host then cuts each macro-tile of that round into runs of K
// steps, one workgroup each, which write their partial sums into a scratch buffer (256 x 256
// fp32 per run); this kernel adds the runs of a macro-tile up in ascending k and writes C.  Fixed
// cut, fixed order, no atomics: the result is deterministic.
struct FixItem {
  void *dst;             // top-left of the macro-tile in the C tile
  int64_t ldc;           // elements
  const float *parts;    // nparts consecutive 256 x 256 fp32 tiles
  int32_t m_ext, n_ext;
  int32_t nparts;
  int32_t c_es;          // bytes per element of dst: 4 = fp32, 2 = bf16 (the sum rounded to nearest even)
  int32_t row0, col0;    // where the region that goes to dst begins inside the partial tiles (merged macro-tiles
                         // are written piece by piece; col0 is a multiple of 4)
};
constexpr int FIX_ROWS = 4;           // rows of a macro-tile one workgroup sums: 4 rows x 64 float4 columns

__global__ __launch_bounds__(256) void sum_parts_kernel(const FixItem *__restrict__ fixes) {
  const FixItem f = fixes[blockIdx.x / (BM / FIX_ROWS)];
  const int r = (blockIdx.x % (BM / FIX_ROWS)) * FIX_ROWS + (threadIdx.x >> 6);
  const int c = (threadIdx.x & 63) << 2;
  if (r >= f.m_ext || c >= f.n_ext) return;
  const float *p = f.parts + (int64_t)(f.row0 + r) * BN + f.col0 + c;
  floatx4 s = __builtin_nontemporal_load((const floatx4 *)p);
  // eight runs' loads in flight at a time; the adds follow in ascending k (the order is part of the result)
  constexpr int QB = 8;
  for (int q0 = 1; q0 < f.nparts; q0 += QB) {
    floatx4 v[QB];
#pragma unroll
    for (int qq = 0; qq < QB; ++qq)
      if (q0 + qq < f.nparts) v[qq] = __builtin_nontemporal_load((const floatx4 *)(p + (int64_t)(q0 + qq) * (BM * BN)));
#pragma unroll
    for (int qq = 0; qq < QB; ++qq)
      if (q0 + qq < f.nparts) {
        s.x = s.x + v[qq].x;
        s.y = s.y + v[qq].y;
        s.z = s.z + v[qq].z;
        s.w = s.w + v[qq].w;
      }
  }
  const float e[4] = {s.x, s.y, s.z, s.w};
  if (f.c_es == 4) {
    float *d = (float *)f.dst + (int64_t)r * f.ldc + c;
#pragma unroll
    for (int x = 0; x < 4; ++x)
      if (c + x < f.n_ext) __builtin_nontemporal_store(e[x], d + x);
  } else {
    unsigned short *d = (unsigned short *)f.dst + (int64_t)r * f.ldc + c;
#pragma unroll
    for (int x = 0; x < 4; ++x)
      if (c + x < f.n_ext) __builtin_nontemporal_store(__builtin_bit_cast(unsigned short, (__bf16)e[x]), d + x);
  }
}

// ------------------------------------------------------------------ matrix-pipe rate probe

// Eight independent accumulators per wave, operands held in registers: the MFMA pipe is never
// idle and nothing else on the chip is busy.  Reports elapsed shader cycles of wave 0 per block.
__global__ __launch_bounds__(256) void mfma_rate_kernel(unsigned long long *cycles, float *sink, int iters,
                                                        int random_operands) {
  floatx16 acc[8];
  bf16x8 a[8], b[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[s][r] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      unsigned h = (threadIdx.x * 977u + blockIdx.x * 131071u + s * 8u + e) * 2654435761u;
      h ^= h >> 15;
      h *= 0x846ca68bu;
      h ^= h >> 16;
      a[s][e] = (__bf16)(random_operands ? ((int)(h & 0xFFFFu) - 32768) * (1.0f / 32768.0f) : 1.0f);
      b[s][e] = (__bf16)(random_operands ? ((int)(h >> 16) - 32768) * (1.0f / 32768.0f) : 0.5f);
    }
  }
#pragma unroll
  for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(a[s]), "+v"(b[s]));
  const unsigned long long t0 = __builtin_amdgcn_s_memtime();
  for (int it = 0; it < iters; it += 4) {
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int u = 0; u < 8; ++u)
        acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[(u + 3 * v) & 7], acc[u], 0, 0, 0);
  }
  const unsigned long long t1 = __builtin_amdgcn_s_memtime();
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 8; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[u][r];
  if (s == 12345.678f) sink[0] = s;       // keeps the accumulators alive; never true in practice
  if (threadIdx.x == 0) cycles[blockIdx.x] = t1 - t0;
}

}  // namespace dmm
