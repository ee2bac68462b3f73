// Grouped GEMM kernel for gfx950 (device code only; included by exec.hip).
//
// Executes the whole op list of the plan in one launch: the "local matrix
// multiplication" step of direct execution (Section 4.2) for every virtual rank
// at once.  One workgroup owns one 256 x 256 macro-tile of one output sub-tile
// and walks the group's K-segments in ascending k; each segment's A slice and B
// slice are read straight out of the owning rank's tile buffer (the one-sided
// "get" of Section 3 becomes a strided load).  fp32 accumulation in MFMA
// registers; each C element is written once, so there are no atomics and the
// summation order is fixed.
//
// Layout of the work
//   8 waves (2 x 4), wave tile 128 x 64 = 4 x 2 MFMA tiles of 32 x 32.
//   K step: 64 (bf16) or 32 (fp32) elements = 128 bytes of every A row.
//   Two LDS stages of 64 KB: A stage 256 rows x 128 B, B stage K rows x 256 columns.
//   16-byte chunks are XOR-swizzled (A by row, B by k) so that ds_read_b128 of A
//   fragments and ds_read_b64_tr_b16 of B fragments are free of bank conflicts.
//
// Global -> LDS
//   global_load_lds_dwordx4: every lane moves 16 bytes from an arbitrary global
//   address to LDS, lane l landing at M0 + 16 l, with no register staging.  A wave
//   fills 1 KB per instruction (8 A rows, or 2 / 1 B rows); the swizzle is realised
//   by permuting which global chunk a lane fetches.  Sources need only element
//   alignment (odd leading dimensions are fine).  The loads of step s + 1 are in
//   flight while step s is multiplied.
//
// Edges, without a second load path
//   rows past the item's extent    -> the lane reads the last valid row instead
//                                     (the results of such rows are never stored);
//   columns past the item's extent -> loaded as they are (garbage columns of C are
//                                     never stored);
//   chunks that would cross the end of the tile buffer -> the lane is masked out of
//                                     the load and patches its own LDS slot element
//                                     by element afterwards;
//   K tail of a segment            -> after the loads have landed, every lane zeroes
//                                     (or masks) the part of its own slots with
//                                     k >= remaining length, on both operands.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#ifdef DMM_NO_SCHED_BARRIER
#define DMM_SCHED_BARRIER
#else
#define DMM_SCHED_BARRIER __builtin_amdgcn_sched_barrier(0)
#endif

namespace dmm {

struct SegDev {          // one K-segment of a group; pointers at the group's (m0, k0) / (k0, n0)
  const char *a;
  const char *b;
  int64_t lda, ldb;      // elements
  int64_t a_bytes;       // readable bytes from `a` to the end of its tile buffer
  int64_t b_bytes;       // readable bytes from `b` to the end of its tile buffer
  int32_t klen;
  int32_t pad;
};

struct ItemDev {         // one macro-tile
  float *c;              // top-left of the macro-tile in the C tile
  int64_t ldc;
  int32_t seg_begin;
  int32_t nsteps;        // K steps of the item: sum over its segments of ceil(klen / K step); 0 = zero fill
  int32_t m_off, n_off;  // offset inside the group's sub-tile
  int32_t m_ext, n_ext;
};

constexpr int BM = 256, BN = 256;
constexpr int A_STAGE = BM * 128;             // bytes: 256 rows x 128 B
constexpr int B_STAGE = 32 * 1024;            // bytes: 64 x 512 B (bf16) or 32 x 1024 B (fp32)
constexpr int STAGE = A_STAGE + B_STAGE;
constexpr int LDS_BYTES = 2 * STAGE;          // 128 KB

// Wave arrangement of a workgroup: WAVES_M x WAVES_N waves, each owning a
// (256 / WAVES_M) x (256 / WAVES_N) part of the macro-tile as FM x FN MFMA tiles of 32 x 32.
template <int WAVES_M_, int WAVES_N_>
struct Waves {
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NW = WAVES_M * WAVES_N;
  static constexpr int NT = 64 * NW;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int FM = WTM / 32, FN = WTN / 32;
  static constexpr int LOADS = 32 / NW;      // wave-wide 1 KB loads per wave, per operand, per K step
};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4_t *lds_short4_ptr;
typedef __attribute__((address_space(3))) void *lds_void_ptr;
// Pointers read from the work table would otherwise be treated as generic (flat) addresses.
typedef const __attribute__((address_space(1))) char *gptr;
typedef __attribute__((address_space(1))) float *gfloat_ptr;

template <int ES>
struct Shape;
template <>
struct Shape<2> {                              // bf16
  static constexpr int BK = 64;                // elements per K step
  static constexpr int B_ROW = 512;            // bytes per k row of the B stage
  static constexpr int B_CHUNKS = 32;          // 16-byte chunks per k row
  static constexpr int KSUB = 4;               // MFMA sub-steps per K step (16 k each)
};
template <>
struct Shape<4> {                              // fp32
  static constexpr int BK = 32;
  static constexpr int B_ROW = 1024;
  static constexpr int B_CHUNKS = 64;
  static constexpr int KSUB = 4;               // 8 k each
};

template <int ES, int FM, int FN>
struct FragSet;
template <int FM, int FN>
struct FragSet<2, FM, FN> {        // bf16: A rows x 8 k and B columns x 8 k per lane
  bf16x8 a[FM], b[FN];
};
template <int FM, int FN>
struct FragSet<4, FM, FN> {        // fp32: A rows x 4 k per lane; B value per MFMA e and column block
  float4 a[FM];
  float b[4][FN];
};

__device__ __forceinline__ int a_swizzle(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// byte offset of 16-byte chunk `c` (0..7) of row `row` in the A stage
__device__ __forceinline__ int a_lds_off(int row, int c) { return row * 128 + ((c ^ a_swizzle(row)) << 4); }

// chunk position <-> logical chunk inside a k row of the B stage (an involution).
// bf16: 64-byte segments (4 chunks) XOR-ed with k & 3, so the four k rows that one
// transposed read touches fall into different banks; fp32: 128-byte segments (8 chunks)
// XOR-ed with (k >> 2) & 7, so rows k and k + 4, read together, do not collide.
template <int ES>
__device__ __forceinline__ int b_swizzle_chunk(int k, int c) {
  if (ES == 2) return (((c >> 2) ^ (k & 3)) << 2) | (c & 3);
  return (((c >> 3) ^ ((k >> 2) & 7)) << 3) | (c & 7);
}
template <int ES>
__device__ __forceinline__ int b_lds_off(int k, int c) {
  return k * Shape<ES>::B_ROW + (b_swizzle_chunk<ES>(k, c) << 4);
}

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at LDS byte
// address lds_base + 16 l (lds_base wave-uniform, passed in M0); lanes switched off by the
// exec mask leave their slot untouched.  The source is a wave-uniform 64-bit base plus a
// 32-bit per-lane byte offset.  Issued as inline assembly so that the compiler does not
// serialise it against LDS reads of the *other* stage (it cannot tell the stages apart and
// would wait for vmcnt(0) before every ds_read); completion is awaited explicitly with
// s_waitcnt vmcnt(0) before the barrier that publishes the stage.
__device__ __forceinline__ void load_to_lds_16(gptr base, unsigned lane_off, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_off), "s"(base), "s"(lds_base)
               : "memory");
}

// The first `n` (< 16 / ES) elements at p, the rest zero; n <= 0 reads nothing.
template <int ES>
__device__ __forceinline__ u32x4 load_partial(gptr p, int n) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (ES == 2) {
    const __attribute__((address_space(1))) unsigned short *q =
        (const __attribute__((address_space(1))) unsigned short *)p;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const unsigned int e = i < n ? (unsigned int)q[i] : 0u;
      v[i >> 1] |= e << ((i & 1) * 16);
    }
  } else {
    const __attribute__((address_space(1))) unsigned int *q =
        (const __attribute__((address_space(1))) unsigned int *)p;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = i < n ? q[i] : 0u;
  }
  return v;
}

// Keep the first `n` elements of a 16-byte chunk, zero the rest (0 < n < 16 / ES).
template <int ES>
__device__ __forceinline__ u32x4 keep_first(u32x4 v, int n) {
  if (ES == 2) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int left = n - 2 * w;            // elements of this dword that survive
      v[w] = left >= 2 ? v[w] : left == 1 ? (v[w] & 0xFFFFu) : 0u;
    }
  } else {
#pragma unroll
    for (int w = 0; w < 4; ++w) v[w] = w < n ? v[w] : 0u;
  }
  return v;
}

template <int ES, class W>
__global__ __launch_bounds__(W::NT) void grouped_gemm_kernel(const ItemDev *__restrict__ items,
                                                             const SegDev *__restrict__ segs) {
  using S = Shape<ES>;
  constexpr int WAVES_N = W::WAVES_N, NW = W::NW, WTM = W::WTM, WTN = W::WTN, FM = W::FM, FN = W::FN,
                LOADS = W::LOADS;
  constexpr int BK = S::BK;
  constexpr int PER = 16 / ES;                          // elements per 16-byte chunk
  constexpr int B_ROWS_PER_KB = 1024 / S::B_ROW;        // k rows one wave-wide load covers
  constexpr int KSUB = S::KSUB;

  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const ItemDev it = items[blockIdx.x];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const unsigned lds_base = (unsigned)(uintptr_t)(lds_void_ptr)lds;   // LDS byte address of stage 0

  floatx16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- global -> LDS ------------------------------------------------------------------
  // Wave w, load i fills KB number NW i + w of the A stage (rows 8 (NW i + w) .. + 7) and KB
  // number NW i + w of the B stage (k rows B_ROWS_PER_KB (NW i + w) ..).  Lane l owns the slot at
  // +16 l of that KB; a_src / b_src are the byte offsets of the chunk it fetches, relative
  // to the step's base address.
  unsigned a_src[LOADS], b_src[LOADS];
  const int a_slot_row = lane >> 3;                      // row of this lane's slot inside an A KB
  const int b_slot_k = lane / S::B_CHUNKS;               // k row of this lane's slot inside a B KB
  const int b_slot_pos = lane % S::B_CHUNKS;             // chunk position inside that k row

  int seg = 0, kpos = 0;
  SegDev sd;
  // state of the step whose loads were issued last (the one being landed into LDS)
  gptr st_a = nullptr, st_b = nullptr;                   // base addresses of the step
  int64_t st_a_left = 0, st_b_left = 0;                  // readable bytes from those bases
  int st_krem = 0;                                       // k elements of the segment left at the step
  bool st_fix = false;                                   // the step needs patching before it is published

  auto open_segment = [&]() {
    sd = segs[it.seg_begin + seg];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int row = (i * NW + wave) * 8 + a_slot_row;
      const int src_row = row < it.m_ext ? row : it.m_ext - 1;
      const int c = (lane & 7) ^ a_swizzle(row);
      a_src[i] = (unsigned)(((int64_t)src_row * sd.lda + c * PER) * ES);
    }
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int k = (i * NW + wave) * B_ROWS_PER_KB + b_slot_k;
      const int c = b_swizzle_chunk<ES>(k, b_slot_pos);
      b_src[i] = (unsigned)(((int64_t)k * sd.ldb + c * PER) * ES);
    }
  };

  // issue the loads of the K step at (seg, kpos) into LDS stage `stage`
  auto fetch = [&](int stage) {
    const unsigned sa = lds_base + stage * STAGE + wave * 1024;
    st_a = (gptr)sd.a + ((int64_t)it.m_off * sd.lda + kpos) * ES;
    st_b = (gptr)sd.b + ((int64_t)kpos * sd.ldb + it.n_off) * ES;
    st_a_left = sd.a_bytes - ((int64_t)it.m_off * sd.lda + kpos) * ES;
    st_b_left = sd.b_bytes - ((int64_t)kpos * sd.ldb + it.n_off) * ES;
    st_krem = sd.klen - kpos;
    // largest offset any lane uses in this step, against the last offset that is safe to read 16 bytes at
    const int rows = it.m_ext < BM ? it.m_ext : BM;
    const int64_t a_max = ((int64_t)(rows - 1) * sd.lda + 7 * PER) * ES;
    const int64_t b_max = ((int64_t)(BK - 1) * sd.ldb + (S::B_CHUNKS - 1) * PER) * ES;
    const bool safe = a_max + 16 <= st_a_left && b_max + 16 <= st_b_left;
    st_fix = !safe || st_krem < BK;
    if (safe) {
#pragma unroll
      for (int i = 0; i < LOADS; ++i) load_to_lds_16(st_a, a_src[i], sa + i * (NW * 1024));
#pragma unroll
      for (int i = 0; i < LOADS; ++i) load_to_lds_16(st_b, b_src[i], sa + A_STAGE + i * (NW * 1024));
    } else {
#pragma unroll
      for (int i = 0; i < LOADS; ++i)
        if ((int64_t)a_src[i] + 16 <= st_a_left) load_to_lds_16(st_a, a_src[i], sa + i * (NW * 1024));
#pragma unroll
      for (int i = 0; i < LOADS; ++i)
        if ((int64_t)b_src[i] + 16 <= st_b_left) load_to_lds_16(st_b, b_src[i], sa + A_STAGE + i * (NW * 1024));
    }
  };

  // After this wave's loads have landed: every lane repairs its own slots of stage `stage`:
  // chunks it was masked out of are read element by element, and everything at k >= st_krem
  // is zeroed on both operands (so that stale or non-finite bytes cannot reach a sum).
  auto fixup = [&](int stage) {
    char *sa = lds + stage * STAGE + wave * 1024 + lane * 16;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int row = (i * NW + wave) * 8 + a_slot_row;
      const int c = (lane & 7) ^ a_swizzle(row);
      int keep = st_krem - c * PER;                       // elements of the chunk inside the segment
      keep = keep > PER ? PER : keep;
      u32x4 *slot = (u32x4 *)(sa + i * (NW * 1024));
      const int64_t room = st_a_left - (int64_t)a_src[i];  // readable bytes at the chunk
      if (room < 16) {
        const int avail = (int)(room > 0 ? room / ES : 0);
        *slot = load_partial<ES>(st_a + a_src[i], keep < avail ? keep : avail);
      } else if (keep <= 0) {
        *slot = u32x4{0u, 0u, 0u, 0u};
      } else if (keep < PER) {
        *slot = keep_first<ES>(*slot, keep);
      }
    }
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int k = (i * NW + wave) * B_ROWS_PER_KB + b_slot_k;
      u32x4 *slot = (u32x4 *)(sa + A_STAGE + i * (NW * 1024));
      const int64_t room = st_b_left - (int64_t)b_src[i];
      if (k >= st_krem) {
        *slot = u32x4{0u, 0u, 0u, 0u};
      } else if (room < 16) {
        *slot = load_partial<ES>(st_b + b_src[i], (int)(room > 0 ? room / ES : 0));
      }
    }
  };

  auto advance = [&]() {                                 // to the next K step (the caller knows one exists)
    kpos += BK;
    if (kpos >= sd.klen) {
      ++seg;
      kpos = 0;
      open_segment();
    }
  };

  // ---- LDS -> registers -> MFMA, software-pipelined over the KSUB sub-steps of a K step ----
  // A K step is consumed in KSUB sub-steps (16 k for bf16, 8 k for fp32).  The fragments of
  // sub-step q + 1 are read from LDS while the MFMAs of sub-step q run; the last sub-step's
  // MFMAs are issued after the barrier so that they overlap the first reads of the next stage.
  using Frags = FragSet<ES, FM, FN>;
  Frags fr[2];

  auto load_frags = [&](int stage, int q, Frags &f) {
    const char *sa = lds + stage * STAGE;
    const char *sb = sa + A_STAGE;
    if constexpr (ES == 2) {
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int row = wm * WTM + i * 32 + (lane & 31);
        f.a[i] = *(const bf16x8 *)(sa + a_lds_off(row, q * 2 + (lane >> 5)));
      }
      // ds_read_b64_tr_b16: in every group of 16 lanes, lane i supplies the address of 4
      // consecutive columns of k row i / 4 and receives column i of those 4 k rows.
      const int g = lane >> 4, li = lane & 15;
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int ncol = wn * WTN + j * 32 + (g & 1) * 16 + (li & 3) * 4;   // 4 columns, 8 bytes
        const int k0 = q * 16 + (g >> 1) * 8 + (li >> 2);
        short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_short4_ptr)(sb + b_lds_off<2>(k0, ncol >> 3) + (ncol & 7) * 2));
        short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_short4_ptr)(sb + b_lds_off<2>(k0 + 4, ncol >> 3) + (ncol & 7) * 2));
        union { short4_t h[2]; bf16x8 v; } u;
        u.h[0] = lo;
        u.h[1] = hi;
        f.b[j] = u.v;
      }
    } else {
      // fp32: lane half h reads the float4 at k = 8 q + 4 h .. + 3 of its A row; MFMA number e
      // consumes element e, i.e. k = 8 q + 4 h + e, and the B side reads that same k row.
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int row = wm * WTM + i * 32 + (lane & 31);
        f.a[i] = *(const float4 *)(sa + a_lds_off(row, q * 2 + (lane >> 5)));
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = q * 8 + (lane >> 5) * 4 + e;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const int ncol = wn * WTN + j * 32 + (lane & 31);
          f.b[e][j] = *(const float *)(sb + b_lds_off<4>(k, ncol >> 2) + (ncol & 3) * 4);
        }
      }
    }
  };
  auto mma = [&](const Frags &f) {
    if constexpr (ES == 2) {
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < FM; ++i) {
          const float av = e == 0 ? f.a[i].x : e == 1 ? f.a[i].y : e == 2 ? f.a[i].z : f.a[i].w;
#pragma unroll
          for (int j = 0; j < FN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, f.b[e][j], acc[i][j], 0, 0, 0);
        }
    }
  };
  // pin the order: one LDS read after every MFMA of the previous sub-step
  auto interleave = [&]() {
#ifdef DMM_NO_INTERLEAVE
    return;
#endif
    if constexpr (ES == 2) {
      constexpr int READS = FM + 2 * FN;
#pragma unroll
      for (int n = 0; n < FM * FN; ++n) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);              // 1 MFMA
        if (n < READS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
      }
    }
  };

  if (it.nsteps > 0) {
    open_segment();
    fetch(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#ifndef DMM_NO_FIXUP
    if (st_fix) fixup(0);
#endif
    __syncthreads();
    int stage = 0;
    load_frags(0, 0, fr[0]);
#pragma clang loop unroll(disable)
    for (int s = 0; s < it.nsteps; ++s) {
      st_fix = false;
      if (s + 1 < it.nsteps) {                 // global loads of the next step fly during the MFMAs
        advance();
        fetch(stage ^ 1);
      }
      DMM_SCHED_BARRIER;
#pragma unroll
      for (int q = 0; q + 1 < KSUB; ++q) {
        load_frags(stage, q + 1, fr[(q + 1) & 1]);
        mma(fr[q & 1]);
        interleave();
        DMM_SCHED_BARRIER;
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#ifndef DMM_NO_FIXUP
      if (st_fix) fixup(stage ^ 1);
#endif
      __syncthreads();                         // every wave has read this stage; the next one has landed
      stage ^= 1;
      load_frags(stage, 0, fr[0]);             // (after the last step this reads a stale stage: unused)
      mma(fr[(KSUB - 1) & 1]);
      interleave();
      DMM_SCHED_BARRIER;
    }
  }

  // epilogue: lane holds column (lane & 31), rows 8 (r / 4) + 4 (lane / 32) + r % 4 of each 32 x 32 tile
  gfloat_ptr cbase = (gfloat_ptr)it.c;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int col = wn * WTN + j * 32 + (lane & 31);
      if (col < it.n_ext) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = wm * WTM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (row < it.m_ext) cbase[(int64_t)row * it.ldc + col] = acc[i][j][r];
        }
      }
    }
}

}  // namespace dmm
