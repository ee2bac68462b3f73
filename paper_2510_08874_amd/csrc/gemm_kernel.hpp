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
// Shape of the work
//   4 waves (2 x 2), one per SIMD; wave tile 128 x 128 = 4 x 4 MFMA tiles of
//   32 x 32 (256 accumulator registers per lane, held in AGPRs).
//   K step: 64 bytes of every A row = 32 bf16 or 16 fp32, consumed as two MFMA
//   sub-steps (v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32).
//   LDS: a ring of 4 stages of 32 KB (A: 256 rows x 64 B, B: K rows x 256 columns).
//   16-byte chunks are XOR-swizzled (A by row, B by k) so that ds_read_b128 of A
//   fragments and ds_read_b64_tr_b16 of B fragments are free of bank conflicts.
//
// Global -> LDS
//   global_load_lds_dwordx4: every lane moves 16 bytes from an arbitrary global
//   address to LDS, lane l landing at M0 + 16 l, with no register staging.  A wave
//   fills 1 KB per instruction (16 A rows, or 2 / 1 B rows); the swizzle is realised
//   by permuting which global chunk a lane fetches.  Sources need only element
//   alignment (odd leading dimensions are fine).
//   A CU's memory pipeline takes ~16-20 cycles per such instruction and stalls the
//   issuing wave meanwhile, and with one wave per SIMD a stalled wave starves its
//   matrix pipe.  So the loads are not issued in bursts: the loads of step s + 3 are
//   spread over the MFMA stream of step s, one per four MFMAs per wave, and the four
//   waves use different slots (the loop body is instantiated once per wave with a
//   rotated schedule), so that at most one wave of the CU issues a load in any slot.
//   Data therefore has more than two K steps (> 2000 cycles) to land.
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

#include <type_traits>

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

struct ItemDev {         // one macro-tile, or a run of K steps of one
  void *c;               // top-left of the macro-tile in the C tile (or in a partial-sum buffer)
  int64_t ldc;           // elements
  int32_t seg_begin;
  int32_t nsteps;        // K steps this item performs; 0 = zero fill
  int32_t m_off, n_off;  // offset inside the group's sub-tile
  int32_t m_ext, n_ext;
  int32_t first_step;    // where it starts in the group's step sequence (steps of a segment:
                         // ceil(klen / K step); the sequence runs over the segments in order)
  int32_t c_es;          // bytes per element of the destination: 4 = fp32, 2 = bf16 (rounded to nearest even)
  int32_t red_first;     // fused replica sum: the other replicas' partial sums of this macro-tile are
  int32_t red_count;     // added before the store, red[red_first .. + red_count) in that order (0: none)
};

struct RedSrc {          // one other replica's partial sum of a macro-tile: its top-left element, its pitch
  const float *p;
  int64_t ld;            // elements
};

// Merged macro-tiles.  Where the tiles of A, B and C are small against 256 x 256, a macro-tile may
// cover several output sub-tiles at once: its rows fall into up to PMAX row pieces (rows of one
// A tile and one C tile each), its columns into up to PMAX column pieces (one B tile, one C
// tile), and every K-segment then names one A slice per row piece and one B slice per column
// piece.  A lane's loads go to whichever piece holds its row or its 16-byte chunk of columns
// (column pieces start at multiples of eight columns, so a chunk never straddles two B tiles).
constexpr int PMAX = 8;

struct PieceDev {        // one slice of a tile: where it starts, how far one may read, its row pitch
  const char *ptr;
  int64_t room;          // readable bytes from ptr to the end of the tile buffer
  uint32_t pitch;        // bytes
  uint32_t pad;
};

struct CompItemDev {     // one merged macro-tile
  int32_t m_ext, n_ext;
  int32_t R, Q, S;       // row pieces, column pieces, K-segments
  int32_t nsteps;        // K steps over all segments
  int32_t c_es;          // bytes per element of C
  int32_t a_first, a_stride;   // A slice of (row piece p, segment s): a_pieces[a_first + p * a_stride + s]
  int32_t b_first, b_stride;   // B slice of (segment s, column piece q): b_pieces[b_first + s * b_stride + q]
  int32_t c_first, c_stride;   // C slice of (p, q): c_pieces[c_first + p * c_stride + q]
  int32_t k_first;             // length of segment s: klen[k_first + s]
  int32_t rb[PMAX + 1];        // first row of every row piece relative to the macro-tile (rb[0] <= 0: the
                               // first piece may begin above it), rb[R] >= m_ext
  int32_t cb[PMAX + 1];        // likewise for the column pieces
  float *scratch;              // a run of K steps of a macro-tile cut along K: its partial sums go here, as a
                               // plain 256-wide fp32 tile, instead of to the C slices (null otherwise)
  int32_t first_step;          // where the run starts in the macro-tile's step sequence
  int32_t pad;
};

struct CompCtx {         // a merged macro-tile's descriptors, staged in LDS behind the stages
  const int32_t *klen;   // [S]
  const PieceDev *ad;    // [S][R]
  const PieceDev *bd;    // [S][Q]
  const int32_t *rb, *cb;
  int R, Q;
};

constexpr int BM = 256, BN = 256;
constexpr int A_ROW = 64;                     // bytes of an A row per K step
constexpr int A_STAGE = BM * A_ROW;           // 16 KB
constexpr int B_STAGE = 16 * 1024;            // 32 x 512 B (bf16) or 16 x 1024 B (fp32)
constexpr int STAGE = A_STAGE + B_STAGE;      // 32 KB
constexpr int NSTAGE = 4;
constexpr int LDS_BYTES = NSTAGE * STAGE;     // 128 KB
constexpr int DESC_LDS = 32 * 1024;           // behind the stages: a merged macro-tile's descriptors
constexpr int DESC_GEO = 2048;                // ... of which the piece boundaries and the C slices take the first bytes
constexpr int NW = 4;                         // waves per workgroup, 2 x 2
constexpr int NT = 64 * NW;
constexpr int WAVES_N = 2;
constexpr int WTM = 128, WTN = 128;           // wave tile
constexpr int FM = 4, FN = 4;                 // MFMA tiles of 32 x 32 per wave
constexpr int LOADS = 16 / NW;                // wave-wide 1 KB loads per wave, per operand, per K step
constexpr int KSUB = 2;                       // MFMA sub-steps per K step
constexpr int SLOTS = KSUB * FM * FN;         // MFMA slots per K step (32)
static_assert(LOADS == 4 && SLOTS == 2 * LOADS * NW, "the load slots of run_item are written out for 8 loads per step");

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4_t *lds_short4_ptr;
typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(3))) char *lds_cptr;
// Pointers read from the work table would otherwise be treated as generic (flat) addresses.
typedef const __attribute__((address_space(1))) char *gptr;
typedef __attribute__((address_space(1))) float *gfloat_ptr;
typedef __attribute__((address_space(1))) unsigned short *gushort_ptr;

template <int ES>
struct Shape;
template <>
struct Shape<2> {                              // bf16
  static constexpr int BK = 32;                // elements per K step
  static constexpr int B_ROW = 512;            // bytes per k row of the B stage
  static constexpr int B_CHUNKS = 32;          // 16-byte chunks per k row
};
template <>
struct Shape<4> {                              // fp32
  static constexpr int BK = 16;
  static constexpr int B_ROW = 1024;
  static constexpr int B_CHUNKS = 64;
};

template <int ES>
struct FragSet;
template <>
struct FragSet<2> {                // bf16: A rows x 8 k and B columns x 8 k per lane
  bf16x8 a[FM];
  short4_t b[FN][2];
};
template <>
struct FragSet<4> {                // fp32: A rows x 4 k per lane; B value per MFMA e and column block
  f32x4 a[FM];
  float b[4][FN];
};

// A stage: row r at r * 64, its four 16-byte chunks XOR-ed with a function of the row that
// spreads both 8 and 16 consecutive rows reading the same logical chunk over all banks.
__device__ __forceinline__ int a_swizzle(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }
__device__ __forceinline__ int a_lds_off(int row, int c) { return row * A_ROW + ((c ^ a_swizzle(row)) << 4); }

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
// serialise it against LDS reads of *other* stages (it cannot tell the stages apart and
// would wait for vmcnt(0) before every ds_read); completion is awaited explicitly with
// s_waitcnt vmcnt before the barrier that publishes a stage.
__device__ __forceinline__ void load_to_lds_16(gptr base, unsigned lane_off, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_off), "s"(base), "s"(lds_base)
               : "memory");
}
// (M0 and EXEC cannot be named as clobbered: the compiler treats both as reserved, refuses them
// in a clobber list with a warning, and never carries a value of its own in M0 across a statement:
// it writes M0 right in front of each instruction of its own that reads it.  The masked forms
// leave EXEC at all ones: they are only ever reached in wave-uniform control flow with every lane
// active, which is how the whole of run_item runs; the divergent repairs of publish_fix use none
// of them.)
// The form used in the K loop: the LDS address is a wave-uniform base plus a compile-time
// constant, and the lanes that take part are given as an exec mask (all ones for an ordinary
// step, fewer when some lanes would overrun a tile buffer, zero when there is nothing to load),
// so a load slot is five instructions and no branch.  Every instruction costs a wave at
// least 4 issue cycles and only about seven fit in the shadow of one MFMA.  The s_mov to exec
// doubles as the wait state required between the M0 write and the LDS-DMA instruction.
template <int IMM>
__device__ __forceinline__ void load_to_lds_16_masked(gptr base, unsigned lane_off, unsigned lds_base,
                                                      unsigned lo, unsigned hi) {
  asm volatile("s_add_u32 m0, %2, %3\n\ts_mov_b32 exec_lo, %4\n\ts_mov_b32 exec_hi, %5\n\t"
               "global_load_lds_dwordx4 %0, %1\n\ts_mov_b64 exec, -1"
               :
               : "v"(lane_off), "s"(base), "s"(lds_base), "n"(IMM), "s"(lo), "s"(hi)
               : "memory", "scc");
}

// The form of the quiet iterations of the K loop, where every lane takes part for certain: no exec
// mask to set and restore, two instructions fewer per load slot (s_nop is the wait state between
// the M0 write and the LDS-DMA instruction).
template <int IMM>
__device__ __forceinline__ void load_to_lds_16_plain(gptr base, unsigned lane_off, unsigned lds_base) {
  asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_off), "s"(base), "s"(lds_base), "n"(IMM)
               : "memory", "scc");
}
template <int IMM>
__device__ __forceinline__ void load_to_lds_16_plain_v(gptr addr, unsigned lds_base) {
  asm volatile("s_add_u32 m0, %1, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(addr), "s"(lds_base), "n"(IMM)
               : "memory", "scc");
}

// The same two forms with a full 64-bit address per lane (merged macro-tiles: the lanes of one
// instruction read from different tile buffers).
__device__ __forceinline__ void load_to_lds_16_v(gptr addr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(addr), "s"(lds_base)
               : "memory");
}
template <int IMM>
__device__ __forceinline__ void load_to_lds_16_masked_v(gptr addr, unsigned lds_base, unsigned lo, unsigned hi) {
  asm volatile("s_add_u32 m0, %1, %2\n\ts_mov_b32 exec_lo, %3\n\ts_mov_b32 exec_hi, %4\n\t"
               "global_load_lds_dwordx4 %0, off\n\ts_mov_b64 exec, -1"
               :
               : "v"(addr), "s"(lds_base), "n"(IMM), "s"(lo), "s"(hi)
               : "memory", "scc");
}

// p + d where the caller knows that the low half of the address does not carry.
__device__ __forceinline__ gptr add_low(gptr p, unsigned d) {
  const uint64_t a = (uint64_t)(uintptr_t)p;
  return (gptr)(uintptr_t)((a & 0xFFFFFFFF00000000ull) | (uint32_t)((uint32_t)a + d));
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

// ---- the accumulators ----------------------------------------------------------------------
// The 256 partial sums of a lane live in the accumulator registers a0 .. a255 by name: tile (i, j)
// of the wave's 4 x 4 tiles of 32 x 32 owns a[16 t .. 16 t + 15], t = 4 i + j.  Every instruction
// that touches them is written out below with those names, so the register allocator has no say
// in where they are.  (Held in C++ variables tied to the MFMAs' operands, the item loop's joins
// made it shuffle all 256 of them, or spill them around single MFMAs.)  Each of these statements
// names the whole file as clobbered: the compiler must never keep a value of its own in it.
#define DMM_ACC_REGS "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63", "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95", "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127", "a128", "a129", "a130", "a131", "a132", "a133", "a134", "a135", "a136", "a137", "a138", "a139", "a140", "a141", "a142", "a143", "a144", "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", "a153", "a154", "a155", "a156", "a157", "a158", "a159", "a160", "a161", "a162", "a163", "a164", "a165", "a166", "a167", "a168", "a169", "a170", "a171", "a172", "a173", "a174", "a175", "a176", "a177", "a178", "a179", "a180", "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191", "a192", "a193", "a194", "a195", "a196", "a197", "a198", "a199", "a200", "a201", "a202", "a203", "a204", "a205", "a206", "a207", "a208", "a209", "a210", "a211", "a212", "a213", "a214", "a215", "a216", "a217", "a218", "a219", "a220", "a221", "a222", "a223", "a224", "a225", "a226", "a227", "a228", "a229", "a230", "a231", "a232", "a233", "a234", "a235", "a236", "a237", "a238", "a239", "a240", "a241", "a242", "a243", "a244", "a245", "a246", "a247", "a248", "a249", "a250", "a251", "a252", "a253", "a254", "a255"

template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>): a loop whose index is a constant
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F &&>(f));
}

// all partial sums = 0: 0 * 0 + 0 through the matrix pipe, one instruction per tile
template <int ES, int T>
__device__ __forceinline__ void acc_clear_tile(u32x4 z) {
  if constexpr (ES == 2)
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%1:%2], %0, %0, 0" : : "v"(z), "n"(16 * T), "n"(16 * T + 15) : DMM_ACC_REGS);
  else
    asm volatile("v_mfma_f32_32x32x2_f32 a[%1:%2], %0, %0, 0" : : "v"(z[0]), "n"(16 * T), "n"(16 * T + 15) : DMM_ACC_REGS);
}
template <int ES, int... T>
__device__ __forceinline__ void acc_clear_tiles(u32x4 z, std::integer_sequence<int, T...>) {
  (acc_clear_tile<ES, T>(z), ...);
}
template <int ES>
__device__ __forceinline__ void acc_clear() {
  u32x4 z = {0u, 0u, 0u, 0u};
  // (the zeros have just been written by vector moves: the matrix pipe must not read them in the
  // very next cycles, and the compiler, which inserts such wait states, does not look into assembly)
  asm volatile("s_nop 7" : "+v"(z));
  acc_clear_tiles<ES>(z, std::make_integer_sequence<int, FM * FN>{});
}
// partial sum number REG to base + off + IMM (a non-temporal store straight from the accumulator file).
// The base travels in a scalar register pair.  Where the compiler has only just fetched that pair with
// a vector instruction (v_readlane from a spill lane, v_readfirstlane), a memory instruction must not
// read it for five cycles; the compiler inserts such wait states between its own instructions but does
// not look into assembly, so the statement brings them along.
template <int REG, int IMM>
__device__ __forceinline__ void acc_store(unsigned off, const __attribute__((address_space(1))) char *base) {
  asm volatile("s_nop 4\n\tglobal_store_dword %0, a[%2], %1 offset:%3 nt" : : "v"(off), "s"(base), "n"(REG), "n"(IMM) : "memory");
}
// one row of a full macro-tile: partial sums R0, R0 + 16, R0 + 32, R0 + 48 (the row's four column blocks)
template <int R0>
__device__ __forceinline__ void acc_store_row(unsigned off, const __attribute__((address_space(1))) char *base) {
  asm volatile("s_nop 4\n\t"
               "global_store_dword %0, a[%2], %1 offset:0 nt\n\t"
               "global_store_dword %0, a[%3], %1 offset:128 nt\n\t"
               "global_store_dword %0, a[%4], %1 offset:256 nt\n\t"
               "global_store_dword %0, a[%5], %1 offset:384 nt"
               : : "v"(off), "s"(base), "n"(R0), "n"(R0 + 16), "n"(R0 + 32), "n"(R0 + 48) : "memory");
}
// partial sum number REG (= 16 t + r) as a value
template <int REG>
__device__ __forceinline__ float acc_read() {
  float v;
  asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(v) : "n"(REG));
  return v;
}
// partial sum number REG := v
template <int REG>
__device__ __forceinline__ void acc_write(float v) {
  asm volatile("v_accvgpr_write_b32 a[%0], %1" : : "n"(REG), "v"(v) : DMM_ACC_REGS);
}

template <bool FUSE>
__device__ __forceinline__ void store_macro_tile(const ItemDev &it, const RedSrc *__restrict__ red, int wm, int wn, int lane);

// The work of one wave on one item, or (LOOP) on every `stride`-th item of the list from number
// `idx` on.  ROT = this wave's index: it selects the MFMA slots in which the wave issues its
// global->LDS loads (slot % 4 == ROT).
// LOOP: the workgroup stays on its CU and walks its share of the work list.  When an item's K
// loop is done, the loads of the next item's first three K steps are issued first and the item's
// C stores second, so that those loads travel while the stores drain; the accumulators are
// cleared behind the stores.  (Without LOOP the caller stores, and `first_item` is the one item.)
template <int ES, int ROT, bool COMP = false, bool LOOP = false, bool FUSE = false>
__device__ __forceinline__ void run_item(const ItemDev &first_item, const SegDev *__restrict__ segs, char *lds,
                                         const CompCtx &cx = CompCtx{},
                                         const ItemDev *__restrict__ items = nullptr, int idx = 0, int stride = 0,
                                         int n_items = 0, const RedSrc *__restrict__ red = nullptr) {
  ItemDev it = first_item;
  using S = Shape<ES>;
  constexpr int BK = S::BK;
  constexpr int PER = 16 / ES;                          // elements per 16-byte chunk
  constexpr int B_ROWS_PER_KB = 1024 / S::B_ROW;        // k rows one wave-wide load covers
  constexpr int wave = ROT;
  constexpr int wm = wave / WAVES_N, wn = wave % WAVES_N;

  const int lane = threadIdx.x & 63;
  const unsigned lds_base = (unsigned)(uintptr_t)(lds_void_ptr)lds;   // LDS byte address of stage 0
  const lds_cptr lds3 = (lds_cptr)(lds_void_ptr)lds;
  // Stage 2's address in a register of its own that the optimiser cannot see through: an LDS
  // instruction's immediate offset reaches 64 KB, so with this second base every read address of
  // the iterations that know their stage is one of a few per-lane registers plus an immediate.
  // (Seen through, base + 64 KB + ... is folded into a separate address register per read.)
  lds_cptr lds3_hi = lds3 + 2 * STAGE;
  asm volatile("" : "+v"(lds3_hi));

  // ---- global -> LDS ------------------------------------------------------------------
  // Wave w, load i fills KB number NW i + w of the A stage (rows 16 (NW i + w) .. + 15) and KB
  // number NW i + w of the B stage (k rows B_ROWS_PER_KB (NW i + w) ..).  Lane l owns the slot at
  // +16 l of that KB.
  const int a_slot_row = lane >> 2;                      // row of this lane's slot inside an A KB
  const int a_slot_pos = lane & 3;                       // chunk position inside that row
  const int b_slot_k = lane / S::B_CHUNKS;               // k row of this lane's slot inside a B KB
  const int b_slot_pos = lane % S::B_CHUNKS;             // chunk position inside that k row

  // Byte offset, from a step's base address, of the chunk this lane fetches with load i:
  // (source row) * (row pitch in bytes) + (chunk inside the row) * 16.  The row and the chunk
  // depend on the item only; the pitch is a scalar of the segment.  So a segment switch touches
  // scalars only, and a load slot rebuilds its offset with one 24-bit multiply-add (pitches are
  // below 2^24 bytes: the host rejects larger leading dimensions).
  unsigned a_srow[LOADS], a_c16[LOADS], b_srow[LOADS], b_c16[LOADS];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int row = (i * NW + wave) * 16 + a_slot_row;
    a_c16[i] = (unsigned)((a_slot_pos ^ a_swizzle(row)) << 4);
    const int k = (i * NW + wave) * B_ROWS_PER_KB + b_slot_k;
    b_srow[i] = (unsigned)k;
    b_c16[i] = (unsigned)(b_swizzle_chunk<ES>(k, b_slot_pos) << 4);
  }
  auto set_rows = [&]() {                                // the source rows depend on the item's height
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int row = (i * NW + wave) * 16 + a_slot_row;
      a_srow[i] = (unsigned)(row < it.m_ext ? row : it.m_ext - 1);
    }
  };
  set_rows();
  auto a_offset = [&](unsigned pitch, int i) -> unsigned { return __umul24(a_srow[i], pitch) + a_c16[i]; };
  auto b_offset = [&](unsigned pitch, int i) -> unsigned { return __umul24(b_srow[i], pitch) + b_c16[i]; };
  // Merged macro-tiles: the piece that holds each of this lane's four A rows and four B chunks, the
  // row inside that piece and the byte column inside that piece; then, per segment, a full address
  // per load (ca, cbv), advanced by the load slot itself after every load, and the bytes one K
  // step advances in B (the pitch of the lane's own B tile).  The slot adds to the low half of the
  // address only (a 64-bit add costs the wave three times as long); a segment in which some
  // lane's address would carry into the high half is loaded step by step from freshly computed
  // addresses instead, like a segment that touches the end of a tile buffer.
  int ap[LOADS], bp[LOADS];
  unsigned a_lrow[LOADS], b_lcol[LOADS];
  gptr ca[LOADS], cbv[LOADS];
  unsigned bstep[LOADS];
  if constexpr (COMP) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int crow = (int)a_srow[i];
      int p = 0, base = cx.rb[0];
#pragma unroll
      for (int x = 1; x < PMAX; ++x)
        if (x < cx.R && cx.rb[x] <= crow) { p = x; base = cx.rb[x]; }
      ap[i] = p;
      a_lrow[i] = (unsigned)(crow - base);
      const int col = (int)(b_c16[i] >> 4) * PER;
      int q = 0, cbase = cx.cb[0];
#pragma unroll
      for (int x = 1; x < PMAX; ++x)
        if (x < cx.Q && cx.cb[x] <= col) { q = x; cbase = cx.cb[x]; }
      bp[i] = q;
      b_lcol[i] = (unsigned)(col - cbase) * ES;
      ca[i] = cbv[i] = nullptr;
      bstep[i] = 0;
    }
  }
  auto seg_klen = [&](int seg) -> int {
    if constexpr (COMP) return cx.klen[seg];
    else return segs[it.seg_begin + seg].klen;
  };
  // address of, and readable bytes at, this lane's chunk of load i in the K step at (seg, kpos)
  auto a_chunk = [&](int seg, int kpos, int i, gptr &p, int64_t &room) {
    if constexpr (COMP) {
      const PieceDev d = cx.ad[seg * cx.R + ap[i]];
      const int64_t off = (int64_t)a_lrow[i] * d.pitch + a_c16[i] + (int64_t)kpos * ES;
      p = (gptr)d.ptr + off;
      room = d.room - off;
    } else {
      const SegDev sd = segs[it.seg_begin + seg];
      const int64_t o0 = ((int64_t)it.m_off * sd.lda + kpos) * ES;
      const unsigned off = a_offset((unsigned)(sd.lda * ES), i);
      p = (gptr)sd.a + o0 + off;
      room = sd.a_bytes - o0 - (int64_t)off;
    }
  };
  auto b_chunk = [&](int seg, int kpos, int i, gptr &p, int64_t &room) {
    if constexpr (COMP) {
      const PieceDev d = cx.bd[seg * cx.Q + bp[i]];
      const int64_t off = (int64_t)(kpos + (int)b_srow[i]) * d.pitch + b_lcol[i];
      p = (gptr)d.ptr + off;
      room = d.room - off;
    } else {
      const SegDev sd = segs[it.seg_begin + seg];
      const int64_t o0 = ((int64_t)kpos * sd.ldb + it.n_off) * ES;
      const unsigned off = b_offset((unsigned)(sd.ldb * ES), i);
      p = (gptr)sd.b + o0 + off;
      room = sd.b_bytes - o0 - (int64_t)off;
    }
  };

  // `lead` is the K step whose loads are being issued (three steps ahead of the one being
  // multiplied).  Whatever is done between two K steps is exposed (nothing hides it), so the loop
  // has a quiet mode: while the lead stays inside a segment, away from its K tail and from the
  // end of the tile buffers, and no stage waits for a repair, an iteration only bumps two
  // addresses and a counter.  Everything else (segment switches, tails, buffer ends, the drain
  // at the end of the item) goes through the general bookkeeping below, a few times per segment.
  int lead_seg = 0, lead_kpos = 0;                       // lead cursor
  int lead_left = 0;                                     // steps left in its segment, the current one included
  bool lead_tail = false;                                // the segment's last step is a K tail
  int lead_unsafe = 0;                                   // the segment's last this-many steps may overrun a tile buffer
  bool lead_seg_carry = false;                           // (merged items) some lane's address crosses a 4 GB line in it
  unsigned ld_a_pitch = 0, ld_b_pitch = 0;               // row pitch in bytes of the lead segment's A and B tiles
  unsigned ld_a_off[LOADS], ld_b_off[LOADS];             // this lane's byte offsets at those pitches (per segment)
  gptr ld_a = nullptr, ld_b = nullptr;                   // base addresses of the lead step
  gptr ld_a_next = nullptr, ld_b_next = nullptr;         // ... and of the step after it, if in the same segment
  int64_t ld_b_step = 0;                                 // bytes one K step advances in B
  unsigned ld_lo = 0, ld_hi = 0;                         // exec mask of the lead step's loads: all lanes or none
  // Repair flags as a shift register: every prepared step pushes one bit; the step that is
  // published in an iteration is the one pushed three pushes earlier (bit 2).
  unsigned fix_bits = 0;

  // geometry of the K step at (sd, kpos): base addresses and the bytes readable from them
  auto step_geometry = [&](const SegDev &sd, int kpos, gptr &pa, gptr &pb, int64_t &a_left, int64_t &b_left) {
    pa = (gptr)sd.a + ((int64_t)it.m_off * sd.lda + kpos) * ES;
    pb = (gptr)sd.b + ((int64_t)kpos * sd.ldb + it.n_off) * ES;
    a_left = sd.a_bytes - ((int64_t)it.m_off * sd.lda + kpos) * ES;
    b_left = sd.b_bytes - ((int64_t)kpos * sd.ldb + it.n_off) * ES;
  };
  // bytes a step reads at most from its base addresses
  auto step_need = [&](const SegDev &sd, int64_t &a_need, int64_t &b_need) {
    const int rows = it.m_ext < BM ? it.m_ext : BM;
    a_need = ((int64_t)(rows - 1) * sd.lda + 3 * PER) * ES + 16;
    b_need = ((int64_t)(BK - 1) * sd.ldb + (S::B_CHUNKS - 1) * PER) * ES + 16;
  };
  // the lead enters, at kpos0 (a multiple of BK), the segment whose record is sd
  auto open_lead_at = [&](const SegDev &sd, int kpos0) {
    lead_kpos = kpos0;
    lead_left = (sd.klen - kpos0 + BK - 1) / BK;
    lead_tail = sd.klen % BK != 0;
    ld_a_pitch = (unsigned)(sd.lda * ES);
    ld_b_pitch = (unsigned)(sd.ldb * ES);
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      ld_a_off[i] = a_offset(ld_a_pitch, i);
      ld_b_off[i] = b_offset(ld_b_pitch, i);
    }
    ld_b_step = (int64_t)BK * sd.ldb * ES;
    int64_t a_left, b_left, a_need, b_need;
    step_geometry(sd, kpos0, ld_a, ld_b, a_left, b_left);
    step_need(sd, a_need, b_need);
    // A later step reads further.  Where a segment ends at the end of its tile, its last step (a K
    // tail, as a rule) reaches past the tile buffer in the tile's last rows, and only that step:
    // so the question is how many steps at the end of the segment are not safe, not whether all are.
    lead_unsafe = lead_left;
#pragma unroll
    for (int u = 3; u >= 0; --u) {
      const int64_t last = (int64_t)lead_left - 1 - u;   // the step in front of the last u
      if (last >= 0 && a_left - last * (BK * ES) >= a_need && b_left - last * ld_b_step >= b_need) lead_unsafe = u;
    }
  };
  auto open_lead = [&](int kpos0) {                      // lead enters segment lead_seg at kpos0 (a multiple of BK)
    if constexpr (COMP) {
      const int klen = seg_klen(lead_seg);
      lead_kpos = kpos0;
      lead_left = (klen - kpos0 + BK - 1) / BK;
      lead_tail = klen % BK != 0;
      const int64_t more = lead_left - 1;                // the segment's last step reads furthest
      bool overrun = false, overrun1 = false, carry = false;   // overrun1: already in the step before the last
#pragma unroll
      for (int i = 0; i < LOADS; ++i) {
        int64_t room;
        a_chunk(lead_seg, kpos0, i, ca[i], room);
        overrun |= room - more * (BK * ES) < 16;
        overrun1 |= room - (more - 1) * (BK * ES) < 16;
        carry |= (uint64_t)(uint32_t)(uintptr_t)ca[i] + (uint64_t)more * (BK * ES) > 0xFFFFFFFFull;
      }
#pragma unroll
      for (int i = 0; i < LOADS; ++i) {
        int64_t room;
        b_chunk(lead_seg, kpos0, i, cbv[i], room);
        bstep[i] = (unsigned)BK * cx.bd[lead_seg * cx.Q + bp[i]].pitch;
        overrun |= room - more * (int64_t)bstep[i] < 16;
        overrun1 |= room - (more - 1) * (int64_t)bstep[i] < 16;
        carry |= (uint64_t)(uint32_t)(uintptr_t)cbv[i] + (uint64_t)more * bstep[i] > 0xFFFFFFFFull;
      }
      lead_seg_carry = __builtin_amdgcn_ballot_w64(carry) != 0;
      // none, the last step only, or (also where an address would carry) all of them
      lead_unsafe = lead_seg_carry ? lead_left
                    : __builtin_amdgcn_ballot_w64(overrun) == 0 ? 0
                    : (more >= 1 && __builtin_amdgcn_ballot_w64(overrun1) == 0) ? 1 : lead_left;
      return;
    }
    open_lead_at(segs[it.seg_begin + lead_seg], kpos0);
  };
  auto advance_lead = [&]() {                            // to the next K step (the caller knows one exists)
    if (__builtin_expect(--lead_left == 0, 0)) {
      ++lead_seg;
      open_lead(0);
    } else {
      lead_kpos += BK;
      if constexpr (!COMP) {                             // (a merged item's addresses advance in the load slots)
        ld_a += BK * ES;
        ld_b += ld_b_step;
      }
    }
  };
  // Make the lead step ready for the load slots and push its repair flag.  An ordinary step is
  // loaded by the slots with all lanes; when there is no step the slots run with no lane (and
  // move nothing); a step in which some lane would overrun a tile buffer is loaded here and
  // now, lane-masked, and the slots again run empty.  `stage` is the free stage the step goes to.
  auto prepare_lead = [&](bool exists, int stage) {
    unsigned all = 0u;
    unsigned fix = 0u;
    if (exists) {
      fix = lead_tail && lead_left == 1 ? 1u : 0u;
      all = ~0u;
      if (__builtin_expect(lead_left <= lead_unsafe, 0)) {
        if constexpr (COMP) {
          // (addresses computed afresh: in a segment with a carry the slots' own may have wrapped)
          bool a_ok[LOADS], b_ok[LOADS], bad = lead_seg_carry;
          gptr pa[LOADS], pb[LOADS];
#pragma unroll
          for (int i = 0; i < LOADS; ++i) {
            int64_t room;
            a_chunk(lead_seg, lead_kpos, i, pa[i], room);
            a_ok[i] = room >= 16;
            b_chunk(lead_seg, lead_kpos, i, pb[i], room);
            b_ok[i] = room >= 16;
            bad |= !a_ok[i] || !b_ok[i];
          }
          if (__builtin_amdgcn_ballot_w64(bad) != 0) {
            all = 0u;
            fix = 1u;
            const unsigned sa = lds_base + stage * STAGE + wave * 1024;
#pragma unroll
            for (int i = 0; i < LOADS; ++i)
              if (a_ok[i]) load_to_lds_16_v(pa[i], sa + i * (NW * 1024));
#pragma unroll
            for (int i = 0; i < LOADS; ++i)
              if (b_ok[i]) load_to_lds_16_v(pb[i], sa + A_STAGE + i * (NW * 1024));
          }
        } else {
        const SegDev sd = segs[it.seg_begin + lead_seg];
        gptr pa, pb;
        int64_t a_left, b_left, a_need, b_need;
        step_geometry(sd, lead_kpos, pa, pb, a_left, b_left);
        step_need(sd, a_need, b_need);
        if (!(a_left >= a_need && b_left >= b_need)) {
          all = 0u;
          fix = 1u;
          const unsigned sa = lds_base + stage * STAGE + wave * 1024;
#pragma unroll
          for (int i = 0; i < LOADS; ++i) {
            const unsigned off = ld_a_off[i];
            if ((int64_t)off + 16 <= a_left) load_to_lds_16(ld_a, off, sa + i * (NW * 1024));
          }
#pragma unroll
          for (int i = 0; i < LOADS; ++i) {
            const unsigned off = ld_b_off[i];
            if ((int64_t)off + 16 <= b_left) load_to_lds_16(ld_b, off, sa + A_STAGE + i * (NW * 1024));
          }
        }
        }
      }
    }
    fix_bits = (fix_bits << 1) | fix;
    ld_lo = ld_hi = __builtin_amdgcn_readfirstlane(all);
  };
  // load number j of the lead step (0 .. LOADS - 1: A, LOADS .. 2 LOADS - 1: B) into the LDS stage
  // whose base address (plus this wave's KB offset) is `stage_base`
  auto dma = [&](auto jc, unsigned stage_base, auto quiet_tag) {
    constexpr int j = decltype(jc)::value;
    constexpr bool QUIET = decltype(quiet_tag)::value;   // every lane loads: no exec mask
    constexpr int IMM = j < LOADS ? j * (NW * 1024) : A_STAGE + (j - LOADS) * (NW * 1024);
    if constexpr (COMP) {
      if constexpr (j < LOADS) {
        if constexpr (QUIET) load_to_lds_16_plain_v<IMM>(ca[j], stage_base);
        else load_to_lds_16_masked_v<IMM>(ca[j], stage_base, ld_lo, ld_hi);
        ca[j] = add_low(ca[j], BK * ES);
      } else {
        if constexpr (QUIET) load_to_lds_16_plain_v<IMM>(cbv[j - LOADS], stage_base);
        else load_to_lds_16_masked_v<IMM>(cbv[j - LOADS], stage_base, ld_lo, ld_hi);
        cbv[j - LOADS] = add_low(cbv[j - LOADS], bstep[j - LOADS]);
      }
    } else {
      if constexpr (j < LOADS) {
        if constexpr (QUIET) load_to_lds_16_plain<IMM>(ld_a, ld_a_off[j], stage_base);
        else load_to_lds_16_masked<IMM>(ld_a, ld_a_off[j], stage_base, ld_lo, ld_hi);
      } else {
        if constexpr (QUIET) load_to_lds_16_plain<IMM>(ld_b, ld_b_off[j - LOADS], stage_base);
        else load_to_lds_16_masked<IMM>(ld_b, ld_b_off[j - LOADS], stage_base, ld_lo, ld_hi);
      }
    }
  };

  // After this wave's loads of the step being published have landed: every lane repairs its own slots of
  // `stage`: chunks it was masked out of are read element by element, and everything at
  // k >= remaining segment length is zeroed on both operands (so that stale or non-finite
  // bytes cannot reach a sum).  Rare: K tails and tile-buffer ends only.
  int pub_seg = 0, pub_first = 0;                        // cursor of publish_fix: a segment and the number of its first step
  auto publish_fix = [&](int t) {                        // t = number of the step being published
    if (__builtin_expect((fix_bits & 4u) == 0u, 1)) return;
    const int stage = t & 3;
    // find the step's segment and position (the item's steps lie inside the group's sequence).
    // Repairs come in ascending step order, so the search goes on from where the last one ended:
    // one look at a segment's length per segment instead of one per segment per repair.
    const int t_abs = it.first_step + t;
    for (;;) {
      const int cnt = (seg_klen(pub_seg) + BK - 1) / BK;
      if (t_abs < pub_first + cnt) break;
      pub_first += cnt;
      ++pub_seg;
    }
    const int seg = pub_seg, first = pub_first;
    const int kpos = (t_abs - first) * BK;
    const int krem = seg_klen(seg) - kpos;
    char *sa = lds + stage * STAGE + wave * 1024 + lane * 16;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int row = (i * NW + wave) * 16 + a_slot_row;
      const int c = a_slot_pos ^ a_swizzle(row);
      gptr pc;
      int64_t room;                                       // readable bytes at the chunk
      a_chunk(seg, kpos, i, pc, room);
      int keep = krem - c * PER;                          // elements of the chunk inside the segment
      keep = keep > PER ? PER : keep;
      u32x4 *slot = (u32x4 *)(sa + i * (NW * 1024));
      if (room < 16) {
        const int avail = (int)(room > 0 ? room / ES : 0);
        *slot = load_partial<ES>(pc, keep < avail ? keep : avail);
      } else if (keep <= 0) {
        *slot = u32x4{0u, 0u, 0u, 0u};
      } else if (keep < PER) {
        *slot = keep_first<ES>(*slot, keep);
      }
    }
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int k = (i * NW + wave) * B_ROWS_PER_KB + b_slot_k;
      gptr pc;
      int64_t room;
      b_chunk(seg, kpos, i, pc, room);
      u32x4 *slot = (u32x4 *)(sa + A_STAGE + i * (NW * 1024));
      if (k >= krem) {
        *slot = u32x4{0u, 0u, 0u, 0u};
      } else if (room < 16) {
        *slot = load_partial<ES>(pc, (int)(room > 0 ? room / ES : 0));
      }
    }
    // the repairs must have reached LDS before the barrier that publishes the stage (the K loop's
    // barrier is the bare instruction, without the fence of __syncthreads)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  };

  // ---- LDS -> registers ----------------------------------------------------------------
  using Frags = FragSet<ES>;
  Frags fr[2];
  constexpr int READS = ES == 2 ? FM + 2 * FN : FM + 4 * FN;   // LDS reads per sub-step

  // read number r of sub-step q of `stage` into f.  bf16 order: B0 (2 reads), A0, B1, B2, B3, A1..A3,
  // so that the operands of the next sub-step's first MFMAs arrive first.
  auto read_op = [&](lds_cptr sa, int q, int r, Frags &f) {   // sa: the stage
    const lds_cptr sb = sa + A_STAGE;
    if constexpr (ES == 2) {
      constexpr int kind[12] = {4, 4, 0, 5, 5, 6, 6, 7, 7, 1, 2, 3};   // 0..3: A frag i; 4..7: B frag j
      constexpr int half[12] = {0, 1, 0, 0, 1, 0, 1, 0, 1, 0, 0, 0};
      const int what = kind[r];
      if (what < 4) {
        const int row = wm * WTM + what * 32 + (lane & 31);
        f.a[what] = *(const __attribute__((address_space(3))) bf16x8 *)(sa + a_lds_off(row, q * 2 + (lane >> 5)));
      } else {
        // ds_read_b64_tr_b16: in every group of 16 lanes, lane i supplies the address of 4
        // consecutive columns of k row i / 4 and receives column i of those 4 k rows.
        const int j = what - 4, h = half[r];
        const int g = lane >> 4, li = lane & 15;
        const int ncol = wn * WTN + j * 32 + (g & 1) * 16 + (li & 3) * 4;   // 4 columns, 8 bytes
        const int k0 = q * 16 + (g >> 1) * 8 + (li >> 2) + 4 * h;
        f.b[j][h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_short4_ptr)(sb + b_lds_off<2>(k0, ncol >> 3) + (ncol & 7) * 2));
      }
    } else {
      // fp32: lane half h reads the float4 at k = 8 q + 4 h .. + 3 of its A row; MFMA number e
      // consumes element e, i.e. k = 8 q + 4 h + e, and the B side reads that same k row.
      if (r < FM) {
        const int row = wm * WTM + r * 32 + (lane & 31);
        f.a[r] = *(const __attribute__((address_space(3))) f32x4 *)(sa + a_lds_off(row, q * 2 + (lane >> 5)));
      } else {
        const int e = (r - FM) / FN, j = (r - FM) % FN;
        const int k = q * 8 + (lane >> 5) * 4 + e;
        const int ncol = wn * WTN + j * 32 + (lane & 31);
        f.b[e][j] = *(const __attribute__((address_space(3))) float *)(sb + b_lds_off<4>(k, ncol >> 2) + (ncol & 3) * 4);
      }
    }
  };
  // The MFMAs are issued as volatile assembly with a memory clobber: that pins every one of them
  // between the LDS read (or load slot) before it and the one after it, exactly as written here.
  // (As a plain builtin the instruction selector is free to sink sixteen of them behind all the
  // reads and loads of the sub-step, which then execute with nothing to hide them.)  The compiler
  // still sees the register operands and waits for the LDS reads that produce them; what it can
  // no longer see is the result hazard of the matrix pipe, covered after the loop.
  auto mfma_op = [&](const Frags &f, auto nc) {          // MFMA slot n of a sub-step: tile (n / FN, n % FN)
    constexpr int n = decltype(nc)::value;
    constexpr int i = n / FN, j = n % FN;
    if constexpr (ES == 2) {
      union { short4_t h[2]; bf16x8 v; } u;
      u.h[0] = f.b[j][0];
      u.h[1] = f.b[j][1];
      asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3]"
                   :
                   : "v"(f.a[i]), "v"(u.v), "n"(16 * n), "n"(16 * n + 15)
                   : "memory", DMM_ACC_REGS);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float av = e == 0 ? f.a[i].x : e == 1 ? f.a[i].y : e == 2 ? f.a[i].z : f.a[i].w;
        asm volatile("v_mfma_f32_32x32x2_f32 a[%2:%3], %0, %1, a[%2:%3]"
                     :
                     : "v"(av), "v"(f.b[e][j]), "n"(16 * n), "n"(16 * n + 15)
                     : "memory", DMM_ACC_REGS);
      }
    }
  };
  // MFMA slot n of a sub-step and, in its shadow, load number j of the lead step, every lane taking
  // part (bf16, quiet iterations only): see the slots of sub_step
  auto mfma_dma = [&](const Frags &f, auto nc, auto jc, unsigned stage_base) {
    constexpr int n = decltype(nc)::value;
    constexpr int i = n / FN, jj = n % FN;
    constexpr int j = decltype(jc)::value;
    constexpr int IMM = j < LOADS ? j * (NW * 1024) : A_STAGE + (j - LOADS) * (NW * 1024);
    if constexpr (ES == 2) {
      union { short4_t h[2]; bf16x8 v; } u;
      u.h[0] = f.b[jj][0];
      u.h[1] = f.b[jj][1];
      if constexpr (COMP) {
        gptr &addr = j < LOADS ? ca[j < LOADS ? j : 0] : cbv[j < LOADS ? 0 : j - LOADS];
        asm volatile("s_add_u32 m0, %1, %2\n\tv_mfma_f32_32x32x16_bf16 a[%5:%6], %3, %4, a[%5:%6]\n\t"
                     "global_load_lds_dwordx4 %0, off"
                     :
                     : "v"(addr), "s"(stage_base), "n"(IMM), "v"(f.a[i]), "v"(u.v), "n"(16 * n), "n"(16 * n + 15)
                     : "memory", "scc", DMM_ACC_REGS);
        addr = add_low(addr, j < LOADS ? (unsigned)(BK * ES) : bstep[j < LOADS ? 0 : j - LOADS]);
      } else {
        const unsigned off = j < LOADS ? ld_a_off[j < LOADS ? j : 0] : ld_b_off[j < LOADS ? 0 : j - LOADS];
        const gptr base = j < LOADS ? ld_a : ld_b;
        asm volatile("s_add_u32 m0, %2, %3\n\tv_mfma_f32_32x32x16_bf16 a[%6:%7], %4, %5, a[%6:%7]\n\t"
                     "global_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(off), "s"(base), "s"(stage_base), "n"(IMM), "v"(f.a[i]), "v"(u.v), "n"(16 * n), "n"(16 * n + 15)
                     : "memory", "scc", DMM_ACC_REGS);
      }
    }
  };
  // One sub-step: its FM FN MFMA slots; after slot n either one of this wave's loads (when
  // slot % 4 == ROT) or the next LDS read of the following sub-step.  `first` = index of the
  // sub-step's first slot within the K step (0 or 16).
  auto sub_step = [&](auto first_tag, auto quiet_tag, const Frags &cur, Frags &nxt, lds_cptr rd_stage, int rd_q, int ld_stage) {
    constexpr int first = decltype(first_tag)::value;
    const unsigned ld_base = lds_base + ld_stage * STAGE + wave * 1024;
    // (unrolled by hand over the 16 slots so that slot numbers are compile-time constants)
    auto slot = [&](auto nc) {
      constexpr int n = decltype(nc)::value;
      constexpr int r = n - (n + NW - 1 - ROT) / NW;    // LDS reads issued in earlier slots of this sub-step
      constexpr int g = first + n;
      constexpr bool QUIET_SLOT = decltype(quiet_tag)::value;
      // A bf16 load slot of a quiet iteration is one statement: M0 write, MFMA, load.  The MFMA
      // is the wait state the M0 write needs before the LDS-DMA instruction reads it, so the slot
      // is three instructions, which fit the 32 cycles of the MFMA; with a separate wait state
      // they do not quite.
      constexpr bool FUSED = ES == 2 && QUIET_SLOT && g % NW == ROT;
      if constexpr (FUSED) mfma_dma(cur, nc, std::integral_constant<int, g / NW>{}, ld_base);
      else mfma_op(cur, nc);
      if constexpr (!COMP && g == NW + ((ROT + 1) % NW)) {   // a slot without a load: addresses of the next step
        ld_a_next = ld_a + BK * ES;
        ld_b_next = ld_b + ld_b_step;
      }
      if constexpr (FUSED) {
      } else if constexpr (g % NW == ROT) {
        dma(std::integral_constant<int, g / NW>{}, ld_base, quiet_tag);
      } else if (ES == 2) {
        read_op(rd_stage, rd_q, r, nxt);
      }
      if (ES == 4 && n == 0) {                           // fp32: all reads up front (64 MFMAs follow)
#pragma unroll
        for (int x = 0; x < READS; ++x) read_op(rd_stage, rd_q, x, nxt);
      }
      DMM_SCHED_BARRIER;
    };
    slot(std::integral_constant<int, 0>{});  slot(std::integral_constant<int, 1>{});
    slot(std::integral_constant<int, 2>{});  slot(std::integral_constant<int, 3>{});
    slot(std::integral_constant<int, 4>{});  slot(std::integral_constant<int, 5>{});
    slot(std::integral_constant<int, 6>{});  slot(std::integral_constant<int, 7>{});
    slot(std::integral_constant<int, 8>{});  slot(std::integral_constant<int, 9>{});
    slot(std::integral_constant<int, 10>{}); slot(std::integral_constant<int, 11>{});
    slot(std::integral_constant<int, 12>{}); slot(std::integral_constant<int, 13>{});
    slot(std::integral_constant<int, 14>{}); slot(std::integral_constant<int, 15>{});
  };

  // ---- the K loop ------------------------------------------------------------------------
  // Iteration s multiplies stage s % 4 while the loads of step s + 3 are issued into stage
  // (s + 3) % 4, which every wave finished reading before the barrier of iteration s - 1.
  int n = 0;                                             // K steps of the current item
  int issued = 0;                                        // steps whose loads the prologue has issued
  // Cursors to the item's first step, then its prologue: steps 0, 1, 2 in flight.
  auto begin_item = [&](const SegDev *first_seg) {        // first_seg: the record of the item's first segment, if at hand
    n = it.nsteps;
    lead_seg = 0;
    fix_bits = 0;
    pub_seg = pub_first = 0;
    if (!COMP && first_seg != nullptr) {
      open_lead_at(*first_seg, 0);
    } else {
      // the item's first step: segment and position (first_step lies inside the group's sequence)
      int first = 0;
      for (;;) {
        const int cnt = (seg_klen(lead_seg) + BK - 1) / BK;
        if (it.first_step < first + cnt) break;
        first += cnt;
        ++lead_seg;
      }
      open_lead((it.first_step - first) * BK);
    }
    issued = 0;
#pragma unroll
    for (int t = 0; t < NSTAGE - 1; ++t) {
      if (t < n) {
        prepare_lead(true, t);
        const unsigned base = lds_base + t * STAGE + wave * 1024;
        dma(std::integral_constant<int, 0>{}, base, std::false_type{}); dma(std::integral_constant<int, 1>{}, base, std::false_type{});
        dma(std::integral_constant<int, 2>{}, base, std::false_type{}); dma(std::integral_constant<int, 3>{}, base, std::false_type{});
        dma(std::integral_constant<int, 4>{}, base, std::false_type{}); dma(std::integral_constant<int, 5>{}, base, std::false_type{});
        dma(std::integral_constant<int, 6>{}, base, std::false_type{}); dma(std::integral_constant<int, 7>{}, base, std::false_type{});
        ++issued;
        if (t + 1 < n) advance_lead();
      } else {
        fix_bits <<= 1;                                  // keep the register in step: no such step, no repair
      }
    }
  };
  bool loads_on = false;
  int quiet = 0;                                         // iterations whose end is a plain advance of the lead
  int mid_plain = 0;                                     // the coming publication needs no repair and loads go on
  // After the lead step number `lead_idx` has been prepared by the general path: how many plain
  // advances follow it.  Their effect on the cursor is booked here, in advance.
  auto plan_quiet = [&](int lead_idx) {
    int q = 0;
    if (loads_on && (fix_bits & 7u) == 0u) {
      // inside the segment, short of its K tail and of the steps that may overrun a tile buffer
      const int keep = lead_tail && lead_unsafe == 0 ? 1 : lead_unsafe;
      q = lead_left - 1 - keep;
      const int r = n - 1 - lead_idx;                    // inside the item
      q = q < r ? q : r;
      q = q > 0 ? q : 0;
    }
    // (both are wave-uniform; saying so keeps them in scalar registers inside the loop)
    quiet = __builtin_amdgcn_readfirstlane(q);
    mid_plain = __builtin_amdgcn_readfirstlane(loads_on && (fix_bits & 4u) == 0u ? 1 : 0);
    lead_left -= quiet;
    lead_kpos += quiet * BK;
  };
  // The iteration exists in two copies.  The general one takes its loads' exec mask and its mid-
  // iteration wait from what the bookkeeping prepared; the quiet one, which runs `quiet` times after
  // it, knows that every lane loads and that nothing needs a repair, so its load slots are two
  // instructions shorter and its wait is a constant.  The quiet loop carries only s, the counter
  // and the two addresses; the general bookkeeping runs between such runs.
  // A quiet iteration can also be told its stage at compile time (`stage_tag` 0 .. 3 instead of -1):
  // every LDS address is then a register fixed per lane plus an immediate, and the vector adds
  // that otherwise rebuild the read addresses from the stage's base (each right in front of the
  // read that needs it, which waits for it) are gone, with the scalar arithmetic behind them.
  int s = 0;
  auto iteration = [&](auto quiet_tag, auto stage_tag) {
    constexpr bool QUIET = decltype(quiet_tag)::value;
    constexpr int FIXED = decltype(stage_tag)::value;
    const int stage = FIXED >= 0 ? FIXED : (s & (NSTAGE - 1));
    const int ld_stage = FIXED >= 0 ? ((FIXED + NSTAGE - 1) & (NSTAGE - 1)) : ((s + NSTAGE - 1) & (NSTAGE - 1));
    auto stage_ptr = [&](int st) -> lds_cptr {
      if constexpr (FIXED >= 0) return (st >= 2 ? lds3_hi : lds3) + (st & 1) * STAGE;
      else return lds3 + st * STAGE;
    };
    sub_step(std::integral_constant<int, 0>{}, quiet_tag, fr[0], fr[1], stage_ptr(stage), 1, ld_stage);
    // publish step s + 1: this wave's loads of it must have landed; steps s + 2 and (half of)
    // s + 3 may stay in flight (loads return in order)
    if (QUIET || __builtin_expect(mid_plain != 0, 1)) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS + LOADS) : "memory");
    } else {
      if (loads_on) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS + LOADS) : "memory");
      else if (s + 2 < n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (s + 1 < n) publish_fix(s + 1);
    }
    // Every wave has issued its reads of stage s; step s + 1 is complete.  The bare barrier
    // instruction, not __syncthreads: its fence would make every wave wait here for the LDS reads
    // it issued in the last slots (the operands of the coming sub-step's later MFMAs), with the
    // matrix pipe idle meanwhile.  The reads in flight at this point are reads of stage s, whose
    // next writer is a load of step s + 4, issued an iteration from now behind another barrier and
    // landing a memory latency later still; the compiler waits for each operand before its MFMA.
    __builtin_amdgcn_s_barrier();
    sub_step(std::integral_constant<int, FM * FN>{}, quiet_tag, fr[1], fr[0], stage_ptr((stage + 1) & (NSTAGE - 1)), 0, ld_stage);
    ++s;
  };

  // LOOP: the next item's record and that of its first segment are read while the current item
  // waits for its first loads, not when they are needed: a scalar load that misses the caches
  // takes a microsecond, and three of them in a row stood between two items.
  ItemDev ahead = it;
  SegDev ahead_seg = {};
  bool ahead_seg_valid = false;
  if (!LOOP || it.nsteps > 0) begin_item(nullptr);
  for (;;) {
    if constexpr (LOOP) {
      const int nxt = idx + stride;
      if (nxt < n_items) {
        ahead = items[nxt];
        ahead_seg_valid = ahead.nsteps > 0 && ahead.first_step == 0;
        if (ahead_seg_valid) ahead_seg = segs[ahead.seg_begin];
      }
    }
    if (!LOOP || it.nsteps > 0) {
      // publish step 0
      if constexpr (LOOP) {
        // (also the previous item's stores: the counter is shared and too narrow to tell them apart)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      } else {
        if (issued >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(4 * LOADS) : "memory");
        else if (issued == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
      publish_fix(0);
      __syncthreads();
#pragma unroll
      for (int r = 0; r < READS; ++r) read_op(lds3, 0, r, fr[0]);
      // here the lead cursor is at step min(3, n - 1), which has been issued iff n <= 3
      loads_on = n > NSTAGE - 1;                         // a step s + 3 exists for s = 0
      prepare_lead(loads_on, NSTAGE - 1);
      plan_quiet(NSTAGE - 1);
      s = 0;
      auto quiet_iteration = [&](auto stage_tag) {
        if constexpr (!COMP) {
          ld_a = ld_a_next;
          ld_b = ld_b_next;
        }
        iteration(std::true_type{}, stage_tag);
      };
      for (;;) {
        iteration(std::false_type{}, std::integral_constant<int, -1>{});
#pragma clang loop unroll(disable)
        while (quiet != 0) {
          if ((s & (NSTAGE - 1)) == 0 && quiet >= NSTAGE) {
            // a run of four from stage 0 on: the copies with their stages built in
#pragma clang loop unroll(disable)
            do {
              quiet -= NSTAGE;
              quiet_iteration(std::integral_constant<int, 0>{});
              quiet_iteration(std::integral_constant<int, 1>{});
              quiet_iteration(std::integral_constant<int, 2>{});
              quiet_iteration(std::integral_constant<int, 3>{});
            } while (quiet >= NSTAGE);
            continue;
          }
          --quiet;
          quiet_iteration(std::integral_constant<int, -1>{});
        }
        if (s >= n) break;
        loads_on = s - 1 + NSTAGE < n;           // step s + 3 exists (s is the coming iteration)
        if (loads_on) advance_lead();
        prepare_lead(loads_on, (s - 1) & (NSTAGE - 1));   // it goes to the stage the last iteration consumed
        plan_quiet(s - 1 + NSTAGE);
      }
      // nothing may land in LDS after the workgroup has gone; and the last MFMA results must have left
      // the matrix pipe before other instructions read the accumulators (18 wait states and more)
      asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 7" ::: "memory");
    }
    if constexpr (!LOOP) {
      return;
    } else {
      const ItemDev done = it;
      const int nxt = idx + stride;
      // every wave is out of the K loop (all its LDS reads have been issued long since): the stages
      // may be filled again
      __builtin_amdgcn_s_barrier();
      if (nxt < n_items) {
        it = ahead;
        idx = nxt;
        set_rows();
        if (it.nsteps > 0) begin_item(ahead_seg_valid ? &ahead_seg : nullptr);
      }
      store_macro_tile<FUSE>(done, red, wm, wn, lane);
      if (nxt >= n_items) return;
      // (the stores above read the accumulators as they issue; a few idle cycles for good measure)
      asm volatile("s_nop 7" ::: "memory");
      acc_clear<ES>();
    }
  }
}

// The C stores of one macro-tile: lane holds column (lane & 31), rows 8 (r / 4) + 4 (lane / 32) + r % 4 of
// each 32 x 32 tile.  Addresses are the item's base plus a 32-bit byte offset (the host rejects C
// pitches of 2^24 bytes and more): one add per row, the four column blocks of a row through the
// immediate offset.  A full 256 x 256 item stores without predicates.  A bf16 destination receives
// the fp32 sum rounded to nearest even, one 2-byte store per element.
// FUSE: the instantiation that can add other replicas' partial sums (fused replica sum).
template <bool FUSE>
__device__ __forceinline__ void store_macro_tile(const ItemDev &it, const RedSrc *__restrict__ red, int wm, int wn, int lane) {
  // (the lane number is hidden from the optimiser here: inside the item loop it would otherwise
  // move everything below that depends on the lane alone, the 64 row numbers of the predicates
  // among it, in front of the loop and keep it in registers all the way through the K loops)
  asm volatile("" : "+v"(lane));
  const __attribute__((address_space(1))) char *cbytes = (const __attribute__((address_space(1))) char *)it.c;
  const int row0 = wm * WTM + 4 * (lane >> 5);
  const int col0 = wn * WTN + (lane & 31);
  const bool wide = it.c_es == 4;
  const unsigned pitch = (unsigned)it.ldc * (unsigned)it.c_es;
  const unsigned voff = (unsigned)row0 * pitch + (unsigned)col0 * (unsigned)it.c_es;
  auto store_all = [&](auto full_tag, auto wide_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    constexpr bool wide = decltype(wide_tag)::value;       // fp32 destination (else bf16)
    // the row offset is carried from row to row (rows go +1, +1, +1, +5) and hidden from the
    // optimiser after every step: it would otherwise work out all 64 offsets ahead of the stores
    unsigned o = voff;
    const unsigned pitch5 = 5u * pitch;
    static_for<FM * 16>([&](auto xc) {
      constexpr int i = decltype(xc)::value / 16, r = decltype(xc)::value % 16;
      constexpr int dr = i * 32 + 8 * (r >> 2) + (r & 3);
      asm volatile("" : "+v"(o));
      if constexpr (FULL && wide) {
        static_assert(FN == 4, "acc_store_row stores four column blocks");
        acc_store_row<16 * i * FN + r>(o, cbytes);
      } else if (FULL || row0 + dr < it.m_ext) {
        static_for<FN>([&](auto jc) {
          constexpr int j = decltype(jc)::value;
          constexpr int REG = 16 * (i * FN + j) + r;
          if (FULL || col0 + j * 32 < it.n_ext) {
            if constexpr (wide) {
              // data straight from the accumulator file, one offset register
              acc_store<REG, j * 128>(o, cbytes);
            } else {
              __builtin_nontemporal_store(__builtin_bit_cast(unsigned short, (__bf16)acc_read<REG>()),
                                          (gushort_ptr)(cbytes + o + j * 64));
            }
          }
        });
      }
      o += (r & 3) == 3 ? pitch5 : pitch;
    });
  };
  // Fused replica sum (fp32 C only): the macro-tile of the origin replica adds the other replicas'
  // partial sums of its region to its own, ((own + p_1) + p_2) ..., the order and precision of the
  // replica-sum kernel, and then stores like any other macro-tile.  The sums go back into the
  // accumulator file, so that this phase has nothing but loads in flight: with loads and stores
  // mixed, the one counter that tracks both says nothing about which of them has returned, and
  // every batch of loads would have to wait for the whole queue to drain.  Eight rows of a 32 x 32
  // tile per batch (32 values per lane), three batches in flight.
  auto add_partials = [&](auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    constexpr int RB = 8;                                  // accumulator registers (rows) per batch
    constexpr int NB = FM * (16 / RB);                     // batches per macro-tile and source
    constexpr int DEPTH = 4;                               // ring of batches: DEPTH - 1 in flight
    static_assert(NB % DEPTH == 0 && NB >= DEPTH, "a batch's place in the ring must not depend on the source");
    float v[DEPTH][RB][FN];
    // the loads of batch b of the partial sum `src` (the macro-tile's region of another replica)
    auto issue = [&](auto bc, const RedSrc &src) {
      constexpr int b = decltype(bc)::value, i = b / (16 / RB), rb = (b % (16 / RB)) * RB, slot = b % DEPTH;
      const __attribute__((address_space(1))) char *pbytes = (const __attribute__((address_space(1))) char *)src.p;
      const unsigned ppitch = (unsigned)src.ld * 4u;
      const unsigned poff = (unsigned)row0 * ppitch + (unsigned)col0 * 4u;
      static_for<RB * FN>([&](auto yc) {
        constexpr int r = decltype(yc)::value / FN, j = decltype(yc)::value % FN;
        constexpr int dr = i * 32 + 8 * ((rb + r) >> 2) + ((rb + r) & 3);
        v[slot][r][j] = 0.f;
        if (FULL || (row0 + dr < it.m_ext && col0 + j * 32 < it.n_ext))
          v[slot][r][j] = __builtin_nontemporal_load(
              (const __attribute__((address_space(1))) float *)(pbytes + (poff + (unsigned)dr * ppitch) + j * 128));
      });
    };
    // ((own + p_1) + p_2) ...: one pass over the macro-tile per source, the sources' passes back to
    // back in one stream of batches (the last batches of a pass already load the next source's first)
    RedSrc src = red[it.red_first];
    static_for<DEPTH - 1>([&](auto bc) { issue(bc, src); });
    for (int q = 0; q < it.red_count; ++q) {
      const bool more = q + 1 < it.red_count;
      const RedSrc next = more ? red[it.red_first + q + 1] : src;
      static_for<NB>([&](auto bc) {
        constexpr int b = decltype(bc)::value, i = b / (16 / RB), rb = (b % (16 / RB)) * RB, slot = b % DEPTH;
        if constexpr (b + DEPTH - 1 < NB) {
          issue(std::integral_constant<int, b + DEPTH - 1>{}, src);
        } else {
          if (more) issue(std::integral_constant<int, b + DEPTH - 1 - NB>{}, next);
        }
        static_for<RB * FN>([&](auto yc) {
          constexpr int r = decltype(yc)::value / FN, j = decltype(yc)::value % FN;
          constexpr int REG = 16 * (i * FN + j) + rb + r;
          acc_write<REG>(acc_read<REG>() + v[slot][r][j]);
        });
      });
      src = next;
    }
  };
  const bool full = it.m_ext == BM && it.n_ext == BN;
  if constexpr (FUSE) {
    if (it.red_count > 0) {
      if (full) add_partials(std::true_type{});
      else add_partials(std::false_type{});
    }
  }
  if (wide) {
    if (full) store_all(std::true_type{}, std::true_type{});
    else store_all(std::false_type{}, std::true_type{});
  } else {
    if (full) store_all(std::true_type{}, std::false_type{});
    else store_all(std::false_type{}, std::false_type{});
  }
}

// The launch: one workgroup per CU (or fewer), workgroup w taking items w, w + gridDim.x, ... of the
// `n_items` of the list, which the planner has ordered so that this keeps the macro-tiles of one
// block on one XCD.  FUSE: a kernel of its own, so that the plain one keeps its size and its
// register allocation.
template <int ES, bool FUSE = false>
__global__ __launch_bounds__(NT) void grouped_gemm_kernel(const ItemDev *__restrict__ items,
                                                          const SegDev *__restrict__ segs,
                                                          const RedSrc *__restrict__ red, int n_items) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int idx = blockIdx.x;
  if (idx >= n_items) return;
  const ItemDev it = items[idx];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  acc_clear<ES>();
  // one instantiation per wave: the four waves of the CU issue their loads in different slots
  const int stride = (int)gridDim.x;
  if (wave == 0) run_item<ES, 0, false, true, FUSE>(it, segs, lds, CompCtx{}, items, idx, stride, n_items, red);
  else if (wave == 1) run_item<ES, 1, false, true, FUSE>(it, segs, lds, CompCtx{}, items, idx, stride, n_items, red);
  else if (wave == 2) run_item<ES, 2, false, true, FUSE>(it, segs, lds, CompCtx{}, items, idx, stride, n_items, red);
  else run_item<ES, 3, false, true, FUSE>(it, segs, lds, CompCtx{}, items, idx, stride, n_items, red);
}

// The same multiplication for merged macro-tiles.  The item's descriptors (segment lengths, one A
// slice per row piece and segment, one B slice per segment and column piece) are first copied
// into LDS behind the stages, where a segment switch reads them without touching the counter
// that tracks the loads in flight.  The epilogue writes through a table of row addresses (one
// per row and column piece, built in the stage area once the K loop is done), since the rows
// and columns of the macro-tile end up in different C tiles.
template <int ES>
__global__ __launch_bounds__(NT) void grouped_gemm_comp_kernel(const CompItemDev *__restrict__ items,
                                                               const PieceDev *__restrict__ a_pieces,
                                                               const PieceDev *__restrict__ b_pieces,
                                                               const PieceDev *__restrict__ c_pieces,
                                                               const int32_t *__restrict__ klen) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const CompItemDev *ci = items + blockIdx.x;
  const int R = ci->R, Q = ci->Q, S = ci->S;
  const int m_ext = ci->m_ext, n_ext = ci->n_ext;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  int32_t *geo = (int32_t *)(lds + LDS_BYTES);            // piece boundaries, where lanes can index them
  PieceDev *cd = (PieceDev *)(geo + 32);                  // [R][Q] C slices
  int32_t *klen_s = geo + DESC_GEO / 4;
  PieceDev *ad = (PieceDev *)(klen_s + ((S + 3) & ~3));
  PieceDev *bd = ad + S * R;
  for (int x = threadIdx.x; x < R * Q; x += NT) cd[x] = c_pieces[ci->c_first + (x / Q) * ci->c_stride + x % Q];
  for (int x = threadIdx.x; x < S; x += NT) klen_s[x] = klen[ci->k_first + x];
  for (int x = threadIdx.x; x < S * R; x += NT) ad[x] = a_pieces[ci->a_first + (x % R) * ci->a_stride + x / R];
  for (int x = threadIdx.x; x < S * Q; x += NT) bd[x] = b_pieces[ci->b_first + (x / Q) * ci->b_stride + x % Q];
  if (threadIdx.x <= PMAX) {
    geo[threadIdx.x] = ci->rb[threadIdx.x];
    geo[PMAX + 1 + threadIdx.x] = ci->cb[threadIdx.x];
  }
  __syncthreads();

  acc_clear<ES>();

  if (ci->nsteps > 0) {
    ItemDev it;
    it.c = nullptr;
    it.ldc = 0;
    it.seg_begin = 0;
    it.nsteps = ci->nsteps;
    it.m_off = it.n_off = 0;
    it.m_ext = m_ext;
    it.n_ext = n_ext;
    it.first_step = ci->first_step;
    it.c_es = ci->c_es;
    it.red_first = it.red_count = 0;
    CompCtx cx;
    cx.klen = klen_s;
    cx.ad = ad;
    cx.bd = bd;
    cx.rb = geo;
    cx.cb = geo + PMAX + 1;
    cx.R = R;
    cx.Q = Q;
    if (wave == 0) run_item<ES, 0, true>(it, nullptr, lds, cx);
    else if (wave == 1) run_item<ES, 1, true>(it, nullptr, lds, cx);
    else if (wave == 2) run_item<ES, 2, true>(it, nullptr, lds, cx);
    else run_item<ES, 3, true>(it, nullptr, lds, cx);
  }

  // ---- epilogue ------------------------------------------------------------------------------
  if (ci->scratch) {
    // a run of a macro-tile cut along K: partial sums to the scratch tile, to be added up later
    float *out = ci->scratch;
    const int row0 = wm * WTM + 4 * (lane >> 5);
    const int col0 = wn * WTN + (lane & 31);
    static_for<FM * 16>([&](auto xc) {
      constexpr int i = decltype(xc)::value / 16, r = decltype(xc)::value % 16;
      const int row = row0 + i * 32 + 8 * (r >> 2) + (r & 3);
      if (row < m_ext) {
        static_for<FN>([&](auto jc) {
          constexpr int j = decltype(jc)::value;
          if (col0 + j * 32 < n_ext)
            __builtin_nontemporal_store(acc_read<16 * (i * FN + j) + r>(), out + row * BN + col0 + j * 32);
        });
      }
    });
    return;
  }
  __syncthreads();                                        // every wave is out of the K loop: the stages are free
  uint64_t *rowbase = (uint64_t *)lds;                    // [256][PMAX]: address of (row, first column of piece q)
  {
    const int row = threadIdx.x;
    if (row < m_ext) {
      int p = 0, base = geo[0];
      for (int x = 1; x < R; ++x)
        if (geo[x] <= row) { p = x; base = geo[x]; }
      for (int q = 0; q < Q; ++q) {
        const PieceDev d = cd[p * Q + q];
        rowbase[row * PMAX + q] = (uint64_t)(uintptr_t)d.ptr + (uint64_t)(row - base) * d.pitch;
      }
    }
  }
  __syncthreads();
  const int ces = ci->c_es;
  const bool wide = ces == 4;
  const int row0 = wm * WTM + 4 * (lane >> 5);
  const int col0 = wn * WTN + (lane & 31);
  int qj[FN];
  unsigned lcol[FN];                                      // byte column inside the piece
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int col = col0 + j * 32;
    int q = 0, base = geo[PMAX + 1];
    for (int x = 1; x < Q; ++x)
      if (geo[PMAX + 1 + x] <= col) { q = x; base = geo[PMAX + 1 + x]; }
    qj[j] = q;
    lcol[j] = (unsigned)(col - base) * (unsigned)ces;
  }
  // When the four columns of every lane of the wave lie in one column piece (pieces of 128 columns
  // and more, at multiples of 128), a row takes one table read and its four stores differ by a
  // constant; otherwise every store reads its own row address.
  const bool one_piece = __builtin_amdgcn_ballot_w64(qj[0] != qj[FN - 1]) == 0;
  auto store_all = [&](auto one_tag) {
    constexpr bool ONE = decltype(one_tag)::value;
    static_for<FM * 16>([&](auto xc) {
      constexpr int i = decltype(xc)::value / 16, r = decltype(xc)::value % 16;
      const int row = row0 + i * 32 + 8 * (r >> 2) + (r & 3);
      if (row < m_ext) {
        uint64_t a0 = 0;
        if constexpr (ONE) a0 = rowbase[row * PMAX + qj[0]] + lcol[0];
        static_for<FN>([&](auto jc) {
          constexpr int j = decltype(jc)::value;
          if (col0 + j * 32 < n_ext) {
            uint64_t a;
            if constexpr (ONE) a = a0;
            else a = rowbase[row * PMAX + qj[j]] + lcol[j];
            const float v = acc_read<16 * (i * FN + j) + r>();
            if (wide)
              __builtin_nontemporal_store(v, (gfloat_ptr)(uintptr_t)a + (ONE ? j * 32 : 0));
            else
              __builtin_nontemporal_store(__builtin_bit_cast(unsigned short, (__bf16)v),
                                          (gushort_ptr)(uintptr_t)a + (ONE ? j * 32 : 0));
          }
        });
      }
    });
  };
  if (one_piece) store_all(std::true_type{});
  else store_all(std::false_type{});
}

}  // namespace dmm
