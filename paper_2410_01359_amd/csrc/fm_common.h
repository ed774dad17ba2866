// Shared device-side definitions for the gfx950 FlashMask kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fm_kernels.h"

namespace fm {

typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

#define FM_LDS __attribute__((address_space(3)))

#ifndef FM_FAST_LIST
#define FM_FAST_LIST 1
#endif
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Rows of the preprocessing table (Section 4.2), per batch row: [8][T_c].
enum { LTS_MAX = 0, LTS_MIN, LTE_MAX, LTE_MIN, UTS_MAX, UTS_MIN, UTE_MAX, UTE_MIN };

// Tile classes (Equation 4); same encoding as FM_TILE_* in flashmask.h.
enum { T_UNMASKED = 0, T_PARTIAL = 1, T_FULLY = 2, T_NEED_LT = 16, T_NEED_UT = 32 };

struct MinMax8 {
  int v[8];
};

// Equation 4 for the row range [r0, r1) against one key block's min/max values.
__device__ __forceinline__ int classify_tile(int r0, int r1, const MinMax8& t) {
  const bool full_lt = (r0 >= t.v[LTS_MAX]) && (r1 <= t.v[LTE_MIN]);
  const bool full_ut = (r0 >= t.v[UTS_MAX]) && (r1 <= t.v[UTE_MIN]);
  if (full_lt || full_ut) return T_FULLY;
  const bool part_lt = (r1 > t.v[LTS_MIN]) && (r0 < t.v[LTE_MAX]);
  const bool part_ut = (r1 > t.v[UTS_MIN]) && (r0 < t.v[UTE_MAX]);
  if (part_lt || part_ut) return T_PARTIAL | (part_lt ? T_NEED_LT : 0) | (part_ut ? T_NEED_UT : 0);
  return T_UNMASKED;
}

__device__ __forceinline__ MinMax8 load_minmax(const int* __restrict__ table, int t_c, int j) {
  MinMax8 t;
#pragma unroll
  for (int a = 0; a < 8; ++a) t.v[a] = table[a * t_c + j];
  return t;
}

// D(32x32) += A(32x16) * B(16x32), bf16 inputs, fp32 accumulate.
// Lane l holds A[m = l%32][k = 8*(l/32) + t], B[k = 8*(l/32) + t][n = l%32], t = 0..7,
// and D[m = 8*(r/4) + 4*(l/32) + r%4][n = l%32] in register r = 0..15.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// The same product accumulated in place in accumulation registers (AGPRs).  For accumulators that
// live through a whole tile loop and are touched by nothing but their own MFMAs: the compiler picks
// one register file for all of a kernel's MFMA results, and keeping these in the vector file leaves the
// loop's vector work half the registers.  The compiler does not look into the asm, so the wait states
// an MFMA needs are the caller's business:
//  - a vector instruction that writes an A/B source must be two wait states ahead of the MFMA: pass
//    fresh = true (a constant once the caller's step loop is unrolled) for the first MFMA that reads
//    a source just produced by vector instructions (it puts an idle instruction of two cycles in
//    front); sources loaded from LDS only need the wait the compiler already inserts for the asm's
//    operands;
//  - in-place accumulation with one opcode needs none between dependent MFMAs;
//  - a reader of `acc` other than this function must be kept clear of the last MFMA (mfma_acc_drain).
__device__ __forceinline__ void mfma32_acc(f32x16& acc, bf16x8 a, bf16x8 b, bool fresh) {
  const i32x4 ai = __builtin_bit_cast(i32x4, a), bi = __builtin_bit_cast(i32x4, b);
  if (fresh)
    asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(ai), "v"(bi));
  else
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(ai), "v"(bi));
}
// After the last mfma32_acc of a loop nest, in the same block of straight-line code (volatile asm
// statements keep their order): 48 idle cycles, the depth of the matrix pipe for this instruction
// (8 passes of 4 cycles) plus the margin the ISA asks for before another instruction reads the result.
// Code that reads the accumulators must sit behind the loop's exit, where the compiler cannot move it
// ahead of this.
__device__ __forceinline__ void mfma_acc_drain() { asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15"); }

__device__ __forceinline__ bf16x4 lds_read_tr16(const char* lds_generic) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((FM_LDS bf16x4*)lds_generic);
}

// The same reads from an LDS byte address held in a register.
__device__ __forceinline__ bf16x8 lds_read_row16(unsigned addr) { return *(FM_LDS const bf16x8*)(size_t)addr; }
__device__ __forceinline__ bf16x4 lds_read_tr16_at(unsigned addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((FM_LDS bf16x4*)(size_t)addr);
}

__device__ __forceinline__ bf16x8 cat4(bf16x4 lo, bf16x4 hi) {
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Exchange with the lane 32 away: returns the partner's value.
__device__ __forceinline__ float partner32(float x) {
  int xi = __builtin_bit_cast(int, x);
  // permlane32_swap(a, b): r[0] = {a.lo, b.lo}, r[1] = {a.hi, b.hi} (lo/hi = lanes 0-31 / 32-63)
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  // lanes 0-31: r[1] holds x of lanes 32-63; lanes 32-63: r[0] holds x of lanes 0-31
  int other = (threadIdx.x & 32) ? r[0] : r[1];
  return __builtin_bit_cast(float, other);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ u32x4 ldg16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }

// LDS layout of a [rows][D] bf16 tile, shared by all tile loops.
//
// LDS serves 64 banks x 4 B per clock; a 128-bit read is issued 16 lanes per
// clock and the 64-bit transpose read 32 lanes per clock.  A tile is read in
// two ways: as MFMA operand rows (16 consecutive rows, one 16-byte chunk each
// per clock) and through the transpose read (4 consecutive rows x 64 bytes per
// clock).  Rows are stored unpadded (the direct global->LDS copy writes 1 KB
// contiguously per wave) and the 16-byte chunk index of a row is XORed with a
// bit permutation of the row's low four bits, chosen so that 16 consecutive
// rows hit 16 different 16-byte slots of the 256-byte bank line (first
// pattern) and 4 consecutive rows hit 4 different 64-byte groups (second
// pattern): both reads are conflict-free.
// off(row + 16*m, col) == off(row, col) + 16*m*RS, so callers precompute the
// lane-dependent part once.
template <int D>
struct TileLayout {
  static constexpr int RS = D * 2;       // bytes per row
  static constexpr int CPR = D / 8;      // 16-byte chunks per row
  static __device__ __forceinline__ int swz(int row) {
    const int r = row & 15;
    if (D == 128) return ((r & 3) << 2) | (r >> 2);   // 16 chunks per row, one row per bank line
    const int a = r >> 1;                               // D == 64: two rows per bank line
    return ((a & 1) << 2) | (a >> 1);
  }
  static __device__ __forceinline__ int off(int row, int byte_col) {
    return row * RS + ((((byte_col >> 4) ^ swz(row)) << 4) | (byte_col & 15));
  }
  // off(row, col0 + colc) from off(row, col0), for a constant colc that is a
  // multiple of 16 and shares no set bit with col0.
  static __device__ __forceinline__ int add_col(int base, int colc) { return base ^ colc; }
};

// Asynchronous global->LDS copy of a [64][D] bf16 tile (global row stride D)
// into TileLayout<D> order by a 4-wave workgroup.  Wave w copies rows
// 16w..16w+15, a contiguous block on both sides, with NINST instructions of
// 64 x 16 B = 1 KB each straight into LDS (no staging registers); the swizzle is
// applied on the global-address side.  The LDS destination of such an
// instruction is M0 + immediate offset + 16 * lane and the same immediate is
// added to the global address, so one M0 value (async_window) serves all of a
// wave's instructions for a tile: rewriting M0 costs the issuing wave about as
// much as the copy itself.  CopyLanes holds the per-lane source byte offset
// of each instruction (relative to the wave's row block); the swizzle repeats
// every 16 rows, so it does not depend on the wave.
template <int D>
struct CopyLanes {
  using L = TileLayout<D>;
  static constexpr int RPI = 64 / L::CPR;     // rows per instruction
  static constexpr int NINST = 16 / RPI;      // instructions per wave and tile
  unsigned v[NINST];
  // grs: bytes between consecutive rows of the global tensor (TileLayout::RS when it is
  // contiguous).  Instruction s carries the immediate s * 1024 on both sides, so what its rows
  // are really apart in global memory beyond that goes into the lane offset.
  __device__ __forceinline__ void init(int lane, int grs = L::RS) {
#pragma unroll
    for (int s = 0; s < NINST; ++s) {
      const int row = lane / L::CPR;          // row within the instruction's 1 KB
      v[s] = (s * RPI + row) * grs - s * 1024 + (((lane % L::CPR) ^ L::swz(s * RPI + row)) << 4);
    }
  }
};
// One wave-wide asynchronous copy: every active lane moves 16 bytes from its own
// global address to LDS address lds_addr + 16 * lane (lds_addr wave-uniform).
// Issued through inline assembly on purpose: the compiler treats the builtin
// form as an LDS store that any later LDS read may alias and drains ALL
// outstanding copies (s_waitcnt vmcnt(0)) in front of the next LDS read, which
// would serialise the copy of the next tiles with the math of this one.  Here
// the waiting is explicit: async_wait<N>() before the barrier that publishes a
// tile.  (Copies complete in issue order; counting extra outstanding vector
// memory operations only ever makes the compiler's own vmcnt waits stricter.)
__device__ __forceinline__ void async_copy16(const void* gsrc, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(gsrc)
               : "memory", "m0");
}
// Copy by lanes 0..7 only (128 bytes to lds_addr), whatever the wave's execution mask is;
// the mask is narrowed and restored inside the statement, so no branch is needed around it.
__device__ __forceinline__ void async_copy16_lanes8(const void* gsrc, unsigned lds_addr) {
  unsigned long long saved;
  asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 0xff\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
               "global_load_lds_dwordx4 %2, off\n\ts_mov_b64 exec, %0"
               : "=&s"(saved)
               : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(gsrc)
               : "memory", "m0");
}
__device__ __forceinline__ unsigned lds_address(const void* lds_generic) {
  return (unsigned)(size_t)((FM_LDS const char*)lds_generic);
}
// Wait until at most N of this wave's vector-memory operations (async copies
// included) are still in flight.
template <int N>
__device__ __forceinline__ void async_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Workgroup barrier without the memory fence of __syncthreads(): the caller has already waited for
// the async copies that must be visible.  Every LDS read of the buffer about to be overwritten must
// have returned before the wave arrives (another wave's copy may refill it right after): the wait for
// this wave's outstanding LDS reads is part of the barrier, so the invariant holds by construction and
// not by where the compiler happened to place the instructions that consume the reads (the copies are
// issued from inline assembly, so the compiler does not see them as LDS writes it must order against).
// It costs nothing where the reads have been consumed already.
__device__ __forceinline__ void barrier_nofence() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// The same barrier without the wait, for a point in the middle of an instruction stream that keeps LDS
// reads in flight across it on purpose: the caller must know that none of those reads targets the buffer
// that is refilled after the barrier.
__device__ __forceinline__ void barrier_reads_in_flight() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Set the LDS window (M0) of the async_copy16_window copies that follow.  M0 is
// not otherwise used by these kernels; the window stays valid until the next
// async_window / async_copy16* call.
__device__ __forceinline__ void async_window(unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" : : "s"(__builtin_amdgcn_readfirstlane(lds_addr)) : "memory", "m0");
}
// One wave-wide copy inside the current window: lane l moves 16 bytes from
// uniform_base + lane_byte_off + IMM to LDS address M0 + IMM + 16 l.
template <int IMM>
__device__ __forceinline__ void async_copy16_window(const void* uniform_base, unsigned lane_byte_off) {
  static_assert(IMM >= 0 && IMM < 4096, "immediate offset range");
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(lane_byte_off), "s"(uniform_base), "n"(IMM) : "memory");
}
// Instruction S (of CopyLanes<D>::NINST) of a wave's part of a tile copy.
template <int D, int S>
__device__ __forceinline__ void tile_copy_inst(const void* wave_src, const CopyLanes<D>& cl) {
  async_copy16_window<S * 1024>(wave_src, cl.v[S]);
}
// A wave's whole part of a [64][D] tile copy: tile_src / lds_tile are the tile's first row.
template <int D>
__device__ __forceinline__ void tile_load_async(const __bf16* tile_src, const CopyLanes<D>& cl, const char* lds_tile,
                                                int wave, int grs = TileLayout<D>::RS) {
  const char* wave_src = (const char*)tile_src + (size_t)(wave * 16) * grs;
  async_window(lds_address(lds_tile) + wave * 16 * TileLayout<D>::RS);
  tile_copy_inst<D, 0>(wave_src, cl);
  tile_copy_inst<D, 1>(wave_src, cl);
  if (CopyLanes<D>::NINST == 4) {
    tile_copy_inst<D, 2>(wave_src, cl);
    tile_copy_inst<D, 3>(wave_src, cl);
  }
}

// The same tile copy for a tile whose last rows lie past the end of the tensor (sequence length
// not a multiple of the tile): every lane clamps its source row to the last real one, so all
// reads stay in bounds; what lands in the extra rows is finite and the mask keeps it out of the
// result.  tensor_bh is row 0 of the (batch, head) slice, row0 the tile's first row.
template <int D>
__device__ __forceinline__ void tile_load_async_clamped(const __bf16* tensor_bh, int row0, int n_real,
                                                        const char* lds_tile, int wave, int lane,
                                                        int grs = TileLayout<D>::RS) {
  using L = TileLayout<D>;
  constexpr int RPI = 64 / L::CPR, NINST = 16 / RPI;
#pragma unroll
  for (int s = 0; s < NINST; ++s) {
    const int row = wave * 16 + s * RPI + lane / L::CPR;
    const int grow = min(row0 + row, n_real - 1);
    const char* src = (const char*)tensor_bh + (size_t)grow * grs + (((lane % L::CPR) ^ L::swz(row)) << 4);
    async_copy16(src, lds_address(lds_tile) + wave * 16 * L::RS + s * 1024);
  }
}

// Result stores.  The tile loops end with a 32-row x D result per wave held rows-on-lanes: lane (c, g)
// (c = lane % 32, g = lane / 32) has, of row c, the four consecutive elements 32 db + 8 q + 4 g .. +3 for
// every (db, q).  Stored from there, one instruction would touch 32 rows with 16 bytes each.  Each wave
// instead passes its block through a private piece of LDS (rows RS bytes apart: D bf16 plus 16 bytes, so
// that the 8-byte deposits of 32 rows spread over all banks) and writes whole rows, 16 bytes per lane.
// No barrier: a wave reads only what it wrote itself, and LDS serves a wave's accesses in order.
template <int D>
struct RowStage {
  static constexpr int RS = 2 * D + 16;
  static constexpr int BYTES = 32 * RS;   // per wave and result
  static constexpr int LPR = D / 8;       // lanes per row when every lane moves 16 bytes
  static constexpr int RPI = 64 / LPR;    // rows per store instruction
  static __device__ __forceinline__ void put(char* stage, int c, int g, int db, int q, bf16x4 v) {
    *(bf16x4*)(stage + c * RS + (32 * db + 8 * q + 4 * g) * 2) = v;
  }
  // rows [0, n_rows) of the block go to row0, row0 + row_stride, ... (elements)
  static __device__ __forceinline__ void flush(const char* stage, __bf16* row0, int row_stride, int lane, int n_rows) {
#pragma unroll
    for (int i = 0; i < 32 / RPI; ++i) {
      const int r = i * RPI + lane / LPR, col = (lane % LPR) * 16;
      const u32x4 v = *(const u32x4*)(stage + r * RS + col);
      if (r < n_rows) *(u32x4*)((char*)(row0 + (size_t)r * row_stride) + col) = v;
    }
  }
};

// Where a (batch, head) slice of a tensor starts and how far its rows are apart, in elements:
// taken from the stride record in the general instantiations, compile-time otherwise.
template <int D, bool GEN>
__device__ __forceinline__ const __bf16* slice_ptr(const void* base, const FmStride& st, int b, int h, int heads,
                                                   int n_rows) {
  if (GEN) return (const __bf16*)base + (size_t)b * st.b + (size_t)h * st.h;
  return (const __bf16*)base + (size_t)(b * heads + h) * n_rows * D;
}
template <int D, bool GEN>
__device__ __forceinline__ int row_stride(const FmStride& st) {
  return GEN ? (int)st.n : D;
}

// Force a value that was fetched with an ordinary global load to be complete
// (and known complete to the compiler) at this point.  The tile loops issue
// their async copies behind the compiler's back; if the first use of such a
// value sat inside a loop, the compiler's own "s_waitcnt vmcnt(n)" there --
// counted without the async copies -- would drain the copies of the tiles
// being prefetched on every iteration.
template <class T>
__device__ __forceinline__ void settle(T& x) {
  asm volatile("" : "+v"(x));
}

// Make a loop-invariant value opaque so that expressions derived from it are
// recomputed (one VALU op) instead of being kept live in registers.
__device__ __forceinline__ int opaque(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

// Unit queues.  Workgroup x draws a ticket from queue x % FM_QUEUES (ticket t of queue g is slot
// t * FM_QUEUES + g of the slot records); when that queue is used up it draws from the queue that
// has most left, and when all are used up it gets nothing.  Returns the slot record, wave-uniform,
// with unit = -1 for "nothing".  One barrier; lds_word is a scratch word in LDS.  The counters sit
// behind the slot records and are zeroed by the queue-building kernel of every call.
// The slot drawn by the calling thread (one thread per workgroup calls this), -1 for "nothing left".
__device__ __forceinline__ int queue_draw(int* order, int slots) {
  int* counters = order + 4 * (size_t)slots;
  const int per_queue = slots / FM_QUEUES;
  int q = blockIdx.x % FM_QUEUES;
  int t = atomicAdd(counters + q, 1);
  for (int attempt = 0; t >= per_queue && attempt < FM_QUEUES; ++attempt) {
    int best = -1, best_left = 0;
    for (int g = 0; g < FM_QUEUES; ++g) {
      const int left = per_queue - __hip_atomic_load(counters + g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (left > best_left) {
        best_left = left;
        best = g;
      }
    }
    if (best < 0) break;
    q = best;
    t = atomicAdd(counters + q, 1);
  }
  return t < per_queue ? t * FM_QUEUES + q : -1;
}
__device__ __forceinline__ i32x4 queue_take(int* order, int slots, int* lds_word) {
  if (threadIdx.x == 0) *lds_word = queue_draw(order, slots);
  __syncthreads();
  const int slot = __builtin_amdgcn_readfirstlane(*lds_word);
  i32x4 rec = {-1, 0, 0, 0};
  if (slot >= 0) {
    const i32x4 r = *(const i32x4*)(order + 4 * (size_t)slot);
#pragma unroll
    for (int e = 0; e < 4; ++e) rec[e] = __builtin_amdgcn_readfirstlane(r[e]);
  }
  return rec;
}
// A workgroup that goes on to another unit after this one draws that unit's ticket ahead of time: one
// thread calls this while the tile copies of the current unit are in flight (the atomic and the record
// load that depends on it then cost nothing), and every thread picks the record up with
// queue_next_record() after a barrier at the end of the unit.  lds_rec: four words of LDS.
__device__ __forceinline__ void queue_prefetch(int* order, int slots, int* lds_rec) {
  const int slot = queue_draw(order, slots);
  i32x4 r = {-1, 0, 0, 0};
  if (slot >= 0) r = *(const i32x4*)(order + 4 * (size_t)slot);
  *(i32x4*)lds_rec = r;
}
// The same for a pass whose units are key blocks: the unit's eight min/max values (Section 4.2's table,
// row stride t_c, `kv_heads` units per batch row and key block) go into lds_rec[4..11] as well.
__device__ __forceinline__ void queue_prefetch_key_block(int* order, int slots, int* lds_rec, const int* table, int t_c,
                                                         int kv_heads) {
  const int slot = queue_draw(order, slots);
  i32x4 r = {-1, 0, 0, 0};
  if (slot >= 0) r = *(const i32x4*)(order + 4 * (size_t)slot);
  *(i32x4*)lds_rec = r;
  if (r[0] >= 0) {
    const int bh = r[0] / t_c, j = r[0] - bh * t_c, b = bh / kv_heads;
    const MinMax8 mm = load_minmax(table + (size_t)b * 8 * t_c, t_c, j);
#pragma unroll
    for (int e = 0; e < 8; ++e) lds_rec[4 + e] = mm.v[e];
  }
}
__device__ __forceinline__ i32x4 queue_next_record(const int* lds_rec) {
  const i32x4 r = *(const i32x4*)lds_rec;
  i32x4 rec;
#pragma unroll
  for (int e = 0; e < 4; ++e) rec[e] = __builtin_amdgcn_readfirstlane(r[e]);
  return rec;
}

// Ordered compaction shared by the tile loops: every thread of a 256-thread
// workgroup offers one candidate per pass (live or not, with its list entry);
// live entries are appended to list[] in candidate order.  `running` carries
// the count across passes.  Contains two barriers (LDS only: no wait for global memory).
__device__ __forceinline__ void append_live(bool live, int entry, int* list, int* wave_cnt, int& running) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long ballot = __ballot(live);
  const int prefix = __popcll(ballot & ((1ull << lane) - 1ull));
  if (lane == 0) wave_cnt[wave] = __popcll(ballot);
  barrier_nofence();   // only LDS is exchanged: the callers' global loads stay in flight across the list build
  int off = running, tot = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int cw = wave_cnt[w];
    if (w < wave) off += cw;
    tot += cw;
  }
  if (live) list[off + prefix] = entry;
  running += tot;
  barrier_nofence();
}

// Row-parallel loops: classify key blocks [j_begin, j_end) against the
// workgroup's rows [r0, r1) (Equation 4) and list the ones that are not fully
// masked, in order.  Each of the four waves owns rows_per_wave consecutive rows
// of the block and skips what Equation 4 proves fully masked for ITS rows (and
// skips the element mask where its rows are unmasked), so the entry also
// carries the class of each wave's sub-block -- computed here, once, from
// values already in registers, instead of re-reading the table every tile:
//   bits 0-15  j - j_begin      bits 16-17  class of the workgroup's tile
//   bits 18-25 class of wave w's sub-tile in bits 18+2w, 19+2w   (0 unmasked, 1 partial, 2 fully)
//   bits 26, 27  the workgroup's tile needs the element mask of the LT / of the UT pair (Equation 4's
//                partial test per pair; a pair whose bit is clear masks no element of the tile)
//   bit 28       every LT interval of the block reaches the end of the workgroup's rows (min LTE >= r1), so
//                "row >= LTS" alone decides the LT pair;  bit 29: every UT interval starts at or above the first
//                row (max UTS <= r0), so "row < UTE" alone decides the UT pair.  (Causal, window, document and
//                prefix masks are all of this kind: their intervals run to row N resp. from row 0.)
// Returns the number of entries (uniform over the workgroup).
__device__ __forceinline__ int build_live_key_blocks(const int* __restrict__ table, int t_c, int j_begin, int j_end,
                                                     int r0, int r1, int rows_per_wave, int* list, int* wave_cnt) {
  int running = 0;
  for (int base = j_begin; base < j_end; base += 256) {
    const int j = base + threadIdx.x;
    int cls = T_FULLY, entry = 0;
    if (j < j_end) {
      const MinMax8 mm = load_minmax(table, t_c, j);
      cls = classify_tile(r0, r1, mm);
      entry = (j - j_begin) | ((cls & 3) << 16) | (((cls >> 4) & 3) << 26) | ((mm.v[LTE_MIN] >= r1 ? 1 : 0) << 28) |
              ((mm.v[UTS_MAX] <= r0 ? 1 : 0) << 29);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int w0 = min(r0 + w * rows_per_wave, r1), w1 = min(w0 + rows_per_wave, r1);
        entry |= (classify_tile(w0, w1, mm) & 3) << (18 + 2 * w);
      }
    }
    append_live(cls != T_FULLY, entry, list, wave_cnt, running);
  }
  return running;
}
__device__ __forceinline__ int entry_block(int entry, int j_begin) { return j_begin + (entry & 0xFFFF); }
__device__ __forceinline__ int entry_tile_class(int entry) { return (entry >> 16) & 3; }
__device__ __forceinline__ int entry_wave_class(int entry, int wave) { return (entry >> (18 + 2 * wave)) & 3; }
// 1 = LT pair only, 2 = UT pair only, 3 = both (0 only for tiles that are not partially masked)
__device__ __forceinline__ int entry_need_pairs(int entry) { return (entry >> 26) & 3; }
// The same with 4 added where the one pair needed is decided by a single comparison per element (bits 28, 29):
// 5 = "row >= LTS", 6 = "row < UTE".
__device__ __forceinline__ int entry_mask_mode(int entry) {
  const int need = (entry >> 26) & 3;
  if (need == 1 && ((entry >> 28) & 1)) return 5;
  if (need == 2 && ((entry >> 29) & 1)) return 6;
  return need;
}

// Column-parallel loop: classify row blocks [i_begin, i_end) of block_r rows
// against one key block's min/max values; entries are i | class << 24.  The
// blocks that need no element mask come first (n_plain of them), the partially
// masked ones after, each group in ascending order.
__device__ __forceinline__ int build_live_row_blocks(const MinMax8& t, int n, int block_r, int i_begin, int i_end,
                                                     int* list, int* wave_cnt, int& n_plain) {
  if (FM_FAST_LIST && i_end - i_begin <= 64) {
    // Short range (a sliding window, a small document): one wave's lanes cover it, so every wave forms
    // the same two ballots and wave 0 writes the list; one barrier instead of four.
    const int lane = threadIdx.x & 63;
    const int i = i_begin + lane;
    int cls = T_FULLY;
    if (i < i_end) cls = classify_tile(i * block_r, min((i + 1) * block_r, n), t);
    const unsigned long long plain = __ballot(cls == T_UNMASKED), part = __ballot((cls & T_PARTIAL) != 0);
    const unsigned long long below = (1ull << lane) - 1ull;
    const int np = __popcll(plain);
    if (threadIdx.x < 64) {
      if (cls == T_UNMASKED) list[__popcll(plain & below)] = i | (cls << 24);
      if (cls & T_PARTIAL) list[np + __popcll(part & below)] = i | (cls << 24);
    }
    barrier_nofence();   // LDS only: the unit's K / V fragment loads stay in flight
    n_plain = np;
    return np + __popcll(part);
  }
  int running = 0;
#pragma unroll 1
  for (int pass = 0; pass < 2; ++pass) {
    for (int base = i_begin; base < i_end; base += 256) {
      const int i = base + threadIdx.x;
      int cls = T_FULLY;
      if (i < i_end) cls = classify_tile(i * block_r, min((i + 1) * block_r, n), t);
      const bool want = (pass == 0) ? (cls == T_UNMASKED) : ((cls & T_PARTIAL) != 0);
      append_live(want, i | (cls << 24), list, wave_cnt, running);
    }
    if (pass == 0) n_plain = running;
  }
  return running;
}

}  // namespace fm
