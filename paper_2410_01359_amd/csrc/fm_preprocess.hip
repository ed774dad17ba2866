// Preprocessing (Section 4.2): per key-block min/max of the four bound vectors,
// the exported tile-class dump (Equation 4), the per-unit work counts, and
// the unit queues built from them.
#include <climits>

#include "fm_common.h"
#include "fm_kernels.h"

namespace fm {

// One wave per (batch row, key block).  Lanes stride over the block's columns,
// then a butterfly over the 64 lanes leaves the 8 results in every lane.
__device__ __forceinline__ void preprocess_body(const int* __restrict__ lts, const int* __restrict__ lte,
                                                const int* __restrict__ uts, const int* __restrict__ ute, int n,
                                                int block_c, int t_c, int total_blocks, int* __restrict__ minmax,
                                                int block) {
  const int lane = threadIdx.x & 63;
  const int blk = block * 4 + (threadIdx.x >> 6);
  if (blk >= total_blocks) return;
  const int b = blk / t_c, j = blk - b * t_c;
  const int c0 = j * block_c;
  const int c1 = min(c0 + block_c, n);
  const int* vec[4] = {lts + (size_t)b * n, lte + (size_t)b * n, uts + (size_t)b * n, ute + (size_t)b * n};
  int mx[4], mn[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    mx[a] = INT32_MIN;
    mn[a] = INT32_MAX;
  }
  for (int c = c0 + lane; c < c1; c += 64) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int x = vec[a][c];
      mx[a] = max(mx[a], x);
      mn[a] = min(mn[a], x);
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      mx[a] = max(mx[a], __shfl_xor(mx[a], off, 64));
      mn[a] = min(mn[a], __shfl_xor(mn[a], off, 64));
    }
  }
  if (lane == 0) {
    int* out = minmax + (size_t)b * 8 * t_c;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      out[(2 * a) * t_c + j] = mx[a];
      out[(2 * a + 1) * t_c + j] = mn[a];
    }
  }
}

__global__ __launch_bounds__(256) void preprocess_kernel(const int* __restrict__ lts, const int* __restrict__ lte,
                                                         const int* __restrict__ uts, const int* __restrict__ ute,
                                                         int n, int block_c, int t_c, int total_blocks,
                                                         int* __restrict__ minmax) {
  preprocess_body(lts, lte, uts, ute, n, block_c, t_c, total_blocks, minmax, blockIdx.x);
}

// The tables of two block widths in one launch (the backward's two loops tile the keys differently):
// workgroups [0, blocks_a) build table a, the rest table b.
__global__ __launch_bounds__(256) void preprocess2_kernel(const int* __restrict__ lts, const int* __restrict__ lte,
                                                          const int* __restrict__ uts, const int* __restrict__ ute,
                                                          int n, int batch, int block_c_a, int* __restrict__ minmax_a,
                                                          int blocks_a, int block_c_b, int* __restrict__ minmax_b) {
  const bool first = (int)blockIdx.x < blocks_a;
  const int block_c = first ? block_c_a : block_c_b;
  const int t_c = (n + block_c - 1) / block_c;
  preprocess_body(lts, lte, uts, ute, n, block_c, t_c, batch * t_c, first ? minmax_a : minmax_b,
                  first ? blockIdx.x : blockIdx.x - blocks_a);
}

__global__ __launch_bounds__(256) void classify_kernel(const int* __restrict__ minmax, int n, int block_r, int t_r,
                                                       int t_c, uint8_t* __restrict__ cls) {
  const int b = blockIdx.z, i = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= t_c) return;
  const MinMax8 t = load_minmax(minmax + (size_t)b * 8 * t_c, t_c, j);
  const int r0 = i * block_r;
  const int r1 = min(r0 + block_r, n);
  cls[((size_t)b * t_r + i) * t_c + j] = (uint8_t)classify_tile(r0, r1, t);
}

// Padded copies of the bound vectors for a sequence length that is not a multiple of 128: the
// columns past the end get an interval that masks every row (LTS = INT_MIN, LTE = INT_MAX), so
// the tile loops treat them like any other masked key and every vector read stays in bounds.
__global__ __launch_bounds__(256) void pad_bounds_kernel(const int* __restrict__ lts, const int* __restrict__ lte,
                                                         const int* __restrict__ uts, const int* __restrict__ ute,
                                                         int batch, int n, int np, int* __restrict__ padded) {
  const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
  if (gid >= (long long)batch * np) return;
  const int b = (int)(gid / np), j = (int)(gid % np);
  const size_t plane = (size_t)batch * np, src = (size_t)b * n + j;
  const bool in = j < n;
  padded[0 * plane + gid] = in ? lts[src] : INT_MIN;
  padded[1 * plane + gid] = in ? lte[src] : INT_MAX;
  padded[2 * plane + gid] = in ? uts[src] : 0;
  padded[3 * plane + gid] = in ? ute[src] : 0;
}

// Work of one row block = number of key blocks that are not fully masked, and
// the range of key blocks that contains them (the tile loops only scan that).
// One wave per (batch row, row block); lanes stride over the key blocks.
__device__ __forceinline__ void row_work_body(const int* __restrict__ minmax, int n, int block_r, int t_r, int t_c,
                                              int total_units, int* __restrict__ work, int* __restrict__ range,
                                              int block) {
  const int lane = threadIdx.x & 63;
  const int u = block * 4 + (threadIdx.x >> 6);
  if (u >= total_units) return;
  const int b = u / t_r, i = u - b * t_r;
  const int r0 = i * block_r, r1 = min(r0 + block_r, n);
  const int* table = minmax + (size_t)b * 8 * t_c;
  int cnt = 0, lo = t_c, hi = 0;
#pragma unroll 8   // the table loads of several iterations in flight: the scan is bound by their latency
  for (int j = lane; j < t_c; j += 64)
    if (classify_tile(r0, r1, load_minmax(table, t_c, j)) != T_FULLY) {
      ++cnt;
      lo = min(lo, j);
      hi = j + 1;
    }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    cnt += __shfl_xor(cnt, off, 64);
    lo = min(lo, __shfl_xor(lo, off, 64));
    hi = max(hi, __shfl_xor(hi, off, 64));
  }
  if (lane == 0) {
    work[u] = cnt;
    range[2 * u] = cnt ? lo : 0;
    range[2 * u + 1] = hi;
  }
}

__global__ __launch_bounds__(256) void row_work_kernel(const int* __restrict__ minmax, int n, int block_r, int t_r,
                                                       int t_c, int total_units, int* __restrict__ work,
                                                       int* __restrict__ range) {
  row_work_body(minmax, n, block_r, t_r, t_c, total_units, work, range, blockIdx.x);
}

// Work of one key block = number of row blocks that are not fully masked.
__device__ __forceinline__ void col_work_body(const int* __restrict__ minmax, int n, int block_r, int t_r, int t_c,
                                              int total_units, int* __restrict__ work, int* __restrict__ range,
                                              int block) {
  const int lane = threadIdx.x & 63;
  const int u = block * 4 + (threadIdx.x >> 6);
  if (u >= total_units) return;
  const int b = u / t_c, j = u - b * t_c;
  const MinMax8 t = load_minmax(minmax + (size_t)b * 8 * t_c, t_c, j);
  int cnt = 0, lo = t_r, hi = 0;
  for (int i = lane; i < t_r; i += 64) {
    const int r0 = i * block_r, r1 = min(r0 + block_r, n);
    if (classify_tile(r0, r1, t) != T_FULLY) {
      ++cnt;
      lo = min(lo, i);
      hi = i + 1;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    cnt += __shfl_xor(cnt, off, 64);
    lo = min(lo, __shfl_xor(lo, off, 64));
    hi = max(hi, __shfl_xor(hi, off, 64));
  }
  if (lane == 0) {
    work[u] = cnt;
    range[2 * u] = cnt ? lo : 0;
    range[2 * u + 1] = hi;
  }
}

__global__ __launch_bounds__(256) void col_work_kernel(const int* __restrict__ minmax, int n, int block_r, int t_r,
                                                       int t_c, int total_units, int* __restrict__ work,
                                                       int* __restrict__ range) {
  col_work_body(minmax, n, block_r, t_r, t_c, total_units, work, range, blockIdx.x);
}

// One pass's work pre-pass as arguments, so that the backward can run both of its passes' in one launch.
struct WorkJob {
  const int* minmax;
  int block_r, t_r, t_c, total_units;
  int* work;
  int* range;
};
// workgroups [0, blocks_rows) count per row block (job `rows`), the rest per key block (job `cols`)
__global__ __launch_bounds__(256) void work2_kernel(WorkJob rows, int blocks_rows, WorkJob cols, int n) {
  if ((int)blockIdx.x < blocks_rows)
    row_work_body(rows.minmax, n, rows.block_r, rows.t_r, rows.t_c, rows.total_units, rows.work, rows.range, blockIdx.x);
  else
    col_work_body(cols.minmax, n, cols.block_r, cols.t_r, cols.t_c, cols.total_units, cols.work, cols.range,
                  blockIdx.x - blocks_rows);
}

// Unit queues (the tile scheduler).  Workgroup x of a launch runs on XCD x % 8.
// Units are dealt into 8 queues (one per XCD: by slice (batch row, head) when the
// slice count is a multiple of 8, so that the units sharing one head's K/V also
// share one L2), each queue is sorted heaviest first within groups of slices (see
// order_kernel; work quantised to 512 levels), and the queues are interleaved:
// slot 8*s + g = position s of queue g.  A workgroup draws the next ticket of its
// XCD's queue when it starts, so every queue is worked off longest-job-first; the
// launch holds more workgroups than there are slots, and a workgroup that finds its
// own queue empty draws from the queue that has most left.  (The XCDs do not run
// at the same speed: with equal shares the slowest one finishes about a tenth
// later than the fastest.)
// A slot is the record {unit, first live block, one past the last live block, 0},
// so a workgroup learns all it needs to start from one 16-byte load; slots with
// no unit hold unit = -1.  The kernel also zeroes the 8 queue counters behind
// the slots.
constexpr int kLevels = 512;
constexpr int kGroups = FM_QUEUES;
// Queue of block i of slice s (slices = batch rows x heads, numbered batch-major).  Slices go to
// queues whole, slice s to queue s % 8, as long as they fill rounds of 8; the r < 8 slices left over
// (all slices if there are fewer than 8) are shared block by block: four of them between 2 queues
// each, two between 4 queues each, one between all 8 (r = 4a + 2b + c), which keeps the queues
// equally long and every slice in as few L2s as that allows.
__host__ __device__ inline int fm_queue_of(int s, int i, int whole, int r) {
  if (s < whole) return s % FM_QUEUES;
  int j = s - whole;
  if (r & 4) {
    if (j < 4) return 2 * j + (i & 1);
    j -= 4;
  }
  if (r & 2) {
    if (j < 2) return 4 * j + (i & 3);
    j -= 2;
  }
  return i & 7;
}
// Workgroups of the queue-building launch: per queue, one for every FM_QUEUE_CHUNK whole slices and one
// for its part of the slices left over, its unused slots and its counter.
static inline int fm_order_grid(int B, int H) {
  return FM_QUEUES * (((B * H) / FM_QUEUES + FM_QUEUE_CHUNK - 1) / FM_QUEUE_CHUNK + 1);
}

// work and range are indexed [batch row][block]; a unit is (batch row, head, block).
// A queue holds its whole slices in groups of FM_QUEUE_CHUNK, one group after the other, and the
// shared slices last: the units that run at the same time then belong to few slices and share their
// K/V (or Q/dO) in the XCD's L2 and in the memory-side cache.  (Ranking a queue's units of ALL slices
// by work alone spreads the resident workgroups over as many slices as the queue has; with 64 slices
// per queue the loops then stream from HBM and lose a quarter of their rate.)  One workgroup of the
// launch sorts one group of one queue.  Within a group units are ranked as rank_of() describes.
struct OrderJob {
  const int* work;
  const int* range;
  int batch, heads, units_per_bh;   // a queue slice: (batch row, head); with grouped K/V heads `heads` counts K/V
                                    // heads and a slice holds the units of all query heads of the group
  int blocks;                       // blocks per (batch row, query head): units_per_bh = group size x blocks
  int max_work, slots;
  i32x4* order;
  int* counters;
};
// Workgroup `block` of `blocks` = 8 x (groups of whole slices + 1): block % 8 is the queue, block / 8 the
// group; the last group is the shared slices, whose workgroups also clear their queue's unused slots
// and counter.
__device__ __forceinline__ void order_body(const OrderJob& job, int block, int blocks) {
  const int* __restrict__ work = job.work;
  const int* __restrict__ range = job.range;
  const int heads = job.heads, units_per_bh = job.units_per_bh, max_work = job.max_work;
  const int blocks_per_head = job.blocks;
  const int slots = job.slots;
  i32x4* __restrict__ order = job.order;
  __shared__ int hist[kLevels];
  __shared__ int wave_sum[16];
  const int tid = threadIdx.x;
  const int slices = job.batch * heads;
  const int whole = (slices / kGroups) * kGroups, left = slices - whole;
  const int g = block % kGroups, grp = block / kGroups;
  const bool tail = grp == blocks / kGroups - 1;
  constexpr int chunk = FM_QUEUE_CHUNK;
  // Candidates of this workgroup: the units of its queue's whole slices of the group (slice numbers
  // (grp * chunk + c) * 8 + g), or every unit of the shared slices, of which it keeps its queue's.
  const int first_slice = tail ? whole : (grp * chunk) * kGroups + g;
  const int n_slices = tail ? left : min(chunk, (whole - first_slice + kGroups - 1) / kGroups);
  const int candidates = n_slices * units_per_bh;
  const int pos_base = tail ? (whole / kGroups) * units_per_bh : grp * chunk * units_per_bh;
  auto unit_at = [&](int idx) {   // unit number of candidate idx, or -1 if it belongs to another queue
    const int c = idx / units_per_bh, i = idx - c * units_per_bh;
    const int slice = tail ? first_slice + c : first_slice + c * kGroups;
    if (tail && fm_queue_of(slice, i, whole, left) != g) return -1;
    return slice * units_per_bh + i;
  };
  if (tid < kLevels) hist[tid] = 0;
  if (tail) {
    // this queue's positions behind the whole slices: filled below as far as there are shared slices
    for (int p = pos_base + tid; p * kGroups + g < slots; p += 1024) order[p * kGroups + g] = i32x4{-1, 0, 0, 0};
    if (tid == 0) job.counters[g] = 0;
  }
  __syncthreads();
  auto rank_of = [&](int u) {
    const int ru = (u / (heads * units_per_bh)) * blocks_per_head + u % blocks_per_head;
    const int w_u = work[ru], mw = max_work > 0 ? max_work : 1;
    // Heavy units (an eighth of the largest possible work or more) are ranked finely by work: their
    // order decides how evenly the queue ends.  Lighter ones are ranked by octave of work and, within
    // an octave, by where their live range starts: units of similar size that stream the same blocks
    // (the rows of one document) then sit next to each other in the queue, run at the same time and
    // share the blocks in L2.
    constexpr int kFine = 384, kOct = 8, kPos = (kLevels - kFine) / kOct;
    int rank;
    if ((long long)w_u * 8 >= mw) {
      rank = (int)(((long long)(mw - min(w_u, mw)) * 8 * (kFine - 1)) / ((long long)mw * 7));
      rank = min(max(rank, 0), kFine - 1);
    } else {
      const int oct = min(max((int)__log2f((float)mw / (8.f * (float)max(w_u, 1))), 0), kOct - 1);
      const int pos = min((int)(((long long)range[2 * ru] * kPos) / mw), kPos - 1);
      rank = kFine + oct * kPos + pos;
    }
    return rank;
  };
  for (int idx = tid; idx < candidates; idx += 1024) {
    const int u = unit_at(idx);
    if (u >= 0) atomicAdd(&hist[rank_of(u)], 1);
  }
  __syncthreads();
  // exclusive scan of hist (512 entries, one per thread of the first 8 waves)
  const int v = tid < kLevels ? hist[tid] : 0;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(incl, off, 64);
    if ((tid & 63) >= off) incl += y;
  }
  if ((tid & 63) == 63) wave_sum[tid >> 6] = incl;
  __syncthreads();
  int base = 0;
  for (int w = 0; w < (tid >> 6); ++w) base += wave_sum[w];
  __syncthreads();
  if (tid < kLevels) hist[tid] = base + incl - v;   // first queue position (within the group) of this rank
  __syncthreads();
  for (int idx = tid; idx < candidates; idx += 1024) {
    const int u = unit_at(idx);
    if (u < 0) continue;
    const int pos = pos_base + atomicAdd(&hist[rank_of(u)], 1);
    const int slot = pos * kGroups + g;
    const int ru = (u / (heads * units_per_bh)) * blocks_per_head + u % blocks_per_head;
    if (slot < slots) order[slot] = i32x4{u, range[2 * ru], range[2 * ru + 1], 0};
  }
}

__global__ __launch_bounds__(1024) void order_kernel(OrderJob job) { order_body(job, blockIdx.x, gridDim.x); }

// the queues of two passes in one launch: workgroups [0, blocks_a) build job a's, the rest job b's
__global__ __launch_bounds__(1024) void order2_kernel(OrderJob a, int blocks_a, OrderJob b) {
  if ((int)blockIdx.x < blocks_a)
    order_body(a, blockIdx.x, blocks_a);
  else
    order_body(b, blockIdx.x - blocks_a, gridDim.x - blocks_a);
}

}  // namespace fm

using namespace fm;

hipError_t fm_launch_preprocess(const int* lts, const int* lte, const int* uts, const int* ute, int B, int N,
                                int block_c, int* minmax, hipStream_t stream) {
  const int t_c = (N + block_c - 1) / block_c;
  const int total = B * t_c;
  hipLaunchKernelGGL(preprocess_kernel, dim3((total + 3) / 4), dim3(256), 0, stream, lts, lte, uts, ute, N, block_c,
                     t_c, total, minmax);
  return hipGetLastError();
}

hipError_t fm_launch_pad_bounds(const int* lts, const int* lte, const int* uts, const int* ute, int B, int N, int Np,
                                int* padded, hipStream_t stream) {
  const long long total = (long long)B * Np;
  hipLaunchKernelGGL(pad_bounds_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, lts, lte, uts, ute,
                     B, N, Np, padded);
  return hipGetLastError();
}

hipError_t fm_launch_classify(const int* minmax, int B, int N, int block_r, int block_c, uint8_t* cls,
                              hipStream_t stream) {
  const int t_c = (N + block_c - 1) / block_c;
  const int t_r = (N + block_r - 1) / block_r;
  hipLaunchKernelGGL(classify_kernel, dim3((t_c + 255) / 256, t_r, B), dim3(256), 0, stream, minmax, N, block_r, t_r,
                     t_c, cls);
  return hipGetLastError();
}

// H heads per batch row in groups of `group` that share a K/V head (1: no sharing): the heads of a group
// form one queue slice, so that they run on the XCD whose L2 holds their K/V.
static OrderJob order_job(int* work, int* range, int B, int H, int group, int blocks, int max_work, int* order) {
  const int slots = fm_order_slots(B * H * blocks);
  return OrderJob{work, range, B, H / group, group * blocks, blocks, max_work, slots, (i32x4*)order,
                  order + 4 * (size_t)slots};
}

hipError_t fm_launch_row_order(const int* minmax, int B, int H, int Hk, int N, int block_r, int block_c, int* work,
                               int* range, int* order, hipStream_t stream) {
  const int t_c = (N + block_c - 1) / block_c;
  const int t_r = (N + block_r - 1) / block_r;
  const int total = B * t_r;
  hipLaunchKernelGGL(row_work_kernel, dim3((total + 3) / 4), dim3(256), 0, stream, minmax, N, block_r, t_r, t_c, total,
                     work, range);
  hipLaunchKernelGGL(order_kernel, dim3(fm_order_grid(B, Hk)), dim3(1024), 0, stream,
                     order_job(work, range, B, H, H / Hk, t_r, t_c, order));
  return hipGetLastError();
}

hipError_t fm_launch_col_order(const int* minmax, int B, int H, int N, int block_r, int block_c, int* work,
                               int* range, int* order, hipStream_t stream) {
  const int t_c = (N + block_c - 1) / block_c;
  const int t_r = (N + block_r - 1) / block_r;
  const int total = B * t_c;
  hipLaunchKernelGGL(col_work_kernel, dim3((total + 3) / 4), dim3(256), 0, stream, minmax, N, block_r, t_r, t_c, total,
                     work, range);
  hipLaunchKernelGGL(order_kernel, dim3(fm_order_grid(B, H)), dim3(1024), 0, stream,
                     order_job(work, range, B, H, 1, t_c, t_r, order));
  return hipGetLastError();
}

// The backward's setup in three launches: both min/max tables, both work pre-passes, both passes' queues.
hipError_t fm_launch_bwd_setup(const int* lts, const int* lte, const int* uts, const int* ute, int B, int H, int Hk,
                               int N, const FmSetup& rows, const FmSetup& cols, hipStream_t stream) {
  const int tc_r = (N + rows.block_c - 1) / rows.block_c, tr_r = (N + rows.block_r - 1) / rows.block_r;
  const int tc_c = (N + cols.block_c - 1) / cols.block_c, tr_c = (N + cols.block_r - 1) / cols.block_r;
  const int pre_a = (B * tc_r + 3) / 4, pre_b = (B * tc_c + 3) / 4;
  hipLaunchKernelGGL(preprocess2_kernel, dim3(pre_a + pre_b), dim3(256), 0, stream, lts, lte, uts, ute, N, B,
                     rows.block_c, rows.minmax, pre_a, cols.block_c, cols.minmax);
  const WorkJob wr{rows.minmax, rows.block_r, tr_r, tc_r, B * tr_r, rows.work, rows.range};
  const WorkJob wc{cols.minmax, cols.block_r, tr_c, tc_c, B * tc_c, cols.work, cols.range};
  const int work_a = (wr.total_units + 3) / 4, work_b = (wc.total_units + 3) / 4;
  hipLaunchKernelGGL(work2_kernel, dim3(work_a + work_b), dim3(256), 0, stream, wr, work_a, wc, N);
  const int grid_a = fm_order_grid(B, Hk), grid_b = fm_order_grid(B, Hk);
  hipLaunchKernelGGL(order2_kernel, dim3(grid_a + grid_b), dim3(1024), 0, stream,
                     order_job(rows.work, rows.range, B, H, H / Hk, tr_r, tc_r, rows.order), grid_a,
                     order_job(cols.work, cols.range, B, Hk, 1, tc_c, tr_c, cols.order));
  return hipGetLastError();
}
