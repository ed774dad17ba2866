// C ABI of the library: argument validation, workspace carving, launches.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdio>
#include <cstring>

#include "../../include/flashmask.h"
#include "fm_kernels.h"

namespace {

thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e) {
  snprintf(g_hip_error, sizeof(g_hip_error), "%s", hipGetErrorString(e));
  return FM_ERR_HIP;
}

// Optional measurement aid: events recorded between the internal launches.
hipEvent_t* g_prof_events = nullptr;
int g_prof_count = 0;
inline void mark(int idx, hipStream_t stream) {
  if (g_prof_events && idx < g_prof_count && g_prof_events[idx]) (void)hipEventRecord(g_prof_events[idx], stream);
}

// Scratch of flashmask_fwd_noalloc: one copy per device, part of the library's code object.  In host
// code the name below only stands for the symbol; the memory's address on the current device comes from
// hipGetSymbolAddress (static_scratch) and is what kernels, copies and clears must be given.
static __device__ __align__(256) unsigned char scratch[FLASHMASK_NOALLOC_SCRATCH_BYTES];
std::atomic<void*> g_scratch_ptr[FM_MAX_DEVICES];

// Address of `scratch` on the current device, looked up once per device.
hipError_t static_scratch(void** ptr) {
  int dev = 0;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  if (dev < 0 || dev >= FM_MAX_DEVICES) return hipErrorInvalidDevice;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread looks up the same address
  }
  *ptr = p;
  return hipSuccess;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_shape(int B, int H, int N, int d) {
  if (B <= 0 || H <= 0 || N <= 0) return FM_ERR_SHAPE;
  if (d != 64 && d != 128) return FM_ERR_SHAPE;
  if (N > (1 << 30)) return FM_ERR_SHAPE;
  if ((long long)B * H * ((N + 127) / 128 * 2) >= (1ll << 31) / 8) return FM_ERR_SHAPE;
  return FM_OK;
}

// Stride record of a contiguous [B, heads, N, d] tensor.
FmStride dense(int heads, int N, int d) { return FmStride{(long long)heads * N * d, (long long)N * d, (long long)d}; }
FmStride to_kernel(const flashmask_strides& s) { return FmStride{s.batch, s.head, s.row}; }

// Strides the kernels can address: 16-byte vectors along d stay aligned (multiples of 8 elements),
// rows do not overlap (row >= d) and 64 rows fit a 32-bit byte offset; a size-1 axis may have any stride.
int check_strides(const flashmask_strides* s, int B, int heads, int N, int d) {
  if (!s) return FM_ERR_NULL;
  if (s->batch % 8 || s->head % 8 || s->row % 8) return FM_ERR_ALIGN;
  if (s->row < d || s->row >= (1ll << 24)) return FM_ERR_SHAPE;
  if (s->batch < 0 || s->head < 0) return FM_ERR_SHAPE;
  if ((B > 1 && s->batch == 0) || (heads > 1 && s->head == 0)) return FM_ERR_SHAPE;
  return FM_OK;
}

// The tile loops work at the sequence length rounded up to a multiple of 128; a sequence that is
// not such a multiple gets padded copies of its bound vectors at the front of the workspace.
inline int padded_len(int N) { return (N + 127) / 128 * 128; }
inline size_t padded_bounds_bytes(int B, int N) {
  return padded_len(N) == N ? 0 : align_up((size_t)4 * B * padded_len(N) * 4, 256);
}

// Workspace layout of a pass: tables, work counts and unit queues.
struct PassSpace {
  size_t minmax, work, range, order, total;
};
PassSpace pass_space(int B, int H, int N, int block_r, int block_c, bool row_units, size_t start) {
  PassSpace s;
  const size_t t_c = (N + block_c - 1) / block_c, t_r = (N + block_r - 1) / block_r;
  const size_t per = row_units ? t_r : t_c;
  s.minmax = start;
  s.work = align_up(s.minmax + (size_t)B * 8 * t_c * 4, 256);
  s.range = align_up(s.work + (size_t)B * per * 4, 256);
  s.order = align_up(s.range + (size_t)B * per * 8, 256);
  s.total = align_up(s.order + fm_order_bytes((int)((size_t)B * H * per)), 256);
  return s;
}

}  // namespace

extern "C" {

const char* flashmask_strerror(int code) {
  switch (code) {
    case FM_OK: return "ok";
    case FM_ERR_NULL: return "a required pointer is NULL";
    case FM_ERR_SHAPE: return "unsupported shape (need B,H,N > 0, d in {64,128})";
    case FM_ERR_ALIGN: return "a tensor pointer is not 16-byte aligned";
    case FM_ERR_WORKSPACE: return "workspace is NULL, misaligned or too small";
    case FM_ERR_HIP: return "HIP launch failed (see flashmask_last_hip_error)";
    case FM_ERR_ARG: return "bad scalar argument (unknown pass id, or scale not a positive finite number)";
    case FM_ERR_STATIC_LIMIT:
      return "flashmask_fwd_noalloc: the problem needs more scratch than the library's static buffer holds "
             "(flashmask_workspace_bytes(FM_PASS_FWD, ...) > FLASHMASK_NOALLOC_SCRATCH_BYTES)";
    default: return "unknown flashmask error code";
  }
}

const char* flashmask_last_hip_error(void) { return g_hip_error; }

int flashmask_profile_events(void** events, int count) {
  if (count < 0 || (count > 0 && !events)) return FM_ERR_ARG;
  g_prof_events = count ? (hipEvent_t*)events : nullptr;
  g_prof_count = count;
  return FM_OK;
}

int flashmask_mfma_ceiling(const void* operands, float* sink, int workgroups, int iters, int shape, double* flop,
                           void* hip_stream) {
  if (!operands || !sink || !flop) return FM_ERR_NULL;
  if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || iters > (1 << 24) || shape < 0 || shape > 2)
    return FM_ERR_ARG;
  if (misaligned(operands)) return FM_ERR_ALIGN;
  *flop = 2.0 * 32 * 32 * 16 * (double)fm_mfma_ceiling_ops_per_iter() * iters * 4.0 * workgroups;
  hipError_t e = fm_launch_mfma_ceiling(operands, sink, workgroups, iters, shape, (hipStream_t)hip_stream);
  return e == hipSuccess ? FM_OK : hip_fail(e);
}

int flashmask_atomic_ceiling(float* acc, int heads, int n_tiles, int tiles, int workgroups, double* bytes,
                              void* hip_stream) {
  if (!acc || !bytes) return FM_ERR_NULL;
  if (heads <= 0 || n_tiles <= 0 || tiles <= 0 || workgroups <= 0 || workgroups > (1 << 20) || tiles > (1 << 20))
    return FM_ERR_ARG;
  if ((long long)heads * n_tiles >= (1ll << 31) / (64 * 128)) return FM_ERR_SHAPE;
  *bytes = 4.0 * 64 * 128 * (double)tiles * workgroups;
  hipError_t e = fm_launch_atomic_ceiling(acc, n_tiles, tiles, heads, workgroups, (hipStream_t)hip_stream);
  return e == hipSuccess ? FM_OK : hip_fail(e);
}

int flashmask_tile_shape(int pass, int d, int* block_r, int* block_c) {
  if (!block_r || !block_c) return FM_ERR_NULL;
  if (d != 64 && d != 128) return FM_ERR_SHAPE;
  switch (pass) {
    case FM_PASS_FWD: *block_r = FM_FWD_BR; *block_c = FM_FWD_BC; return FM_OK;
    case FM_PASS_BWD_DKDV: *block_r = FM_DKDV_BR; *block_c = FM_DKDV_BC; return FM_OK;
    case FM_PASS_BWD_DQ: *block_r = FM_DQ_BR; *block_c = fm_dq_bc(d); return FM_OK;
    default: return FM_ERR_ARG;
  }
}

size_t flashmask_workspace_bytes(int pass, int B, int H, int N, int d) {
  if (check_shape(B, H, N, d) != FM_OK) return 0;
  const int Np = padded_len(N);
  const size_t pad = padded_bounds_bytes(B, N);
  if (pass == FM_PASS_FWD) return pad + pass_space(B, H, Np, FM_FWD_BR, FM_FWD_BC, true, 0).total;
  if (pass == FM_PASS_BWD) {
    const PassSpace dq = pass_space(B, H, Np, FM_DQ_BR, fm_dq_bc(d), true, 0);
    const PassSpace kv = pass_space(B, H, Np, FM_DKDV_BR, FM_DKDV_BC, false, dq.total);
    return pad + kv.total + 2 * align_up((size_t)B * H * Np * 4, 256);  // + D vector + log2-domain lse
  }
  return 0;
}

int flashmask_preprocess(const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute, int B, int N,
                         int block_c, int32_t* minmax, void* hip_stream) {
  if (!lts || !lte || !uts || !ute || !minmax) return FM_ERR_NULL;
  if (B <= 0 || N <= 0 || block_c <= 0 || block_c % 32 != 0) return FM_ERR_SHAPE;
  hipError_t e = fm_launch_preprocess(lts, lte, uts, ute, B, N, block_c, minmax, (hipStream_t)hip_stream);
  return e == hipSuccess ? FM_OK : hip_fail(e);
}

int flashmask_classify(const int32_t* minmax, int B, int N, int block_r, int block_c, uint8_t* cls, void* hip_stream) {
  if (!minmax || !cls) return FM_ERR_NULL;
  if (B <= 0 || N <= 0 || block_c <= 0 || block_r <= 0) return FM_ERR_SHAPE;
  const long long t_r = (N + block_r - 1) / block_r;
  if (t_r > 65535 || B > 65535) return FM_ERR_SHAPE;
  hipError_t e = fm_launch_classify(minmax, B, N, block_r, block_c, cls, (hipStream_t)hip_stream);
  return e == hipSuccess ? FM_OK : hip_fail(e);
}

static int fwd_impl(const void* q, const void* k, const void* v, const int32_t* lts, const int32_t* lte,
                    const int32_t* uts, const int32_t* ute, float scale, void* out, float* lse, int B, int H, int Hk,
                    int N, int d, const FmStride* st /* q, k, v, out; NULL = contiguous, Hk == H */, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (!q || !k || !v || !lts || !lte || !uts || !ute || !out || !lse) return FM_ERR_NULL;
  if (int rc = check_shape(B, H, N, d)) return rc;
  if (!(scale > 0.f) || !(scale < 3.0e38f)) return FM_ERR_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(lts) || misaligned(lte) ||
      misaligned(uts) || misaligned(ute) || misaligned(lse))
    return FM_ERR_ALIGN;
  const size_t need = flashmask_workspace_bytes(FM_PASS_FWD, B, H, N, d);
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return FM_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)hip_stream;
  const int Np = padded_len(N);
  char* ws = (char*)workspace;
  mark(0, stream);
  hipError_t e;
  if (Np != N) {   // padded bound vectors first
    int* padded = (int*)ws;
    e = fm_launch_pad_bounds(lts, lte, uts, ute, B, N, Np, padded, stream);
    if (e != hipSuccess) return hip_fail(e);
    const size_t plane = (size_t)B * Np;
    lts = padded; lte = padded + plane; uts = padded + 2 * plane; ute = padded + 3 * plane;
    ws += padded_bounds_bytes(B, N);
  }
  const PassSpace sp = pass_space(B, H, Np, FM_FWD_BR, FM_FWD_BC, true, 0);
  int* minmax = (int*)(ws + sp.minmax);
  int* work = (int*)(ws + sp.work);
  int* range = (int*)(ws + sp.range);
  int* order = (int*)(ws + sp.order);
  e = fm_launch_preprocess(lts, lte, uts, ute, B, Np, FM_FWD_BC, minmax, stream);
  if (e != hipSuccess) return hip_fail(e);
  e = fm_launch_row_order(minmax, B, H, Hk, Np, FM_FWD_BR, FM_FWD_BC, work, range, order, stream);
  if (e != hipSuccess) return hip_fail(e);
  mark(1, stream);
  FmFwdArgs a;
  a.q = q; a.k = k; a.v = v;
  a.lts = lts; a.lte = lte; a.uts = uts; a.ute = ute;
  a.minmax = minmax; a.order = order;
  a.out = out; a.lse = lse; a.scale = scale;
  a.B = B; a.H = H; a.N = N; a.Np = Np; a.d = d;
  a.slots = fm_order_slots(B * H * (Np / FM_FWD_BR));
  a.general = st != nullptr;
  a.Hk = Hk;
  if (st) { a.sq = st[0]; a.sk = st[1]; a.sv = st[2]; a.so = st[3]; }
  else { a.sq = a.so = dense(H, N, d); a.sk = a.sv = dense(Hk, N, d); }
  e = fm_launch_fwd(a, stream);
  if (e != hipSuccess) return hip_fail(e);
  mark(2, stream);
  return FM_OK;
}

int flashmask_unit_queues(int pass, const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute,
                          int B, int H, int N, int d, int32_t* records, int* slots, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  if (!lts || !lte || !uts || !ute || !slots) return FM_ERR_NULL;
  if (int rc = check_shape(B, H, N, d)) return rc;
  if (pass != FM_PASS_FWD && pass != FM_PASS_BWD_DQ && pass != FM_PASS_BWD_DKDV) return FM_ERR_ARG;
  const bool rows = pass != FM_PASS_BWD_DKDV;
  const int br = pass == FM_PASS_FWD ? FM_FWD_BR : rows ? FM_DQ_BR : FM_DKDV_BR;
  const int bc = pass == FM_PASS_FWD ? FM_FWD_BC : rows ? fm_dq_bc(d) : FM_DKDV_BC;
  const int Np = padded_len(N);
  *slots = fm_order_slots(B * H * (Np / (rows ? br : bc)));
  if (!records) return FM_OK;   // size query
  if (misaligned(lts) || misaligned(lte) || misaligned(uts) || misaligned(ute) || misaligned(records)) return FM_ERR_ALIGN;
  const size_t need = flashmask_workspace_bytes(rows && pass == FM_PASS_FWD ? FM_PASS_FWD : FM_PASS_BWD, B, H, N, d);
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return FM_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  hipError_t e;
  if (Np != N) {
    int* padded = (int*)ws;
    e = fm_launch_pad_bounds(lts, lte, uts, ute, B, N, Np, padded, stream);
    if (e != hipSuccess) return hip_fail(e);
    const size_t plane = (size_t)B * Np;
    lts = padded; lte = padded + plane; uts = padded + 2 * plane; ute = padded + 3 * plane;
    ws += padded_bounds_bytes(B, N);
  }
  const PassSpace sp = pass_space(B, H, Np, br, bc, rows, 0);
  int* minmax = (int*)(ws + sp.minmax);
  e = fm_launch_preprocess(lts, lte, uts, ute, B, Np, bc, minmax, stream);
  if (e != hipSuccess) return hip_fail(e);
  e = rows ? fm_launch_row_order(minmax, B, H, H, Np, br, bc, (int*)(ws + sp.work), (int*)(ws + sp.range),
                                 (int*)(ws + sp.order), stream)
           : fm_launch_col_order(minmax, B, H, Np, br, bc, (int*)(ws + sp.work), (int*)(ws + sp.range),
                                 (int*)(ws + sp.order), stream);
  if (e != hipSuccess) return hip_fail(e);
  e = hipMemcpyAsync(records, ws + sp.order, (size_t)*slots * 16, hipMemcpyDeviceToDevice, stream);
  return e == hipSuccess ? FM_OK : hip_fail(e);
}

int flashmask_fwd(const void* q, const void* k, const void* v, const int32_t* lts, const int32_t* lte,
                  const int32_t* uts, const int32_t* ute, float scale, void* out, float* lse, int B, int H, int N,
                  int d, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return fwd_impl(q, k, v, lts, lte, uts, ute, scale, out, lse, B, H, H, N, d, nullptr, workspace, workspace_bytes,
                  hip_stream);
}

int flashmask_fwd_noalloc(const void* q, const void* k, const void* v, const int32_t* lts, const int32_t* lte,
                          const int32_t* uts, const int32_t* ute, float scale, void* out, float* lse, int B, int H,
                          int N, int d, void* hip_stream) {
  if (int rc = check_shape(B, H, N, d)) return rc;
  const size_t need = flashmask_workspace_bytes(FM_PASS_FWD, B, H, N, d);
  if (need > (size_t)FLASHMASK_NOALLOC_SCRATCH_BYTES) return FM_ERR_STATIC_LIMIT;
  void* ws = nullptr;
  if (hipError_t e = static_scratch(&ws); e != hipSuccess) return hip_fail(e);
  // every word of the scratch that a call reads it writes first (tables, work counts, queue records,
  // queue counters: the queue-building kernel clears them), so what the previous call left is harmless
  return fwd_impl(q, k, v, lts, lte, uts, ute, scale, out, lse, B, H, H, N, d, nullptr, ws,
                  FLASHMASK_NOALLOC_SCRATCH_BYTES, hip_stream);
}

int flashmask_fwd_ex(const void* q, const void* k, const void* v, const int32_t* lts, const int32_t* lte,
                     const int32_t* uts, const int32_t* ute, float scale, void* out, float* lse, int B, int H,
                     int H_kv, int N, int d, const flashmask_strides* sq, const flashmask_strides* sk,
                     const flashmask_strides* sv, const flashmask_strides* so, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
  if (int rc = check_shape(B, H, N, d)) return rc;
  if (H_kv <= 0 || H % H_kv != 0) return FM_ERR_SHAPE;
  if (int rc = check_strides(sq, B, H, N, d)) return rc;
  if (int rc = check_strides(sk, B, H_kv, N, d)) return rc;
  if (int rc = check_strides(sv, B, H_kv, N, d)) return rc;
  if (int rc = check_strides(so, B, H, N, d)) return rc;
  const FmStride st[4] = {to_kernel(*sq), to_kernel(*sk), to_kernel(*sv), to_kernel(*so)};
  return fwd_impl(q, k, v, lts, lte, uts, ute, scale, out, lse, B, H, H_kv, N, d, st, workspace, workspace_bytes,
                  hip_stream);
}

static int bwd_impl(const void* q, const void* k, const void* v, const void* out, const float* lse, const void* dout,
                    const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute, float scale,
                    void* dq, void* dk, void* dv, int B, int H, int Hk, int N, int d,
                    const FmStride* st /* q, k, v, out, dout, dq, dk, dv; NULL = contiguous, Hk == H */,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!q || !k || !v || !out || !lse || !dout || !lts || !lte || !uts || !ute || !dq || !dk || !dv) return FM_ERR_NULL;
  if (int rc = check_shape(B, H, N, d)) return rc;
  if (!(scale > 0.f) || !(scale < 3.0e38f)) return FM_ERR_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(dout) || misaligned(dq) ||
      misaligned(dk) || misaligned(dv) || misaligned(lts) || misaligned(lte) || misaligned(uts) || misaligned(ute) ||
      misaligned(lse))
    return FM_ERR_ALIGN;
  const size_t need = flashmask_workspace_bytes(FM_PASS_BWD, B, H, N, d);
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return FM_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)hip_stream;
  const int Np = padded_len(N);
  char* ws = (char*)workspace;
  mark(0, stream);
  hipError_t e;
  if (Np != N) {   // padded bound vectors first
    int* padded = (int*)ws;
    e = fm_launch_pad_bounds(lts, lte, uts, ute, B, N, Np, padded, stream);
    if (e != hipSuccess) return hip_fail(e);
    const size_t plane = (size_t)B * Np;
    lts = padded; lte = padded + plane; uts = padded + 2 * plane; ute = padded + 3 * plane;
    ws += padded_bounds_bytes(B, N);
  }
  const PassSpace sq = pass_space(B, H, Np, FM_DQ_BR, fm_dq_bc(d), true, 0);
  const PassSpace skv = pass_space(B, H, Np, FM_DKDV_BR, FM_DKDV_BC, false, sq.total);   // sized for H >= Hk heads
  FmBwdArgs a;
  a.q = q; a.k = k; a.v = v; a.out = out; a.dout = dout; a.lse = lse;
  a.lts = lts; a.lte = lte; a.uts = uts; a.ute = ute;
  a.minmax_dq = (int*)(ws + sq.minmax); a.order_dq = (int*)(ws + sq.order);
  a.minmax_dkdv = (int*)(ws + skv.minmax); a.order_dkdv = (int*)(ws + skv.order);
  a.dvec = (float*)(ws + skv.total);
  a.lse2 = (float*)(ws + skv.total + align_up((size_t)B * H * Np * 4, 256));
  a.dq = dq; a.dk = dk; a.dv = dv; a.scale = scale;
  a.B = B; a.H = H; a.N = N; a.Np = Np; a.d = d;
  a.slots_dq = fm_order_slots(B * H * (Np / FM_DQ_BR));
  a.slots_dkdv = fm_order_slots(B * Hk * (Np / FM_DKDV_BC));   // a dK/dV unit is (batch row, K/V head, key block)
  a.general = st != nullptr;
  a.Hk = Hk;
  if (st) {
    a.sq = st[0]; a.sk = st[1]; a.sv = st[2]; a.so = st[3]; a.sdo = st[4]; a.sdq = st[5]; a.sdk = st[6]; a.sdv = st[7];
  } else {
    a.sq = a.so = a.sdo = a.sdq = dense(H, N, d);
    a.sk = a.sv = a.sdk = a.sdv = dense(Hk, N, d);
  }
  const FmSetup rows{FM_DQ_BR, fm_dq_bc(d), (int*)(ws + sq.minmax), (int*)(ws + sq.work), (int*)(ws + sq.range),
                     (int*)(ws + sq.order)};
  const FmSetup cols{FM_DKDV_BR, FM_DKDV_BC, (int*)(ws + skv.minmax), (int*)(ws + skv.work), (int*)(ws + skv.range),
                     (int*)(ws + skv.order)};
  e = fm_launch_bwd_setup(lts, lte, uts, ute, B, H, Hk, Np, rows, cols, stream);
  if (e != hipSuccess) return hip_fail(e);
  mark(1, stream);
  // the dQ loop first: its prologue is also Algorithm 2's D pre-pass and leaves -D and the log2-domain
  // lse of every row in the workspace for the dK/dV loop
  e = fm_launch_bwd_dq(a, stream);
  if (e != hipSuccess) return hip_fail(e);
  mark(2, stream);
  e = fm_launch_bwd_dkdv(a, stream);
  if (e != hipSuccess) return hip_fail(e);
  mark(3, stream);
  return FM_OK;
}

int flashmask_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse, const void* dout,
                  const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute, float scale,
                  void* dq, void* dk, void* dv, int B, int H, int N, int d, void* workspace, size_t workspace_bytes,
                  void* hip_stream) {
  return bwd_impl(q, k, v, out, lse, dout, lts, lte, uts, ute, scale, dq, dk, dv, B, H, H, N, d, nullptr, workspace,
                  workspace_bytes, hip_stream);
}

int flashmask_bwd_ex(const void* q, const void* k, const void* v, const void* out, const float* lse, const void* dout,
                     const int32_t* lts, const int32_t* lte, const int32_t* uts, const int32_t* ute, float scale,
                     void* dq, void* dk, void* dv, int B, int H, int H_kv, int N, int d,
                     const flashmask_strides* strides, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (int rc = check_shape(B, H, N, d)) return rc;
  if (H_kv <= 0 || H % H_kv != 0) return FM_ERR_SHAPE;
  if (!strides) return FM_ERR_NULL;
  FmStride st[8];
  for (int t = 0; t < 8; ++t) {
    const bool kv = (t == 1 || t == 2 || t == 6 || t == 7);   // k, v, dk, dv have H_kv heads
    if (int rc = check_strides(strides + t, B, kv ? H_kv : H, N, d)) return rc;
    st[t] = to_kernel(strides[t]);
  }
  return bwd_impl(q, k, v, out, lse, dout, lts, lte, uts, ute, scale, dq, dk, dv, B, H, H_kv, N, d, st, workspace,
                  workspace_bytes, hip_stream);
}

}  // extern "C"
