// Host side of libmeft: argument validation, workspace layout and kernel launches behind the C ABI
// declared in include/meft.h.  Nothing here computes on the host; every step of the layer runs in
// the kernels of the headers included below.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/meft.h"
#include "common.h"
#include "gather.h"
#include "gemm_nt.h"
#include "scatter.h"
#include "select.h"

namespace meft {
namespace {

// ---- per-kernel timing ----------------------------------------------------------------------
struct ProfEntry {
  const char* name;
  hipEvent_t start, stop;
};
bool g_prof_on = false;
std::vector<ProfEntry> g_prof;

struct LaunchScope {
  hipStream_t st;
  bool on;
  hipEvent_t stop{};
  LaunchScope(const char* name, hipStream_t s) : st(s), on(g_prof_on) {
    if (!on) return;
    ProfEntry e{name, nullptr, nullptr};
    if (hipEventCreate(&e.start) != hipSuccess || hipEventCreate(&e.stop) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(e.start, st);
    stop = e.stop;
    g_prof.push_back(e);
  }
  ~LaunchScope() {
    if (on) (void)hipEventRecord(stop, st);
  }
};

#define MEFT_LAUNCH(name, kernel, grid, block, shmem, stream, ...)            \
  do {                                                                        \
    LaunchScope scope_(name, stream);                                         \
    hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);      \
  } while (0)

// ---- shape checks ---------------------------------------------------------------------------
constexpr int kMaxD = 16384, kMaxC = 12288, kMaxBlocks = 16384;

meft_status check_shape(const meft_shape* s) {
  if (!s) return MEFT_ERR_INVALID_ARG;
  if (s->T < 0 || s->d < 1 || s->n_blocks < 1 || s->block_size < 1 || s->N < 1) return MEFT_ERR_INVALID_ARG;
  if ((int64_t)s->n_blocks * s->block_size != (int64_t)s->N) return MEFT_ERR_INVALID_ARG;
  if (s->top_e < 1 || s->top_e > s->n_blocks) return MEFT_ERR_INVALID_ARG;
  const int64_t C = (int64_t)s->top_e * s->block_size;
  if (s->top_k < 1 || s->top_k > C) return MEFT_ERR_INVALID_ARG;
  if ((int64_t)s->T * s->top_k >= (1ll << 31) || (int64_t)s->T * C >= (1ll << 31)) return MEFT_ERR_INVALID_ARG;
  if (s->dtype != MEFT_F32 && s->dtype != MEFT_BF16) return MEFT_ERR_INVALID_ARG;
  if (s->activation != 0) return MEFT_ERR_INVALID_ARG;
  if (s->flags & ~(uint32_t)MEFT_FLAG_HOST_KV) return MEFT_ERR_INVALID_ARG;
  if (s->d % 8 != 0 || s->d > kMaxD || C > kMaxC || s->n_blocks > kMaxBlocks) return MEFT_ERR_UNSUPPORTED;
  if (s->flags & MEFT_FLAG_HOST_KV) return MEFT_ERR_UNSUPPORTED;
  return MEFT_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- workspace layout -----------------------------------------------------------------------
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <typename T>
  T* take(size_t n) {
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += (n * sizeof(T) + 255) & ~(size_t)255;
    return p;
  }
};

struct RouteWs {
  float* p;
  size_t bytes;
  RouteWs(const meft_shape& s, void* ws) {
    Carver c(ws);
    p = c.take<float>((size_t)s.T * s.n_blocks);
    bytes = c.off;
  }
};

struct FwdWs {
  int32_t *sblk, *cnt, *group_off, *tile_off, *perm;
  float* sc;
  size_t bytes;
  FwdWs(const meft_shape& s, void* ws) {
    Carver c(ws);
    const size_t n_ent = (size_t)s.T * s.top_e;
    sblk = c.take<int32_t>(n_ent);
    cnt = c.take<int32_t>(s.n_blocks);
    group_off = c.take<int32_t>((size_t)s.n_blocks + 1);
    tile_off = c.take<int32_t>((size_t)s.n_blocks + 1);
    perm = c.take<int32_t>(n_ent);
    sc = c.take<float>(n_ent * s.block_size);
    bytes = c.off;
  }
};

struct BwdWs {
  float* ds;
  int32_t *cnt, *cursor, *seg_off, *pair_list, *pair_sorted;
  size_t bytes;
  BwdWs(const meft_shape& s, void* ws) {
    Carver c(ws);
    const size_t P = (size_t)s.T * s.top_k;
    ds = c.take<float>(P);
    cnt = c.take<int32_t>(s.N);     // cnt and cursor are adjacent: cleared by one fill
    cursor = c.take<int32_t>(s.N);
    seg_off = c.take<int32_t>((size_t)s.N + 1);
    pair_list = c.take<int32_t>(P);
    pair_sorted = c.take<int32_t>(P);
    bytes = c.off;
  }
};

size_t workspace_bytes(const meft_shape& s) {
  const size_t a = RouteWs(s, nullptr).bytes, b = FwdWs(s, nullptr).bytes, c = BwdWs(s, nullptr).bytes;
  const size_t m = a > b ? (a > c ? a : c) : (b > c ? b : c);
  return m < 256 ? 256 : m;
}

// every entry point asks for the same size, the one meft_workspace_bytes() reports
meft_status check_ws(const meft_shape& s, const void* ws, size_t have) {
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || have < workspace_bytes(s)) return MEFT_ERR_WORKSPACE;
  return MEFT_OK;
}

meft_status launch_status() { return hipGetLastError() == hipSuccess ? MEFT_OK : MEFT_ERR_DEVICE; }

// threads per workgroup and 8-column groups per thread for the row kernels
void row_launch(int d, int& nthr, int& nv) {
  const int vecs = d / 8;
  nthr = vecs >= 256 ? 256 : ((vecs + 63) / 64) * 64;
  const int need = (vecs + nthr - 1) / nthr;
  nv = need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : 8;
}

void launch_gemm_nt(const meft_shape& s, const GemmNTArgs& a, int max_mtiles_bf16, int max_mtiles_f32,
                    const char* name, hipStream_t st) {
  if (s.dtype == MEFT_BF16) {
    dim3 grid(max_mtiles_bf16, (a.Ng + kGemmBN - 1) / kGemmBN);
    MEFT_LAUNCH(name, gemm_nt_bf16_kernel, grid, dim3(256), 0, st, a);
  } else {
    dim3 grid(max_mtiles_f32, (a.Ng + kGemmF32BN - 1) / kGemmF32BN);
    MEFT_LAUNCH(name, gemm_nt_f32_kernel, grid, dim3(256), 0, st, a);
  }
}

template <typename T>
void launch_gather_fwd(const meft_shape& s, const void* V, const int32_t* idx, const float* act, void* out,
                       hipStream_t st) {
  int nthr, nv;
  row_launch(s.d, nthr, nv);
  const T* v = static_cast<const T*>(V);
  T* o = static_cast<T*>(out);
#define GF(NV) MEFT_LAUNCH("gather_fwd", (gather_fwd_kernel<T, NV>), dim3(s.T), dim3(nthr), 0, st, v, idx, act, s.d, s.top_k, s.N, o)
  switch (nv) { case 1: GF(1); break; case 2: GF(2); break; case 4: GF(4); break; default: GF(8); }
#undef GF
}

template <typename T>
void launch_gather_bwd(const meft_shape& s, const void* K, const void* V, const void* dOut, const int32_t* idx,
                       const float* act, float* ds, void* dh, hipStream_t st) {
  int nthr, nv;
  row_launch(s.d, nthr, nv);
  const T *k = static_cast<const T*>(K), *v = static_cast<const T*>(V), *g = static_cast<const T*>(dOut);
  T* o = static_cast<T*>(dh);
#define GB(NV, PB) MEFT_LAUNCH("gather_bwd", (gather_bwd_kernel<T, NV, PB>), dim3(s.T), dim3(nthr), 0, st, k, v, g, idx, act, s.d, s.top_k, s.N, ds, o)
  switch (nv) { case 1: GB(1, 8); break; case 2: GB(2, 8); break; case 4: GB(4, 4); break; default: GB(8, 2); }
#undef GB
}

template <typename T>
void launch_seg_reduce(const meft_shape& s, const BwdWs& w, const int32_t* touched, const int32_t* n_touched,
                       const float* act, const void* h, const void* dOut, void* dK, void* dV, int grid,
                       hipStream_t st) {
  int nthr, nv;
  row_launch(s.d, nthr, nv);
  const T *hh = static_cast<const T*>(h), *g = static_cast<const T*>(dOut);
  T *pk = static_cast<T*>(dK), *pv = static_cast<T*>(dV);
#define SR(NV) MEFT_LAUNCH("seg_reduce", (seg_reduce_kernel<T, NV>), dim3(grid), dim3(nthr), 0, st, touched, n_touched, w.seg_off, w.pair_sorted, act, w.ds, hh, g, s.d, s.top_k, pk, pv)
  switch (nv) { case 1: SR(1); break; case 2: SR(2); break; case 4: SR(4); break; default: SR(8); }
#undef SR
}

}  // namespace
}  // namespace meft

using namespace meft;

extern "C" {

meft_status meft_check_shape(const meft_shape* shape) { return check_shape(shape); }

size_t meft_workspace_bytes(const meft_shape* shape) {
  if (check_shape(shape) != MEFT_OK) return 0;
  return workspace_bytes(*shape);
}

const char* meft_status_string(meft_status status) {
  switch (status) {
    case MEFT_OK: return "ok";
    case MEFT_ERR_INVALID_ARG: return "invalid argument";
    case MEFT_ERR_UNSUPPORTED: return "unsupported shape or flag";
    case MEFT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MEFT_ERR_DEVICE: return "device error";
  }
  return "unknown status";
}

meft_status meft_route(const meft_shape* shape, const void* h, const void* Wg, const float* bias,
                       int32_t* block_idx, float* block_score, void* ws, size_t ws_bytes, void* stream) {
  meft_status rc = check_shape(shape);
  if (rc != MEFT_OK) return rc;
  const meft_shape& s = *shape;
  if (!h || !Wg || !block_idx || !aligned16(h) || !aligned16(Wg)) return MEFT_ERR_INVALID_ARG;
  RouteWs w(s, ws);
  if ((rc = check_ws(s, ws, ws_bytes)) != MEFT_OK) return rc;
  if (s.T == 0) return MEFT_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);

  GemmNTArgs a{};
  a.A = h; a.Bm = Wg; a.C = w.p; a.perm = nullptr; a.group_off = nullptr; a.tile_off = nullptr;
  a.n_groups = 1; a.M = s.T; a.Ng = s.n_blocks; a.Kdim = s.d; a.lda = s.d; a.ldb = s.d; a.ldc = s.n_blocks;
  a.e = 1;
  launch_gemm_nt(s, a, (s.T + kGemmBM - 1) / kGemmBM, (s.T + kGemmF32BM - 1) / kGemmF32BM, "router_gemm", st);
  MEFT_LAUNCH("route_topk", route_topk_kernel, dim3(s.T), dim3(64), (size_t)s.n_blocks * 4, st, w.p, bias,
              s.n_blocks, s.top_e, block_idx, block_score);
  return launch_status();
}

meft_status meft_sparse_fwd(const meft_shape* shape, const void* h, const void* K, const void* V,
                            const int32_t* block_idx, void* out, int32_t* idx, float* act, void* ws,
                            size_t ws_bytes, void* stream) {
  meft_status rc = check_shape(shape);
  if (rc != MEFT_OK) return rc;
  const meft_shape& s = *shape;
  if (!h || !K || !V || !block_idx || !out || !idx || !act) return MEFT_ERR_INVALID_ARG;
  if (!aligned16(h) || !aligned16(K) || !aligned16(V) || !aligned16(out)) return MEFT_ERR_INVALID_ARG;
  FwdWs w(s, ws);
  if ((rc = check_ws(s, ws, ws_bytes)) != MEFT_OK) return rc;
  if (s.T == 0) return MEFT_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int n_ent = s.T * s.top_e;
  const int C = s.top_e * s.block_size;
  const int BM = s.dtype == MEFT_BF16 ? kGemmBM : kGemmF32BM;

  MEFT_LAUNCH("sort_blocks", sort_blocks_kernel, dim3((s.T + 255) / 256), dim3(256), 0, st, block_idx, s.T,
              s.top_e, s.n_blocks, w.sblk);
  MEFT_LAUNCH("count_blocks", count_blocks_kernel, dim3(s.n_blocks), dim3(256), 0, st, w.sblk, n_ent, w.cnt);
  MEFT_LAUNCH("fill_groups", fill_groups_kernel, dim3(s.n_blocks), dim3(256), 0, st, w.sblk, n_ent, w.cnt,
              s.n_blocks, BM, w.group_off, w.tile_off, w.perm);

  GemmNTArgs a{};
  a.A = h; a.Bm = K; a.C = w.sc; a.perm = w.perm; a.group_off = w.group_off; a.tile_off = w.tile_off;
  a.n_groups = s.n_blocks; a.M = 0; a.Ng = s.block_size; a.Kdim = s.d; a.lda = s.d; a.ldb = s.d;
  a.ldc = s.block_size; a.e = s.top_e;
  // upper bound on the number of m-tiles: every group may end with one partial tile
  const int nb_used = s.n_blocks < n_ent ? s.n_blocks : n_ent;
  launch_gemm_nt(s, a, n_ent / kGemmBM + nb_used, n_ent / kGemmF32BM + nb_used, "score_gemm", st);

  MEFT_LAUNCH("topk_select", topk_select_kernel, dim3(s.T), dim3(256), (size_t)C * 4, st, w.sc, w.sblk, C,
              s.block_size, s.top_e, s.top_k, idx, act);
  if (s.dtype == MEFT_BF16) launch_gather_fwd<bf16_t>(s, V, idx, act, out, st);
  else launch_gather_fwd<float>(s, V, idx, act, out, st);
  return launch_status();
}

meft_status meft_sparse_bwd(const meft_shape* shape, const void* h, const void* K, const void* V,
                            const int32_t* idx, const float* act, const void* dOut, void* dh, void* dK,
                            void* dV, int32_t* touched, int32_t* n_touched, void* ws, size_t ws_bytes,
                            void* stream) {
  meft_status rc = check_shape(shape);
  if (rc != MEFT_OK) return rc;
  const meft_shape& s = *shape;
  if (!h || !K || !V || !idx || !act || !dOut || !dK || !dV || !touched || !n_touched) return MEFT_ERR_INVALID_ARG;
  if (!aligned16(h) || !aligned16(K) || !aligned16(V) || !aligned16(dOut) || !aligned16(dK) || !aligned16(dV) ||
      (dh && !aligned16(dh)))
    return MEFT_ERR_INVALID_ARG;
  BwdWs w(s, ws);
  if ((rc = check_ws(s, ws, ws_bytes)) != MEFT_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (s.T == 0) {
    MEFT_LAUNCH("fill_i32", fill_i32_kernel, dim3(1), dim3(64), 0, st, n_touched, (size_t)1, 0);
    return launch_status();
  }
  const int P = s.T * s.top_k;

  if (s.dtype == MEFT_BF16) launch_gather_bwd<bf16_t>(s, K, V, dOut, idx, act, w.ds, dh, st);
  else launch_gather_bwd<float>(s, K, V, dOut, idx, act, w.ds, dh, st);

  const size_t n_clear = (size_t)(w.cursor - w.cnt) + s.N;  // cnt, its padding, cursor
  MEFT_LAUNCH("fill_i32", fill_i32_kernel, dim3((unsigned)((n_clear + 255) / 256)), dim3(256), 0, st, w.cnt,
              n_clear, 0);
  MEFT_LAUNCH("pair_count", pair_count_kernel, dim3((P + 255) / 256), dim3(256), 0, st, idx, P, s.N, w.cnt);
  MEFT_LAUNCH("pair_scan", pair_scan_kernel, dim3(1), dim3(1024), 0, st, w.cnt, s.N, w.seg_off, touched,
              n_touched);
  MEFT_LAUNCH("pair_fill", pair_fill_kernel, dim3((P + 255) / 256), dim3(256), 0, st, idx, P, s.N, w.seg_off,
              w.cursor, w.pair_list);
  const int n_seg = s.N < P ? s.N : P;  // upper bound on the number of touched neurons
  MEFT_LAUNCH("seg_sort", seg_sort_kernel, dim3(n_seg), dim3(256), 0, st, touched, n_touched, w.seg_off,
              w.pair_list, w.pair_sorted);
  if (s.dtype == MEFT_BF16) launch_seg_reduce<bf16_t>(s, w, touched, n_touched, act, h, dOut, dK, dV, n_seg, st);
  else launch_seg_reduce<float>(s, w, touched, n_touched, act, h, dOut, dK, dV, n_seg, st);
  return launch_status();
}

meft_status meft_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || !aligned16(dst) || !aligned16(src) || bytes % 16 != 0) return MEFT_ERR_INVALID_ARG;
  if (bytes == 0) return MEFT_OK;
  const size_t n = bytes / 16;
  MEFT_LAUNCH("probe_copy", probe_copy_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
              static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), n);
  return launch_status();
}

void meft_profile_enable(int on) {
  for (auto& e : g_prof) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  g_prof.clear();
  g_prof_on = on != 0;
}

int meft_profile_read(const char** names, int32_t* launches, float* total_ms, int cap) {
  int n = 0;
  for (auto& e : g_prof) {
    if (hipEventSynchronize(e.stop) != hipSuccess) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, e.start, e.stop) != hipSuccess) continue;
    int slot = -1;
    for (int i = 0; i < n; ++i)
      if (std::strcmp(names[i], e.name) == 0) { slot = i; break; }
    if (slot < 0) {
      if (n >= cap) continue;
      slot = n++;
      names[slot] = e.name;
      launches[slot] = 0;
      total_ms[slot] = 0.f;
    }
    launches[slot] += 1;
    total_ms[slot] += ms;
  }
  return n;
}

}  // extern "C"
