// Host side of libmeft: argument validation, workspace layout and kernel launches behind the C ABI
// declared in include/meft.h.  Nothing here computes on the host; every step of the layer runs in
// the kernels of the headers included below.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/meft.h"
#include "adam.h"
#include "common.h"
#include "dense_path.h"
#include "dispatch.h"
#include "gather.h"
#include "gemm_nt.h"
#include "scatter.h"
#include "select.h"
#include "small_groups.h"
#include "union_path.h"

// Device memory of meft_route_static: part of the library's image, one copy on every GPU the library runs on.  In
// host code this name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[MEFT_ROUTE_STATIC_BYTES];

namespace meft {
namespace {

// The host side of every entry point that enqueues work or touches the library's few pieces of process-wide state
// (the timing list, the side stream and events of the host-resident variant, the table of staged workspaces) runs
// under this lock, so the entry points may be called from several host threads.
std::mutex g_api_mutex;
#define MEFT_API_LOCK() std::lock_guard<std::mutex> api_lock_(g_api_mutex)

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
constexpr int kMaxD = 16384, kMaxBlocks = 16384;
constexpr int kMaxC = 1 << 22;      // candidates per token (top_e * block_size)
constexpr int kMaxLdsC = 12288;     // up to here the top-k selection keeps a token's keys in LDS

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
  if (s->flags & ~(uint32_t)(MEFT_FLAG_HOST_KV | MEFT_FLAG_KEEP_STAGED | MEFT_FLAG_PRESTAGED | MEFT_FLAG_REUSE_FWD))
    return MEFT_ERR_INVALID_ARG;
  if ((s->flags & (MEFT_FLAG_KEEP_STAGED | MEFT_FLAG_PRESTAGED)) && !(s->flags & MEFT_FLAG_HOST_KV))
    return MEFT_ERR_INVALID_ARG;
  if (s->d % 8 != 0 || s->d > kMaxD || C > kMaxC || s->n_blocks > kMaxBlocks) return MEFT_ERR_UNSUPPORTED;
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

// The matrix-core formulation (dense_path.h) is used for bf16 when the hidden size fits its k tiling and
// the selection is dense enough inside the chosen blocks; otherwise, and for fp32, the per-pair gather
// kernels are used.
// The score contraction alone runs on the matrix-core kernel of the block-dense path also for bf16 shapes that
// are not dense enough for the rest of it, when the groups are large enough to fill its 128-row tiles.
bool use_mfma_scores(const meft_shape& s) {
  return s.dtype == MEFT_BF16 && s.d % kTK == 0 && (int64_t)s.T * s.top_e >= (int64_t)128 * s.n_blocks;
}

bool use_dense(const meft_shape& s) {
  const int64_t C = (int64_t)s.top_e * s.block_size;
  return s.dtype == MEFT_BF16 && s.d % kTK == 0 && s.block_size >= 16 && (int64_t)s.top_k * 64 >= C &&
         C <= kMaxLdsC;
}

int round64(int v) { return (v + 63) & ~63; }
// Block-dense path: groups of at most this many tokens go to the per-pair kernels of small_groups.h (0: none).  The
// tile schedule knows the small groups only where it deals the groups out longest first.
// A contraction reads all block_size rows of the block for a group, the per-pair kernels about top_k / top_e rows for
// each of its tokens: at top_e * block_size / top_k tokens both move the same bytes, so the limit is no larger.
int small_rows_of(const meft_shape& s) {
  if (!use_dense(s) || s.n_blocks > kSchedSortMax) return 0;
  const int64_t even = (int64_t)s.top_e * s.block_size / s.top_k;   // >= 1: top_k <= top_e * block_size
  return (int)(even < kSmallRows ? even : kSmallRows);
}
// per XCD: at most n_blocks groups (+1 end entry) and, as a bound that needs no knowledge of the deal, all m tiles
int sched_cap(const meft_shape& s) { return s.n_blocks + 1; }
int sched_max_tiles(const meft_shape& s) { return (int)(((int64_t)s.T * s.top_e) / kTMTok + s.n_blocks); }
// bound of the tile ids of a launch with tn n tiles per m tile (ids beyond the real ones find no tile)
int tile_bound(const meft_shape& s, int tn) {
  const int64_t b = (int64_t)kXcd * sched_max_tiles(s) * tn;
  return (int)(b < (int64_t)INT32_MAX ? b : (int64_t)INT32_MAX);
}

constexpr int kRouterSplitMax = 4;

struct RouteWs {
  float* p;
  size_t bytes;
  RouteWs(const meft_shape& s, void* ws) {
    Carver c(ws);
    p = c.take<float>((size_t)kRouterSplitMax * s.T * s.n_blocks);
    bytes = c.off;
  }
};

// the three-pass dispatch (dispatch.h) covers up to 1024 blocks and 2^20 entries
bool fast_dispatch(const meft_shape& s) {
  const int64_t n_ent = (int64_t)s.T * s.top_e;
  return s.n_blocks <= kDispMaxBlocks && (n_ent + 1023) / 1024 <= kDispMaxChunks;
}

// index structures of the (token, block) dispatch, common to forward and backward
struct DispatchWs {
  int32_t* chunk_hist = nullptr;   // three-pass dispatch: [chunks][n_blocks]
  int32_t *sblk = nullptr, *cnt = nullptr, *group_off = nullptr, *tile_off = nullptr, *perm = nullptr,
          *tok_of_slot = nullptr, *slot_of_ent = nullptr, *sched_len = nullptr;
  int2* sched_pairs = nullptr;
  // the groups of at most small_rows_of(s) tokens and their entries (small_groups.h), and the two list lengths
  int2* small_ent = nullptr;
  int32_t *small_grp = nullptr, *small_cnt = nullptr;
  void carve(const meft_shape& s, Carver& c) {
    const size_t n_ent = (size_t)s.T * s.top_e;
    sblk = c.take<int32_t>(n_ent);
    cnt = c.take<int32_t>(s.n_blocks);
    group_off = c.take<int32_t>((size_t)s.n_blocks + 1);
    tile_off = c.take<int32_t>((size_t)s.n_blocks + 1);
    perm = c.take<int32_t>(n_ent);
    tok_of_slot = c.take<int32_t>(n_ent + kSlotPad);   // padded: see kSlotPad
    slot_of_ent = c.take<int32_t>(n_ent);
    sched_len = c.take<int32_t>(kSchedLenInts);   // list lengths per XCD, the split flag, lengths without small groups
    sched_pairs = c.take<int2>((size_t)kXcd * sched_cap(s));
    chunk_hist = c.take<int32_t>(fast_dispatch(s) ? ((n_ent + 1023) / 1024) * (size_t)s.n_blocks : 0);
    const size_t small = (size_t)small_rows_of(s);
    small_ent = c.take<int2>(small ? small * s.n_blocks : 0);
    small_grp = c.take<int32_t>(small ? (size_t)s.n_blocks : 0);
    small_cnt = c.take<int32_t>(small ? 2 : 0);
  }
};

// Block-dense path: what forward and backward both hold, at the same place in the workspace, so that a backward may
// take the forward's dispatch tables and activation rows as they are (MEFT_FLAG_REUSE_FWD).
struct DenseWs : DispatchWs {
  int32_t *flag = nullptr, *chunk_cnt = nullptr;
  uint16_t *zrow = nullptr, *Ap = nullptr, *DS = nullptr, *part = nullptr;
  float* ds32 = nullptr;   // activation gradients of the pairs of small groups, [T, top_k]
  void carve_dense(const meft_shape& s, Carver& c) {
    carve(s, c);
    const size_t n_ent = (size_t)s.T * s.top_e;
    chunk_cnt = c.take<int32_t>((size_t)(s.N + kFlagChunk - 1) / kFlagChunk);
    flag = c.take<int32_t>(s.N);                               // flag and zrow adjacent: cleared by one fill
    // one piece: the row of zeros, A', DS', each row bsp elements, so that the zero row is row -1 of A' and row
    // -(n_ent + 1) of DS'
    const size_t bsp = round64(s.block_size);
    zrow = c.take<uint16_t>(bsp * (1 + 2 * n_ent));
    Ap = zrow ? zrow + bsp : nullptr;
    DS = zrow ? Ap + n_ent * bsp : nullptr;
    part = c.take<uint16_t>(n_ent * s.d);   // per-entry partial rows [T*e, d] bf16
    ds32 = c.take<float>((size_t)s.T * s.top_k);
  }
};

struct FwdWs : DenseWs {
  float* sc;
  size_t bytes;
  FwdWs(const meft_shape& s, void* ws) {
    Carver c(ws);
    if (use_dense(s)) carve_dense(s, c);
    else carve(s, c);
    sc = c.take<float>((size_t)s.T * s.top_e * s.block_size);
    bytes = c.off;
  }
};

// upper bound of the chunks of neurons with more than one chunk: such a neuron has more than kSegChunk pairs, so its
// ceil(L / kSegChunk) chunks are fewer than 2 L / kSegChunk
size_t seg_multi_chunks(const meft_shape& s) { return 2 * (((size_t)s.T * s.top_k) / kSegChunk) + 1; }

struct BwdWs : DenseWs {
  // gather path
  float* ds;
  int32_t *cnt_n, *cursor, *seg_off, *pair_list, *pair_sorted, *work_off, *multi_off;
  float* seg_part;   // fp32 chunk sums of the neurons with more than kSegChunk pairs: [chunk][dV | dK][d]
  size_t bytes;
  BwdWs(const meft_shape& s, void* ws) {
    Carver c(ws);
    const size_t P = (size_t)s.T * s.top_k;
    ds = nullptr; cnt_n = cursor = seg_off = pair_list = pair_sorted = work_off = multi_off = nullptr; seg_part = nullptr;
    if (use_dense(s)) {
      carve_dense(s, c);
    } else {
      ds = c.take<float>(P);
      cnt_n = c.take<int32_t>(s.N);     // cnt_n and cursor are adjacent: cleared by one fill
      cursor = c.take<int32_t>(s.N);
      seg_off = c.take<int32_t>((size_t)s.N + 1);
      pair_list = c.take<int32_t>(P);
      pair_sorted = c.take<int32_t>(P);
      const size_t n_seg = (size_t)s.N < P ? (size_t)s.N : P;
      work_off = c.take<int32_t>(n_seg + 1);
      multi_off = c.take<int32_t>(n_seg + 1);
      seg_part = c.take<float>(seg_multi_chunks(s) * 2 * (size_t)s.d);
    }
    bytes = c.off;
  }
};

size_t compute_bytes(const meft_shape& s) {
  const size_t a = RouteWs(s, nullptr).bytes, b = FwdWs(s, nullptr).bytes, c = BwdWs(s, nullptr).bytes;
  const size_t m = a > b ? (a > c ? a : c) : (b > c ? b : c);
  return m < 256 ? 256 : m;
}

// With MEFT_FLAG_HOST_KV the workspace also holds device copies of K, V and device staging for dK, dV.
struct HostKvWs {
  char *Kd, *Vd, *dKd, *dVd;
  int32_t *pair_blk, *pair_blk_cnt;   // backward: block of every pair, pairs per block
  size_t bytes;
  HostKvWs(const meft_shape& s, void* ws) {
    Carver c(ws);
    c.off = compute_bytes(s);
    const size_t row_bytes = (size_t)s.d * (s.dtype == MEFT_BF16 ? 2 : 4);
    Kd = c.take<char>((size_t)s.N * row_bytes);
    Vd = c.take<char>((size_t)s.N * row_bytes);
    dKd = c.take<char>((size_t)s.N * row_bytes);
    dVd = c.take<char>((size_t)s.N * row_bytes);
    pair_blk = c.take<int32_t>((size_t)s.T * s.top_k);
    pair_blk_cnt = c.take<int32_t>(s.n_blocks);
    bytes = c.off;
  }
};

size_t workspace_bytes(const meft_shape& s) {
  return (s.flags & MEFT_FLAG_HOST_KV) ? HostKvWs(s, nullptr).bytes : compute_bytes(s);
}

// ---- host-resident keys/values: side stream, events, pinned read-back buffer (created on first use) ----
struct HostKvState {
  hipStream_t side = nullptr;
  hipEvent_t ev_entry = nullptr, ev_cnt = nullptr, ev_k = nullptr, ev_v = nullptr;
  int32_t* host_cnt = nullptr;
  bool ready = false;
};
HostKvState g_hkv;

bool hostkv_init() {
  if (g_hkv.ready) return true;
  if (hipStreamCreateWithFlags(&g_hkv.side, hipStreamNonBlocking) != hipSuccess) return false;
  hipEvent_t* evs[4] = {&g_hkv.ev_entry, &g_hkv.ev_cnt, &g_hkv.ev_k, &g_hkv.ev_v};
  for (hipEvent_t* e : evs)
    if (hipEventCreateWithFlags(e, hipEventDisableTiming) != hipSuccess) return false;
  if (hipHostMalloc(reinterpret_cast<void**>(&g_hkv.host_cnt), (size_t)kMaxBlocks * sizeof(int32_t), hipHostMallocDefault) !=
      hipSuccess)
    return false;
  g_hkv.ready = true;
  return true;
}

// Workspaces whose K, V copies were requested ahead of their forward (meft_hostkv_stage), each with the events
// that follow its K and its V copies.
struct StageSlot {
  const void* ws = nullptr;
  hipEvent_t ev_k = nullptr, ev_v = nullptr;
};
constexpr int kStageSlots = 16;
StageSlot g_slots[kStageSlots];
int g_slot_next = 0;

StageSlot* stage_slot(const void* ws, bool create) {
  for (StageSlot& sl : g_slots)
    if (sl.ws == ws) return &sl;
  if (!create) return nullptr;
  StageSlot& sl = g_slots[g_slot_next];
  g_slot_next = (g_slot_next + 1) % kStageSlots;
  if (!sl.ev_k && hipEventCreateWithFlags(&sl.ev_k, hipEventDisableTiming) != hipSuccess) return nullptr;
  if (!sl.ev_v && hipEventCreateWithFlags(&sl.ev_v, hipEventDisableTiming) != hipSuccess) return nullptr;
  sl.ws = ws;
  return &sl;
}

// Reads the per-block entry counts back (the host blocks until the work queued on `st` so far has produced them),
// then copies the blocks that some token uses from the pinned host matrices to their device copies on the side
// stream: `first` before `second`, each followed by its event.
meft_status hostkv_fetch(const meft_shape& s, const int32_t* cnt_dev, const void* first_host, char* first_dev,
                         hipEvent_t first_ev, const void* second_host, char* second_dev, hipEvent_t second_ev,
                         hipStream_t st) {
  HostKvState& k = g_hkv;
  if (hipMemcpyAsync(k.host_cnt, cnt_dev, (size_t)s.n_blocks * sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
    return MEFT_ERR_DEVICE;
  if (hipEventRecord(k.ev_cnt, st) != hipSuccess || hipEventSynchronize(k.ev_cnt) != hipSuccess) return MEFT_ERR_DEVICE;
  const size_t block_bytes = (size_t)s.block_size * s.d * (s.dtype == MEFT_BF16 ? 2 : 4);
  const void* host[2] = {first_host, second_host};
  char* dev[2] = {first_dev, second_dev};
  hipEvent_t ev[2] = {first_ev, second_ev};
  for (int m = 0; m < 2; ++m) {
    for (int b = 0; b < s.n_blocks; ++b) {
      if (k.host_cnt[b] <= 0) continue;
      if (hipMemcpyAsync(dev[m] + (size_t)b * block_bytes, static_cast<const char*>(host[m]) + (size_t)b * block_bytes,
                         block_bytes, hipMemcpyHostToDevice, k.side) != hipSuccess)
        return MEFT_ERR_DEVICE;
    }
    if (hipEventRecord(ev[m], k.side) != hipSuccess) return MEFT_ERR_DEVICE;
  }
  return MEFT_OK;
}

// ---- batch-union variant: virtual blocks over the compacted rows --------------------------------
struct UnionGeom {
  int cap;        // capacity of S: min(N, T*top_k)
  int vbs, nvb;   // rows per virtual block, number of virtual blocks (nvb * vbs >= cap)
  meft_shape vs;  // the shape the grouped GEMMs see: nvb blocks of vbs rows, every token in every block
};

// false: the variant is not available for this shape (it runs on the bf16 matrix-core kernels only)
bool union_geom(const meft_shape& s, UnionGeom& g) {
  if (s.dtype != MEFT_BF16 || s.d % kTK != 0 || (s.flags & MEFT_FLAG_HOST_KV)) return false;
  const int64_t cap = (int64_t)s.T * s.top_k < (int64_t)s.N ? (int64_t)s.T * s.top_k : (int64_t)s.N;
  g.cap = (int)(cap < 1 ? 1 : cap);
  g.vbs = g.cap >= 1024 ? 1024 : round64(g.cap);
  g.nvb = (g.cap + g.vbs - 1) / g.vbs;
  if (g.nvb > 4096 || (int64_t)g.nvb * (s.T > 0 ? s.T : 1) > ((int64_t)1 << 30)) return false;
  g.vs = s;
  g.vs.n_blocks = g.nvb; g.vs.block_size = g.vbs; g.vs.N = g.nvb * g.vbs; g.vs.top_e = g.nvb; g.vs.top_k = 1;
  return true;
}

struct UnionWs : DispatchWs {
  int32_t *flag, *chunk_cnt, *rowflag;
  uint16_t *Kc, *Vc, *dKc, *dVc, *zrow, *Ap, *DS, *part;
  size_t bytes;
  UnionWs(const meft_shape& s, const UnionGeom& g, void* ws) {
    Carver c(ws);
    carve(g.vs, c);
    const size_t n_ent = (size_t)s.T * g.nvb, rows = (size_t)g.nvb * g.vbs;
    chunk_cnt = c.take<int32_t>((size_t)(s.N + kFlagChunk - 1) / kFlagChunk);
    flag = c.take<int32_t>(s.N);
    rowflag = c.take<int32_t>(rows);
    Kc = c.take<uint16_t>(rows * s.d);
    Vc = c.take<uint16_t>(rows * s.d);
    dKc = c.take<uint16_t>(rows * s.d);
    dVc = c.take<uint16_t>(rows * s.d);
    zrow = c.take<uint16_t>((size_t)g.vbs * (1 + 2 * n_ent));   // one piece: row of zeros, A', DS' (see BwdWs)
    Ap = zrow ? zrow + g.vbs : nullptr;
    DS = zrow ? Ap + n_ent * g.vbs : nullptr;
    part = c.take<uint16_t>(n_ent * s.d);
    bytes = c.off < 256 ? 256 : c.off;
  }
};

// every entry point asks for the same size, the one meft_workspace_bytes() reports
meft_status check_ws(const meft_shape& s, const void* ws, size_t have) {
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || have < workspace_bytes(s)) return MEFT_ERR_WORKSPACE;
  return MEFT_OK;
}

thread_local hipError_t g_last_device_error = hipSuccess;   // what the last MEFT_ERR_DEVICE of this thread was
meft_status launch_status() {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return MEFT_OK;
  g_last_device_error = e;
  return MEFT_ERR_DEVICE;
}
// The runtime keeps the last error of the thread until it is read: an entry point reads it away before its first
// launch, so that MEFT_ERR_DEVICE reports this call's own launches and not a failure some other code left behind.
void clear_stale_error() { (void)hipGetLastError(); }

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
  // one workgroup per chunk: at most one chunk per touched neuron plus one per kSegChunk pairs
  const int64_t work = (int64_t)grid + ((int64_t)s.T * s.top_k) / kSegChunk;
  const int finish = grid < 4096 ? grid : 4096;
#define SR(NV)                                                                                                        \
  do {                                                                                                                \
    MEFT_LAUNCH("seg_reduce", (seg_reduce_kernel<T, NV>), dim3((unsigned)work), dim3(nthr), 0, st, touched, n_touched, \
                w.seg_off, w.work_off, w.multi_off, w.pair_sorted, act, w.ds, hh, g, s.d, s.top_k, pk, pv, w.seg_part); \
    MEFT_LAUNCH("seg_finish", (seg_finish_kernel<T, NV>), dim3(finish), dim3(nthr), 0, st, touched, n_touched,        \
                w.work_off, w.multi_off, w.seg_part, s.d, pk, pv);                                                     \
  } while (0)
  switch (nv) { case 1: SR(1); break; case 2: SR(2); break; case 4: SR(4); break; default: SR(8); }
#undef SR
}


constexpr int kPersistentWgs = 256;   // compute units of an MI355X; a multiple of the 8 XCDs

// Bytes readable from an operand's lowest address; buffer loads (32-bit offsets) where both fit.  Setting
// MEFT_GLOBAL_LOADS=1 in the environment selects the global-load kernels (those for operands of 4 GB and more)
// at any size, so that tests reach them with small inputs.
// (the environment is read once, when the library is loaded; meft_debug_global_loads overrides it)
std::atomic<int> g_force_global_loads{[] {
  const char* env = getenv("MEFT_GLOBAL_LOADS");
  return (env && env[0] == '1') ? 1 : 0;
}()};

template <class P>
void set_gemm_extents(P& p, uint64_t a_bytes, uint64_t b_bytes) {
  constexpr uint64_t kLimit = 0xFFFF0000ull;
  const bool forced_global = g_force_global_loads.load(std::memory_order_relaxed) != 0;
  p.buf = !forced_global && a_bytes < kLimit && b_bytes < kLimit;
  p.a_bytes = p.buf ? (uint32_t)a_bytes : 0u;
  p.b_bytes = p.buf ? (uint32_t)b_bytes : 0u;
}

template <class P>
void launch_gemm_mfma(const char* name, const P& prob, int grid, hipStream_t st) {
  static std::once_flag configured;  // raise the dynamic LDS limit of both instantiations once
  std::call_once(configured, [] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<P, false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, gemm_lds_bytes<P>());
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<P, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, gemm_lds_bytes<P>());
  });
  // persistent workgroups: one per compute unit (the LDS footprint allows no more), each walking the tile ids
  // wg, wg + 256, ... below `grid`
  const int launch = grid < kPersistentWgs ? grid : kPersistentWgs;
  if (prob.buf) {
    MEFT_LAUNCH(name, (gemm_mfma_kernel<P, true>), dim3(launch), dim3(gemm_threads<P>()), gemm_lds_bytes<P>(), st, prob, grid);
  } else {
    MEFT_LAUNCH(name, (gemm_mfma_kernel<P, false>), dim3(launch), dim3(gemm_threads<P>()), gemm_lds_bytes<P>(), st, prob, grid);
  }
}

// (token, block) dispatch from sorted per-token block lists: groups, slot maps, XCD tile schedule
void launch_dispatch(const meft_shape& s, const DispatchWs& w, int BM, bool dense, bool want_sched, hipStream_t st) {
  const int n_ent = s.T * s.top_e;
  const int small = dense ? small_rows_of(s) : 0;
  if (fast_dispatch(s)) {
    const int n_chunks = (n_ent + 1023) / 1024;
    const size_t lds = (size_t)16 * s.n_blocks * sizeof(int);
    MEFT_LAUNCH("dispatch_count", dispatch_count_kernel, dim3(n_chunks), dim3(1024), lds, st, w.sblk, n_ent,
                s.n_blocks, w.chunk_hist);
    MEFT_LAUNCH("dispatch_scan", dispatch_scan_kernel, dim3(1), dim3(1024), 0, st, w.chunk_hist, n_chunks,
                s.n_blocks, BM, w.cnt, w.group_off, w.tile_off, sched_cap(s), want_sched ? w.sched_pairs : nullptr,
                w.sched_len, kTMTok, small, small ? w.small_ent : nullptr, w.small_grp, w.small_cnt);
    MEFT_LAUNCH("dispatch_place", dispatch_place_kernel, dim3(n_chunks), dim3(1024), lds, st, w.sblk, n_ent,
                s.n_blocks, s.top_e, w.chunk_hist, w.group_off, w.perm, dense ? w.tok_of_slot : nullptr,
                w.slot_of_ent, kSlotPad);
    return;
  }
  MEFT_LAUNCH("count_blocks", count_blocks_kernel, dim3(s.n_blocks), dim3(1024), 0, st, w.sblk, n_ent, w.cnt);
  MEFT_LAUNCH("fill_groups", fill_groups_kernel, dim3(s.n_blocks), dim3(1024), 0, st, w.sblk, n_ent, w.cnt,
              s.n_blocks, BM, w.group_off, w.tile_off, w.perm);
  if (dense) {
    MEFT_LAUNCH("slot_maps", slot_maps_kernel, dim3((n_ent + kSlotPad + 255) / 256), dim3(256), 0, st, w.perm, w.group_off,
                s.n_blocks, s.top_e, w.tok_of_slot, w.slot_of_ent);
  }
  if (want_sched) {
    MEFT_LAUNCH("build_sched", build_sched_kernel, dim3(1), dim3(1024), 0, st, w.group_off, s.n_blocks,
                sched_cap(s), w.sched_pairs, w.sched_len, kTMTok, small);
  }
  if (small) {
    MEFT_LAUNCH("small_lists", small_lists_kernel, dim3(1), dim3(1024), 0, st, w.group_off, s.n_blocks, small,
                w.small_ent, w.small_grp, w.small_cnt);
  }
}

void launch_reduce_parts(const meft_shape& s, const uint16_t* part, const DispatchWs& w, void* out, hipStream_t st) {
  int nthr, nv;
  row_launch(s.d, nthr, nv);
  uint16_t* o = static_cast<uint16_t*>(out);
#define RP(NV) MEFT_LAUNCH("reduce_parts", (reduce_parts_kernel<NV>), dim3(s.T), dim3(nthr), 0, st, part, w.sblk, w.slot_of_ent, s.d, s.top_e, o)
  switch (nv) { case 1: RP(1); break; case 2: RP(2); break; case 4: RP(4); break; default: RP(8); }
#undef RP
}

size_t small_list_bytes(const meft_shape& s) {
  return (size_t)s.top_k * sizeof(int);   // top_k <= top_e * block_size <= 12288 on the block-dense path
}

// Launch widths of the kernels that walk the lists of small groups: enough workgroups for the lists of a skewed
// batch to be taken in one pass, few enough that a launch on a batch without small groups costs next to nothing.
constexpr int kSmallEntGrid = 1024, kSmallGrpGrid = 128;

// small groups: their rows of `part` as sums of coef * W rows (forward: act and V; backward: ds and K)
void launch_small_rowsum(const char* name, const meft_shape& s, const DenseWs& w, const void* W, const int32_t* idx,
                         const float* coef, hipStream_t st) {
  const int small = small_rows_of(s);
  if (small == 0) return;
  const int gx = s.n_blocks * small < kSmallEntGrid ? s.n_blocks * small : kSmallEntGrid;
  MEFT_LAUNCH(name, small_rowsum_kernel, dim3(gx, (s.d + kSmallCols - 1) / kSmallCols), dim3(256),
              small_list_bytes(s), st, static_cast<const bf16_t*>(W), idx, coef, w.small_ent, w.small_cnt,
              w.tok_of_slot, s.d, s.top_k, s.N, s.block_size, reinterpret_cast<bf16_t*>(w.part));
}

// backward, small groups: the activation gradients of their pairs
void launch_small_ds(const meft_shape& s, const DenseWs& w, const void* V, const void* dOut, const int32_t* idx,
                     const float* act, hipStream_t st) {
  const int small = small_rows_of(s);
  if (small == 0) return;
  const int gx = s.n_blocks * small < kSmallEntGrid ? s.n_blocks * small : kSmallEntGrid;
  MEFT_LAUNCH("small_ds", small_ds_kernel, dim3(gx, kSmallPairSplit), dim3(256), small_list_bytes(s), st,
              static_cast<const bf16_t*>(V), static_cast<const bf16_t*>(dOut), idx, act, w.small_ent, w.small_cnt,
              w.tok_of_slot, s.d, s.top_k, s.N, s.block_size, w.ds32);
}

// backward, small groups: the dV and dK rows of their blocks
void launch_small_dvdk(const meft_shape& s, const DenseWs& w, const void* h, const void* dOut, const int32_t* idx,
                       const float* act, void* dK, void* dV, hipStream_t st) {
  if (small_rows_of(s) == 0) return;
  const int gx = s.n_blocks < kSmallGrpGrid ? s.n_blocks : kSmallGrpGrid;
  MEFT_LAUNCH("small_dvdk", small_dvdk_kernel, dim3((s.block_size + kSmallRowChunk - 1) / kSmallRowChunk, gx),
              dim3(256), 0, st, static_cast<const bf16_t*>(h), static_cast<const bf16_t*>(dOut), idx, act, w.ds32,
              w.small_grp, w.small_cnt, w.group_off, w.tok_of_slot, s.d, s.top_k, s.N, s.block_size,
              static_cast<bf16_t*>(dK), static_cast<bf16_t*>(dV));
}

// Tile rows of the dV / dK contractions: 256 where that computes no more padded rows of the block than 128 would
int neu_tile_rows(int block_rows) {
  return kTMNeuW == 256 && (block_rows + 255) / 256 * 256 == (block_rows + 127) / 128 * 128 ? 256 : 128;
}

// One weight-gradient contraction (dV: A = A', X = dOut; dK: A = DS', X = h) over the groups of a tile schedule
struct NeuArgs {
  const uint16_t* A; int zrow; const uint16_t* X; uint16_t* G;
  const int32_t *group_off, *tok_of_slot, *flag;
  TokenSched sched;
  int big_only, n_groups, bs, bsp, d;
  uint64_t a_bytes, x_bytes;   // bytes readable from the lowest address of either operand
};

template <int TM>
void launch_neu_tm(const char* name, const NeuArgs& a, hipStream_t st) {
  ProbNeuTN<TM> pn{};
  pn.A = a.A; pn.zrow = a.zrow; pn.X = a.X; pn.G = a.G;
  pn.group_off = a.group_off; pn.tok_of_slot = a.tok_of_slot; pn.flag = a.flag;
  pn.sched = a.sched; pn.big_only = a.big_only; pn.bs = a.bs; pn.bsp = a.bsp; pn.d = a.d;
  set_gemm_extents(pn, a.a_bytes, a.x_bytes);
  // every listed group has the same tiles; in the worst case one XCD holds all groups
  const int64_t tiles = (int64_t)kXcd * a.n_groups * ((a.bs + TM - 1) / TM) * ((a.d + kTN - 1) / kTN);
  launch_gemm_mfma(name, pn, (int)(tiles < (int64_t)INT32_MAX ? tiles : (int64_t)INT32_MAX), st);
}

void launch_neu(const char* name, const NeuArgs& a, hipStream_t st) {
  if (neu_tile_rows(a.bs) == 256) launch_neu_tm<256>(name, a, st);
  else launch_neu_tm<128>(name, a, st);
}

}  // namespace
}  // namespace meft

using namespace meft;

// Router scores (as up to kRouterSplitMax partial sums over slices of the hidden dimension, in `p`) and the top-e
// selection over their sum.
static meft_status route_impl(const meft_shape& s, const void* h, const void* Wg, const float* bias,
                              int32_t* block_idx, float* block_score, float* p, hipStream_t st) {
  int n_part = 1;
  if (s.dtype == MEFT_BF16 && s.d % kTK == 0) {
    const int kt = s.d / kTK;
    n_part = kt % 4 == 0 ? 4 : (kt % 2 == 0 ? 2 : 1);
    ProbRouter pr{static_cast<const uint16_t*>(h), static_cast<const uint16_t*>(Wg), p, s.T, s.d, s.n_blocks, n_part};
    set_gemm_extents(pr, (uint64_t)s.T * s.d * 2, (uint64_t)s.n_blocks * s.d * 2);
    launch_gemm_mfma("router_gemm", pr, n_part * ((s.T + ProbRouter::kTM - 1) / ProbRouter::kTM) * ((s.n_blocks + kTN - 1) / kTN), st);
  } else {
    GemmNTArgs a{};
    a.A = h; a.Bm = Wg; a.C = p; a.perm = nullptr; a.group_off = nullptr; a.tile_off = nullptr;
    a.n_groups = 1; a.M = s.T; a.Ng = s.n_blocks; a.Kdim = s.d; a.lda = s.d; a.ldb = s.d; a.ldc = s.n_blocks;
    a.e = 1;
    launch_gemm_nt(s, a, (s.T + kGemmBM - 1) / kGemmBM, (s.T + kGemmF32BM - 1) / kGemmF32BM, "router_gemm", st);
  }
  MEFT_LAUNCH("route_topk", route_topk_kernel, dim3(s.T), dim3(64), (size_t)s.n_blocks * 4, st, p, n_part,
              (size_t)s.T * s.n_blocks, bias,
              s.n_blocks, s.top_e, block_idx, block_score);
  return launch_status();
}

// Forward on device-resident K, V.  wait_k / wait_v (may be null): events the stream must wait for before
// the first kernel that reads K / V (used when they are being staged from host memory).
static meft_status fwd_impl(const meft_shape& s, const void* h, const void* K, const void* V,
                            const int32_t* block_idx, void* out, int32_t* idx, float* act, const FwdWs& w,
                            hipStream_t st, hipEvent_t wait_k, hipEvent_t wait_v) {
  const int n_ent = s.T * s.top_e;
  const int C = s.top_e * s.block_size;
  const int BM = s.dtype == MEFT_BF16 ? kGemmBM : kGemmF32BM;

  const bool dense = use_dense(s);
  MEFT_LAUNCH("sort_blocks", sort_blocks_kernel, dim3((s.T + 255) / 256), dim3(256), 0, st, block_idx, s.T,
              s.top_e, s.n_blocks, w.sblk);
  const bool mfma_scores = dense || use_mfma_scores(s);
  launch_dispatch(s, w, BM, dense, mfma_scores, st);
  const int bsp = round64(s.block_size);
  const TokenSched sched{w.sched_pairs, w.sched_len, sched_cap(s), sched_max_tiles(s)};
  const uint16_t *hh = static_cast<const uint16_t*>(h), *kk = static_cast<const uint16_t*>(K),
                 *vv = static_cast<const uint16_t*>(V);
  if (wait_k && hipStreamWaitEvent(st, wait_k, 0) != hipSuccess) return MEFT_ERR_DEVICE;
  if (mfma_scores) {
    ProbTokKC<kTokScores> ps{};
    ps.X = hh; ps.W = kk; ps.perm = w.perm; ps.group_off = w.group_off; ps.sched = sched;
    ps.e = s.top_e; ps.bs = s.block_size; ps.bsp = bsp; ps.d = s.d; ps.sc = w.sc;
    set_gemm_extents(ps, (uint64_t)s.T * s.d * 2, (uint64_t)s.N * s.d * 2);
    launch_gemm_mfma("score_gemm", ps, tile_bound(s, (s.block_size + kTN - 1) / kTN), st);
  } else {
    GemmNTArgs a{};
    a.A = h; a.Bm = K; a.C = w.sc; a.perm = w.perm; a.group_off = w.group_off; a.tile_off = w.tile_off;
    a.n_groups = s.n_blocks; a.M = 0; a.Ng = s.block_size; a.Kdim = s.d; a.lda = s.d; a.ldb = s.d;
    a.ldc = s.block_size; a.e = s.top_e;
    // upper bound on the number of m-tiles: every group may end with one partial tile
    const int nb_used = s.n_blocks < n_ent ? s.n_blocks : n_ent;
    launch_gemm_nt(s, a, n_ent / kGemmBM + nb_used, n_ent / kGemmF32BM + nb_used, "score_gemm", st);
  }
  if (C <= kMaxLdsC) {
    // keys in registers, the smallest per-thread count that covers the C candidates with 256 threads
    uint16_t* ap = dense ? w.Ap : nullptr;
#define TK2(KPT, FULL) MEFT_LAUNCH("topk_select", (topk_select_reg_kernel<KPT, FULL>), dim3(s.T), dim3(256), 0, st, w.sc, w.sblk, C, s.block_size, s.top_e, s.top_k, idx, act, w.slot_of_ent, bsp, ap)
#define TK(KPT) do { if (C == 256 * (KPT)) TK2(KPT, true); else TK2(KPT, false); } while (0)
    if (C <= 256 * 4) TK(4);
    else if (C <= 256 * 8) TK(8);
    else if (C <= 256 * 16) TK(16);
    else if (C <= 256 * 32) TK(32);
    else TK(48);
#undef TK
#undef TK2
  }
  else if (C <= 1024 * 64) {
    // e.g. one block holding every neuron: 1024 threads per token, still with the keys in registers
#define TK(KPT) MEFT_LAUNCH("topk_select_big", (topk_select_reg1024_kernel<KPT>), dim3(s.T), dim3(1024), 0, st, w.sc, w.sblk, C, s.block_size, s.top_e, s.top_k, idx, act)
    if (C <= 1024 * 16) TK(16);
    else if (C <= 1024 * 32) TK(32);
    else TK(64);
#undef TK
  } else {   // beyond that the keys stay in global memory and are read once per pass
    MEFT_LAUNCH("topk_select_big", topk_select_big_kernel, dim3(s.T), dim3(1024), 0, st, w.sc, w.sblk, C,
                s.block_size, s.top_e, s.top_k, idx, act);
  }
  // (also when only the selection is wanted: a backward that reuses the staged copies relies on this wait)
  if (wait_v && hipStreamWaitEvent(st, wait_v, 0) != hipSuccess) return MEFT_ERR_DEVICE;
  if (!out) return launch_status();   // selection only
  if (dense) {
    ProbTokNC pv{};
    pv.A = w.Ap; pv.W = vv; pv.group_off = w.group_off; pv.sched = sched; pv.bs = s.block_size; pv.bsp = bsp;
    pv.d = s.d; pv.part = w.part; pv.big_only = small_rows_of(s) > 0;
    set_gemm_extents(pv, (uint64_t)n_ent * bsp * 2, (uint64_t)s.N * s.d * 2);
    launch_gemm_mfma("value_gemm", pv, tile_bound(s, (s.d + kTN - 1) / kTN), st);
    launch_small_rowsum("small_value", s, w, V, idx, act, st);
    launch_reduce_parts(s, w.part, w, out, st);
  } else if (s.dtype == MEFT_BF16) {
    launch_gather_fwd<bf16_t>(s, V, idx, act, out, st);
  } else {
    launch_gather_fwd<float>(s, V, idx, act, out, st);
  }
  return launch_status();
}

// Backward on device-resident K, V, dK, dV.  wait_v / wait_k as in fwd_impl.
static meft_status bwd_impl(const meft_shape& s, const void* h, const void* K, const void* V, const int32_t* idx,
                            const float* act, const void* dOut, void* dh, void* dK, void* dV, int32_t* touched,
                            int32_t* n_touched, const BwdWs& w, hipStream_t st, hipEvent_t wait_k,
                            hipEvent_t wait_v) {
  const int P = s.T * s.top_k;

  if (use_dense(s)) {
    const int bsp = round64(s.block_size);
    const uint16_t *hh = static_cast<const uint16_t*>(h), *kk = static_cast<const uint16_t*>(K),
                   *vv = static_cast<const uint16_t*>(V), *gg = static_cast<const uint16_t*>(dOut);
    // With MEFT_FLAG_REUSE_FWD the dispatch tables and the activation rows A' are the ones the forward of this step
    // left in the workspace; otherwise they are rebuilt from (idx, act).
    const bool reuse = (s.flags & MEFT_FLAG_REUSE_FWD) != 0;
    if (!reuse) {
      MEFT_LAUNCH("blocks_from_idx", blocks_from_idx_kernel, dim3(s.T), dim3(64), (size_t)((s.n_blocks + 31) / 32) * 4,
                  st, idx, s.top_k, s.N, s.block_size, s.n_blocks, s.top_e, w.sblk);
      launch_dispatch(s, w, kGemmBM, true, true, st);
    }
    // the flags and the row of zeros start from zero (adjacent in the workspace); 4-byte fill
    const size_t clear_words = (size_t)(reinterpret_cast<char*>(w.Ap) - reinterpret_cast<char*>(w.flag)) / 4;
    MEFT_LAUNCH("fill_i32", fill_i32_kernel, dim3((unsigned)((clear_words + 255) / 256)), dim3(256), 0, st, w.flag,
                clear_words, 0);
    if (reuse) {
      MEFT_LAUNCH("mark_idx", mark_idx_kernel, dim3((P + 255) / 256), dim3(256), 0, st, idx, P, s.N, w.flag);
    } else {
      // a token's rows take top_e * bsp * 2 bytes of LDS: up to 96 KB where blocks are small and many (the default
      // limit of a launch is 64 KB)
      static std::once_flag act_rows_configured;
      std::call_once(act_rows_configured, [] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&act_rows_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kMaxLdsC * 2);
      });
      MEFT_LAUNCH("act_rows", act_rows_kernel, dim3(s.T), dim3(256), (size_t)s.top_e * bsp * 2, st, idx, act, s.top_k,
                  s.N, s.block_size, bsp, s.top_e, w.sblk, w.slot_of_ent, w.Ap, w.flag);
    }
    const int n_chunks = (s.N + kFlagChunk - 1) / kFlagChunk;
    MEFT_LAUNCH("count_flags", count_flags_kernel, dim3(n_chunks), dim3(256), 0, st, w.flag, s.N, w.chunk_cnt);
    MEFT_LAUNCH("compact_flags", compact_flags_kernel, dim3(n_chunks), dim3(256), 0, st, w.flag, s.N, w.chunk_cnt,
                touched, n_touched);
    const TokenSched sched{w.sched_pairs, w.sched_len, sched_cap(s), sched_max_tiles(s)};
    const int big_only = small_rows_of(s) > 0;   // the small groups: launch_small_* below
    const int n_ent = s.T * s.top_e;
    NeuArgs pn{};
    pn.group_off = w.group_off; pn.tok_of_slot = w.tok_of_slot; pn.flag = w.flag;
    pn.sched = sched; pn.big_only = big_only; pn.n_groups = s.n_blocks; pn.bs = s.block_size; pn.bsp = bsp; pn.d = s.d;
    pn.a_bytes = (uint64_t)(1 + 2 * (uint64_t)n_ent) * bsp * 2; pn.x_bytes = (uint64_t)s.T * s.d * 2;
    // dV first: it needs neither K nor V (so it also runs while host-resident K, V are still on their way), and it
    // gathers the same dOut rows as the activation-gradient GEMM that follows it
    pn.A = w.Ap; pn.zrow = -1; pn.X = gg; pn.G = static_cast<uint16_t*>(dV);
    launch_neu("dV_gemm", pn, st);
    if (wait_v && hipStreamWaitEvent(st, wait_v, 0) != hipSuccess) return MEFT_ERR_DEVICE;
    ProbTokKC<kTokMasked> pg{};
    pg.X = gg; pg.W = vv; pg.perm = w.perm; pg.group_off = w.group_off; pg.sched = sched;
    pg.e = s.top_e; pg.bs = s.block_size; pg.bsp = bsp; pg.d = s.d; pg.Ap = w.Ap; pg.DS = w.DS;
    pg.big_only = big_only;
    set_gemm_extents(pg, (uint64_t)s.T * s.d * 2, (uint64_t)s.N * s.d * 2);
    launch_gemm_mfma("dact_gemm", pg, tile_bound(s, (s.block_size + kTN - 1) / kTN), st);
    if (wait_k && hipStreamWaitEvent(st, wait_k, 0) != hipSuccess) return MEFT_ERR_DEVICE;
    launch_small_ds(s, w, V, dOut, idx, act, st);
    if (dh) {
      ProbTokNC ph{};
      ph.A = w.DS; ph.W = kk; ph.group_off = w.group_off; ph.sched = sched; ph.bs = s.block_size; ph.bsp = bsp;
      ph.d = s.d; ph.part = w.part; ph.big_only = big_only;
      set_gemm_extents(ph, (uint64_t)n_ent * bsp * 2, (uint64_t)s.N * s.d * 2);
      launch_gemm_mfma("dh_gemm", ph, tile_bound(s, (s.d + kTN - 1) / kTN), st);
      launch_small_rowsum("small_dh", s, w, K, idx, w.ds32, st);
      launch_reduce_parts(s, w.part, w, dh, st);
    }
    pn.A = w.DS; pn.zrow = -(n_ent + 1); pn.X = hh; pn.G = static_cast<uint16_t*>(dK);
    launch_neu("dK_gemm", pn, st);
    launch_small_dvdk(s, w, h, dOut, idx, act, dK, dV, st);
    return launch_status();
  }

  if (wait_v && hipStreamWaitEvent(st, wait_v, 0) != hipSuccess) return MEFT_ERR_DEVICE;
  if (wait_k && hipStreamWaitEvent(st, wait_k, 0) != hipSuccess) return MEFT_ERR_DEVICE;
  if (s.dtype == MEFT_BF16) launch_gather_bwd<bf16_t>(s, K, V, dOut, idx, act, w.ds, dh, st);
  else launch_gather_bwd<float>(s, K, V, dOut, idx, act, w.ds, dh, st);

  const size_t n_clear = (size_t)(w.cursor - w.cnt_n) + s.N;  // cnt, its padding, cursor
  MEFT_LAUNCH("fill_i32", fill_i32_kernel, dim3((unsigned)((n_clear + 255) / 256)), dim3(256), 0, st, w.cnt_n,
              n_clear, 0);
  MEFT_LAUNCH("pair_count", pair_count_kernel, dim3((P + 255) / 256), dim3(256), 0, st, idx, P, s.N, w.cnt_n);
  MEFT_LAUNCH("pair_scan", pair_scan_kernel, dim3(1), dim3(1024), 0, st, w.cnt_n, s.N, w.seg_off, touched,
              n_touched, w.work_off, w.multi_off);
  MEFT_LAUNCH("pair_fill", pair_fill_kernel, dim3((P + 255) / 256), dim3(256), 0, st, idx, P, s.N, w.seg_off,
              w.cursor, w.pair_list);
  const int n_seg = s.N < P ? s.N : P;  // upper bound on the number of touched neurons
  MEFT_LAUNCH("seg_sort", seg_sort_kernel, dim3(n_seg), dim3(256), 0, st, touched, n_touched, w.seg_off,
              w.pair_list, w.pair_sorted);
  if (s.dtype == MEFT_BF16) launch_seg_reduce<bf16_t>(s, w, touched, n_touched, act, h, dOut, dK, dV, n_seg, st);
  else launch_seg_reduce<float>(s, w, touched, n_touched, act, h, dOut, dK, dV, n_seg, st);
  return launch_status();
}

// Shared front part of the batch-union forward and backward: index structure from n_S, tile schedule, compacted
// K and V, and A' = ReLU(h K[S]^T).
static void union_front(const meft_shape& s, const UnionGeom& g, const UnionWs& w, const void* h, const void* K,
                        const void* V, const int32_t* S, const int32_t* n_S, hipStream_t st) {
  const size_t n_slots = (size_t)g.nvb * s.T, n_rows = (size_t)g.nvb * g.vbs;
  const size_t n_thr = (n_slots + kSlotPad) > n_rows ? (n_slots + kSlotPad) : n_rows;
  MEFT_LAUNCH("union_maps", union_maps_kernel, dim3((unsigned)((n_thr + 255) / 256)), dim3(256), 0, st, n_S, g.cap,
              s.T, g.vbs, g.nvb, w.sblk, w.perm, w.tok_of_slot, w.slot_of_ent, w.group_off, w.rowflag);
  MEFT_LAUNCH("build_sched", build_sched_kernel, dim3(1), dim3(1024), 0, st, w.group_off, g.nvb, sched_cap(g.vs),
              w.sched_pairs, w.sched_len, kTMTok, 0);
  // the row of zeros that pads the contraction over tokens in the weight-gradient GEMMs (vbs % 64 == 0)
  MEFT_LAUNCH("fill_i32", fill_i32_kernel, dim3((g.vbs / 2 + 255) / 256), dim3(256), 0, st,
              reinterpret_cast<int32_t*>(w.zrow), (size_t)g.vbs / 2, 0);
  const int rows_grid = (int)(n_rows < 4096 ? n_rows : 4096);
  MEFT_LAUNCH("gather_rows", gather_rows_kernel, dim3(rows_grid), dim3(256), 0, st, static_cast<const uint16_t*>(K),
              S, n_S, g.cap, s.N, s.d, g.vbs, w.Kc);
  MEFT_LAUNCH("gather_rows", gather_rows_kernel, dim3(rows_grid), dim3(256), 0, st, static_cast<const uint16_t*>(V),
              S, n_S, g.cap, s.N, s.d, g.vbs, w.Vc);
  const TokenSched sched{w.sched_pairs, w.sched_len, sched_cap(g.vs), sched_max_tiles(g.vs)};
  ProbTokKC<kTokRelu> pr{};
  pr.X = static_cast<const uint16_t*>(h); pr.W = w.Kc; pr.perm = w.perm; pr.group_off = w.group_off;
  pr.sched = sched; pr.e = g.nvb; pr.bs = g.vbs; pr.bsp = g.vbs; pr.d = s.d;
  pr.DS = w.Ap;
  set_gemm_extents(pr, (uint64_t)s.T * s.d * 2, (uint64_t)n_rows * s.d * 2);
  launch_gemm_mfma("union_score_gemm", pr, tile_bound(g.vs, (g.vbs + kTN - 1) / kTN), st);
}

extern "C" {

size_t meft_union_workspace_bytes(const meft_shape* shape) {
  UnionGeom g;
  if (check_shape(shape) != MEFT_OK || !union_geom(*shape, g)) return 0;
  return UnionWs(*shape, g, nullptr).bytes;
}

meft_status meft_union_fwd(const meft_shape* shape, const void* h, const void* K, const void* V, const int32_t* idx,
                           void* out, int32_t* S, int32_t* n_S, void* ws, size_t ws_bytes, void* stream) {
  meft_status rc = check_shape(shape);
  if (rc != MEFT_OK) return rc;
  const meft_shape& s = *shape;
  UnionGeom g;
  if (!union_geom(s, g)) return MEFT_ERR_UNSUPPORTED;
  if (!h || !K || !V || !idx || !out || !S || !n_S) return MEFT_ERR_INVALID_ARG;
  if (!aligned16(h) || !aligned16(K) || !aligned16(V) || !aligned16(out)) return MEFT_ERR_INVALID_ARG;
  const UnionWs w(s, g, ws);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < w.bytes) return MEFT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  MEFT_API_LOCK();
  clear_stale_error();
  if (s.T == 0) {
    MEFT_LAUNCH("fill_i32", fill_i32_kernel, dim3(1), dim3(64), 0, st, n_S, (size_t)1, 0);
    return launch_status();
  }
  // S = ascending ids of the neurons that some token selected
  const int P = s.T * s.top_k;
  MEFT_LAUNCH("fill_i32", fill_i32_kernel, dim3((unsigned)(((size_t)s.N + 255) / 256)), dim3(256), 0, st, w.flag,
              (size_t)s.N, 0);
  MEFT_LAUNCH("mark_idx", mark_idx_kernel, dim3((P + 255) / 256), dim3(256), 0, st, idx, P, s.N, w.flag);
  const int n_chunks = (s.N + kFlagChunk - 1) / kFlagChunk;
  MEFT_LAUNCH("count_flags", count_flags_kernel, dim3(n_chunks), dim3(256), 0, st, w.flag, s.N, w.chunk_cnt);
  MEFT_LAUNCH("compact_flags", compact_flags_kernel, dim3(n_chunks), dim3(256), 0, st, w.flag, s.N, w.chunk_cnt, S,
              n_S);
  union_front(s, g, w, h, K, V, S, n_S, st);
  const TokenSched sched{w.sched_pairs, w.sched_len, sched_cap(g.vs), sched_max_tiles(g.vs)};
  ProbTokNC pv{};
  pv.A = w.Ap; pv.W = w.Vc; pv.group_off = w.group_off; pv.sched = sched; pv.bs = g.vbs; pv.bsp = g.vbs;
  pv.d = s.d; pv.part = w.part;
  set_gemm_extents(pv, (uint64_t)s.T * g.nvb * g.vbs * 2, (uint64_t)g.nvb * g.vbs * s.d * 2);
  launch_gemm_mfma("union_value_gemm", pv, tile_bound(g.vs, (s.d + kTN - 1) / kTN), st);
  launch_reduce_parts(g.vs, w.part, w, out, st);
  return launch_status();
}

meft_status meft_union_bwd(const meft_shape* shape, const void* h, const void* K, const void* V, const int32_t* S,
                           const int32_t* n_S, const void* dOut, void* dh, void* dK, void* dV, void* ws,
                           size_t ws_bytes, void* stream) {
  meft_status rc = check_shape(shape);
  if (rc != MEFT_OK) return rc;
  const meft_shape& s = *shape;
  UnionGeom g;
  if (!union_geom(s, g)) return MEFT_ERR_UNSUPPORTED;
  if (!h || !K || !V || !S || !n_S || !dOut || !dK || !dV) return MEFT_ERR_INVALID_ARG;
  if (!aligned16(h) || !aligned16(K) || !aligned16(V) || !aligned16(dOut) || !aligned16(dK) || !aligned16(dV) ||
      (dh && !aligned16(dh)))
    return MEFT_ERR_INVALID_ARG;
  const UnionWs w(s, g, ws);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < w.bytes) return MEFT_ERR_WORKSPACE;
  if (s.T == 0) return MEFT_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  MEFT_API_LOCK();
  clear_stale_error();
  union_front(s, g, w, h, K, V, S, n_S, st);
  const TokenSched sched{w.sched_pairs, w.sched_len, sched_cap(g.vs), sched_max_tiles(g.vs)};
  const uint16_t *hh = static_cast<const uint16_t*>(h), *gg = static_cast<const uint16_t*>(dOut);
  ProbTokKC<kTokMasked> pg{};
  pg.X = gg; pg.W = w.Vc; pg.perm = w.perm; pg.group_off = w.group_off; pg.sched = sched;
  pg.e = g.nvb; pg.bs = g.vbs; pg.bsp = g.vbs; pg.d = s.d; pg.Ap = w.Ap; pg.DS = w.DS;
  set_gemm_extents(pg, (uint64_t)s.T * s.d * 2, (uint64_t)g.nvb * g.vbs * s.d * 2);
  launch_gemm_mfma("union_dact_gemm", pg, tile_bound(g.vs, (g.vbs + kTN - 1) / kTN), st);
  if (dh) {
    ProbTokNC ph{};
    ph.A = w.DS; ph.W = w.Kc; ph.group_off = w.group_off; ph.sched = sched; ph.bs = g.vbs; ph.bsp = g.vbs;
    ph.d = s.d; ph.part = w.part;
    set_gemm_extents(ph, (uint64_t)s.T * g.nvb * g.vbs * 2, (uint64_t)g.nvb * g.vbs * s.d * 2);
    launch_gemm_mfma("union_dh_gemm", ph, tile_bound(g.vs, (s.d + kTN - 1) / kTN), st);
    launch_reduce_parts(g.vs, w.part, w, dh, st);
  }
  NeuArgs pn{};
  pn.group_off = w.group_off; pn.tok_of_slot = w.tok_of_slot; pn.flag = w.rowflag;
  pn.sched = sched; pn.big_only = 0; pn.n_groups = g.nvb; pn.bs = g.vbs; pn.bsp = g.vbs; pn.d = s.d;
  pn.a_bytes = (1 + 2 * (uint64_t)s.T * g.nvb) * g.vbs * 2; pn.x_bytes = (uint64_t)s.T * s.d * 2;
  pn.A = w.Ap; pn.zrow = -1; pn.X = gg; pn.G = w.dVc;
  launch_neu("union_dV_gemm", pn, st);
  pn.A = w.DS; pn.zrow = -(s.T * g.nvb + 1); pn.X = hh; pn.G = w.dKc;
  launch_neu("union_dK_gemm", pn, st);
  const int rows_grid = g.cap < 4096 ? g.cap : 4096;
  MEFT_LAUNCH("scatter_rows", scatter_rows_kernel, dim3(rows_grid), dim3(256), 0, st, w.dVc, S, n_S, s.N, s.d, g.cap,
              static_cast<uint16_t*>(dV));
  MEFT_LAUNCH("scatter_rows", scatter_rows_kernel, dim3(rows_grid), dim3(256), 0, st, w.dKc, S, n_S, s.N, s.d, g.cap,
              static_cast<uint16_t*>(dK));
  return launch_status();
}

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
  MEFT_API_LOCK();
  clear_stale_error();
  return route_impl(s, h, Wg, bias, block_idx, block_score, w.p, st);
}

// Address of `scratch` on the current device, looked up on the first call with that device current.
static float* static_scratch_ptr() {
  constexpr int kMaxDevices = 64;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    ptr[dev] = p;
  }
  return static_cast<float*>(ptr[dev]);
}

meft_status meft_route_static(const meft_shape* shape, const void* h, const void* Wg, const float* bias,
                              int32_t* block_idx, float* block_score, void* stream) {
  meft_status rc = check_shape(shape);
  if (rc != MEFT_OK) return rc;
  const meft_shape& s = *shape;
  if (!h || !Wg || !block_idx || !aligned16(h) || !aligned16(Wg)) return MEFT_ERR_INVALID_ARG;
  if (RouteWs(s, nullptr).bytes > MEFT_ROUTE_STATIC_BYTES) return MEFT_ERR_WORKSPACE;
  if (s.T == 0) return MEFT_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  MEFT_API_LOCK();
  clear_stale_error();
  float* p = static_scratch_ptr();
  if (!p) { (void)launch_status(); return MEFT_ERR_DEVICE; }
  const bool timing = g_prof_on;   // per-kernel timing creates events: off inside this call
  g_prof_on = false;
  rc = route_impl(s, h, Wg, bias, block_idx, block_score, p, st);
  g_prof_on = timing;
  return rc;
}

meft_status meft_sparse_fwd(const meft_shape* shape, const void* h, const void* K, const void* V,
                            const int32_t* block_idx, void* out, int32_t* idx, float* act, void* ws,
                            size_t ws_bytes, void* stream) {
  meft_status rc = check_shape(shape);
  if (rc != MEFT_OK) return rc;
  const meft_shape& s = *shape;
  if (!h || !K || !V || !block_idx || !idx || !act) return MEFT_ERR_INVALID_ARG;
  if (!aligned16(h) || !aligned16(K) || !aligned16(V) || (out && !aligned16(out))) return MEFT_ERR_INVALID_ARG;
  FwdWs w(s, ws);
  if ((rc = check_ws(s, ws, ws_bytes)) != MEFT_OK) return rc;
  if (s.T == 0) return MEFT_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  MEFT_API_LOCK();
  clear_stale_error();
  if (!(s.flags & MEFT_FLAG_HOST_KV)) return fwd_impl(s, h, K, V, block_idx, out, idx, act, w, st, nullptr, nullptr);

  // K, V in pinned host memory: find the blocks in use, fetch them on the side stream (K first, then V) while
  // the dispatch runs, and let the scoring wait for K and the value stage for V.
  if (!hostkv_init()) return MEFT_ERR_DEVICE;
  HostKvWs hw(s, ws);
  if (s.flags & MEFT_FLAG_PRESTAGED) {   // the copies were requested by meft_hostkv_stage
    StageSlot* sl = stage_slot(ws, false);
    if (!sl) return MEFT_ERR_INVALID_ARG;
    sl->ws = nullptr;   // one stage call serves one forward
    return fwd_impl(s, h, hw.Kd, hw.Vd, block_idx, out, idx, act, w, st, sl->ev_k, sl->ev_v);
  }
  if (hipEventRecord(g_hkv.ev_entry, st) != hipSuccess || hipStreamWaitEvent(g_hkv.side, g_hkv.ev_entry, 0) != hipSuccess)
    return MEFT_ERR_DEVICE;   // the device copies may still be read by work queued earlier on this stream
  MEFT_LAUNCH("sort_blocks", sort_blocks_kernel, dim3((s.T + 255) / 256), dim3(256), 0, st, block_idx, s.T,
              s.top_e, s.n_blocks, w.sblk);
  MEFT_LAUNCH("count_blocks", count_blocks_kernel, dim3(s.n_blocks), dim3(1024), 0, st, w.sblk, s.T * s.top_e, w.cnt);
  if ((rc = hostkv_fetch(s, w.cnt, K, hw.Kd, g_hkv.ev_k, V, hw.Vd, g_hkv.ev_v, st)) != MEFT_OK) return rc;
  return fwd_impl(s, h, hw.Kd, hw.Vd, block_idx, out, idx, act, w, st, g_hkv.ev_k, g_hkv.ev_v);
}

meft_status meft_hostkv_stage(const meft_shape* shape, const int32_t* block_idx, const void* K, const void* V, void* ws,
                              size_t ws_bytes, void* stream) {
  meft_status rc = check_shape(shape);
  if (rc != MEFT_OK) return rc;
  const meft_shape& s = *shape;
  if (!(s.flags & MEFT_FLAG_HOST_KV) || !block_idx || !K || !V || !aligned16(K) || !aligned16(V)) return MEFT_ERR_INVALID_ARG;
  FwdWs w(s, ws);
  if ((rc = check_ws(s, ws, ws_bytes)) != MEFT_OK) return rc;
  if (s.T == 0) return MEFT_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  MEFT_API_LOCK();
  clear_stale_error();
  if (!hostkv_init()) return MEFT_ERR_DEVICE;
  HostKvWs hw(s, ws);
  StageSlot* sl = stage_slot(ws, true);
  if (!sl) return MEFT_ERR_DEVICE;
  if (hipEventRecord(g_hkv.ev_entry, st) != hipSuccess || hipStreamWaitEvent(g_hkv.side, g_hkv.ev_entry, 0) != hipSuccess)
    return MEFT_ERR_DEVICE;   // the device copies may still be read by work queued earlier on this stream
  MEFT_LAUNCH("sort_blocks", sort_blocks_kernel, dim3((s.T + 255) / 256), dim3(256), 0, st, block_idx, s.T,
              s.top_e, s.n_blocks, w.sblk);
  MEFT_LAUNCH("count_blocks", count_blocks_kernel, dim3(s.n_blocks), dim3(1024), 0, st, w.sblk, s.T * s.top_e, w.cnt);
  if ((rc = hostkv_fetch(s, w.cnt, K, hw.Kd, sl->ev_k, V, hw.Vd, sl->ev_v, st)) != MEFT_OK) return rc;
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
  MEFT_API_LOCK();
  clear_stale_error();
  if (s.T == 0) {
    MEFT_LAUNCH("fill_i32", fill_i32_kernel, dim3(1), dim3(64), 0, st, n_touched, (size_t)1, 0);
    return launch_status();
  }
  if (!(s.flags & MEFT_FLAG_HOST_KV))
    return bwd_impl(s, h, K, V, idx, act, dOut, dh, dK, dV, touched, n_touched, w, st, nullptr, nullptr);

  // K, V, dK, dV in pinned host memory: fetch the blocks that hold a selected neuron (V first: the activation
  // gradient needs it before dh needs K), compute into device staging, then write the touched rows back.
  if (!hostkv_init()) return MEFT_ERR_DEVICE;
  HostKvWs hw(s, ws);
  if (s.flags & MEFT_FLAG_KEEP_STAGED) {
    // the forward of this step left the blocks in use in the workspace, and its copies are ordered before
    // anything enqueued here (the forward made `st` wait for them)
    rc = bwd_impl(s, h, hw.Kd, hw.Vd, idx, act, dOut, dh, hw.dKd, hw.dVd, touched, n_touched, w, st, nullptr, nullptr);
  } else {
  if (hipEventRecord(g_hkv.ev_entry, st) != hipSuccess || hipStreamWaitEvent(g_hkv.side, g_hkv.ev_entry, 0) != hipSuccess)
    return MEFT_ERR_DEVICE;
  int32_t* sblk_tmp = hw.pair_blk;
  int32_t* cnt_tmp = hw.pair_blk_cnt;
  MEFT_LAUNCH("blocks_of_pairs", blocks_of_pairs_kernel, dim3((s.T * s.top_k + 255) / 256), dim3(256), 0, st, idx,
              s.T * s.top_k, s.N, s.block_size, sblk_tmp);
  MEFT_LAUNCH("count_blocks", count_blocks_kernel, dim3(s.n_blocks), dim3(1024), 0, st, sblk_tmp, s.T * s.top_k,
              cnt_tmp);
  if ((rc = hostkv_fetch(s, cnt_tmp, V, hw.Vd, g_hkv.ev_v, K, hw.Kd, g_hkv.ev_k, st)) != MEFT_OK) return rc;
  rc = bwd_impl(s, h, hw.Kd, hw.Vd, idx, act, dOut, dh, hw.dKd, hw.dVd, touched, n_touched, w, st, g_hkv.ev_k,
                g_hkv.ev_v);
  }
  if (rc != MEFT_OK) return rc;
  const int n_rows = s.N < s.T * s.top_k ? s.N : s.T * s.top_k;
  const int vec = s.d * (s.dtype == MEFT_BF16 ? 2 : 4) / 16;
  MEFT_LAUNCH("rows_to_host", rows_to_host_kernel, dim3(n_rows), dim3(256), 0, st, touched, n_touched,
              reinterpret_cast<const u32x4*>(hw.dVd), reinterpret_cast<u32x4*>(dV), vec);
  MEFT_LAUNCH("rows_to_host", rows_to_host_kernel, dim3(n_rows), dim3(256), 0, st, touched, n_touched,
              reinterpret_cast<const u32x4*>(hw.dKd), reinterpret_cast<u32x4*>(dK), vec);
  return launch_status();
}

meft_status meft_adam_rows(const meft_shape* shape, const meft_adam* hp, void* W, const void* G, float* m,
                           float* v, float* master, const int32_t* touched, const int32_t* n_touched,
                           void* stream) {
  const meft_status cs = check_shape(shape);
  if (cs != MEFT_OK) return cs;
  const meft_shape& s = *shape;
  if (s.flags & MEFT_FLAG_HOST_KV) return MEFT_ERR_UNSUPPORTED;   // the kernel reads and writes device memory
  if (!hp || !W || !G || !m || !v || !touched || !n_touched) return MEFT_ERR_INVALID_ARG;
  if (!aligned16(W) || !aligned16(G) || !aligned16(m) || !aligned16(v) || (master && !aligned16(master)))
    return MEFT_ERR_INVALID_ARG;
  if (hp->step < 1 || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) ||
      !(hp->eps >= 0.f) || !(hp->lr == hp->lr))
    return MEFT_ERR_INVALID_ARG;
  if (s.T == 0) return MEFT_OK;
  AdamScalars a;
  const double b1 = hp->beta1, b2 = hp->beta2;
  a.lr = hp->lr; a.b1 = hp->beta1; a.b2 = hp->beta2; a.eps = hp->eps;
  a.omb1 = (float)(1.0 - b1); a.omb2 = (float)(1.0 - b2);
  a.inv_c1 = (float)(1.0 / (1.0 - std::pow(b1, (double)hp->step)));
  a.inv_c2 = (float)(1.0 / (1.0 - std::pow(b2, (double)hp->step)));
  const int64_t cap = (int64_t)s.T * s.top_k < (int64_t)s.N ? (int64_t)s.T * s.top_k : (int64_t)s.N;
  const int grid = (int)(cap < 4096 ? cap : 4096);   // rows are walked with a grid stride
  hipStream_t st = static_cast<hipStream_t>(stream);
  MEFT_API_LOCK();
  clear_stale_error();
  if (s.dtype == MEFT_BF16)
    MEFT_LAUNCH("adam_rows", adam_rows_kernel<bf16_t>, dim3(grid), dim3(256), 0, st, static_cast<bf16_t*>(W),
                static_cast<const bf16_t*>(G), m, v, master, touched, n_touched, s.N, s.d, a);
  else
    MEFT_LAUNCH("adam_rows", adam_rows_kernel<float>, dim3(grid), dim3(256), 0, st, static_cast<float*>(W),
                static_cast<const float*>(G), m, v, master, touched, n_touched, s.N, s.d, a);
  return launch_status();
}

meft_status meft_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || !aligned16(dst) || !aligned16(src) || bytes % 16 != 0) return MEFT_ERR_INVALID_ARG;
  if (bytes == 0) return MEFT_OK;
  const size_t n = bytes / 16;
  MEFT_API_LOCK();
  clear_stale_error();
  MEFT_LAUNCH("probe_copy", probe_copy_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
              static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), n);
  return launch_status();
}

meft_status meft_probe_mfma(float* out, int workgroups, int iters, void* stream) {
  if (!out || workgroups < 1 || workgroups > 65536 || iters < 1) return MEFT_ERR_INVALID_ARG;
  MEFT_API_LOCK();
  clear_stale_error();
  MEFT_LAUNCH("probe_mfma", probe_mfma_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), out,
              iters);
  return launch_status();
}

const char* meft_last_device_error(void) { return hipGetErrorString(g_last_device_error); }

void meft_debug_global_loads(int on) { g_force_global_loads.store(on ? 1 : 0, std::memory_order_relaxed); }

void meft_profile_enable(int on) {
  MEFT_API_LOCK();
  for (auto& e : g_prof) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  g_prof.clear();
  g_prof_on = on != 0;
}

int meft_profile_read(const char** names, int32_t* launches, float* total_ms, int cap) {
  MEFT_API_LOCK();
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
