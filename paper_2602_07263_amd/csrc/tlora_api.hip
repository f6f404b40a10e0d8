// Host side of the C ABI: argument validation, the nano-batch plan (integer bookkeeping), workspace
// layout and the launch sequence of the forward and backward passes.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <list>
#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <utility>
#include <vector>

#include "../../include/tlora.h"
#include "tlora_internal.h"
#include "tlora_kernels.h"

// Device memory of tlora_fwd_noalloc: the forward's workspace for callers that cannot allocate.  Every GPU the
// library runs on holds its own copy of this array at its own address until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress: the address that kernels and fills get is the per-device pointer
// looked up below, never the name.
static __device__ __align__(256) unsigned char scratch[TLORA_NOALLOC_SCRATCH_BYTES];

namespace tlora {
namespace {

constexpr int kMaxDevices = 64;
// What the HIP runtime said when a call last failed (for tlora_last_hip_error): the code and the line of this file.
int g_hip_err = 0, g_hip_line = 0;
inline int hip_failed(hipError_t e, int line) {
  g_hip_err = (int)e;  g_hip_line = line;
  return TLORA_EHIP;
}
// TLORA_OK, or TLORA_EHIP if the runtime reports an error from the launches queued so far
inline int launches_ok(int line) {
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? TLORA_OK : hip_failed(e, line);
}
#define TLORA_HIP(expr) do { const hipError_t e_ = (expr); if (e_ != hipSuccess) return hip_failed(e_, __LINE__); } while (0)

constexpr size_t kNoAllocMaxTableBytes = 64 * 3584;   // plan tables of tlora_fwd_noalloc: at most 64 argument chunks
uint8_t* g_scratch_ptr[kMaxDevices] = {};   // per device: address of `scratch` on that device (0 = not looked up yet)

// Address of the static scratch array on the current device (looked up once per device, with that device current).
int scratch_of_current_device(uint8_t** out) {
  int dev = -1;
  TLORA_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return TLORA_EINVAL;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    TLORA_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return TLORA_EHIP;
    g_scratch_ptr[dev] = static_cast<uint8_t*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return TLORA_OK;
}

struct Options {
  int shrink_rows = 0;          // 0 = chosen per problem (32 | 64 | 128), else forced
  int shrink_stages = 4;
  int grad_tokens = 256;
  int dx_transposed_w = 1;
  int plan_cache = 1;           // reuse plans of problems seen before (keyed by their contents)
  int indexed_direct = 1;       // token-indexed bf16 calls fetch rows through the index inside the kernels' loads
  int table_copy_kernel = 1;    // plan tables reach the workspace through a kernel that reads the pinned staging buffer
};
Options g_opt;
std::recursive_mutex g_mu;   // the nano-batch entry points call tlora_fwd / tlora_bwd under it

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- the plan ---------------------------------------------------------------------------------------
struct Plan {
  int J = 0, T = 0, d_in = 0, d_out = 0, dtype = 0;
  int max_rpad = 0;
  int shrink_rows = 128;                                // token rows per unit of the streaming shrink kernel
  std::vector<JobDev> jobs;
  std::vector<TileDev> tile_jobs;
  std::vector<ShrinkUnit> shrink_units;                 // generic kernel: 64 rows x 64 rank columns
  std::vector<ShrinkUnit> stream_units;                 // streaming kernel: shrink_rows x 128 rank columns
  std::vector<GradUnit> gradB_units, gradA_units;      // dB: columns over d_out;  dA: columns over d_in;

  int64_t gradB_partial = 0, gradA_partial = 0;         // floats of partial tiles
  std::vector<GradGroup> gradB_groups, gradA_groups;
  int64_t s_elems = 0;                                  // elements of the packed S (= dS) buffer
  int64_t atp_elems = 0;
  int r_total = 0;                                      // sum of rpad_j
  int64_t sx_elems = 0;                                 // elements of the per-tile K-extension operands
  // workspace byte offsets
  size_t off_tables = 0, off_S = 0, off_dS = 0, off_Shi = 0, off_Slo = 0, off_dShi = 0, off_dSlo = 0, off_Sx = 0, off_dSx = 0, off_atp = 0, off_wt = 0, off_ap = 0, off_bp = 0,
         off_partial = 0, total = 0;
  size_t tables_bytes = 0;
  // offsets of each table inside the table blob
  size_t tb_jobs = 0, tb_tiles = 0, tb_shrink = 0, tb_stream = 0, tb_gBu = 0, tb_gBg = 0, tb_gAu = 0, tb_gAg = 0, tb_f32 = 0;
  size_t off_clock = 0;                                 // 4 words outside the uploaded tables: GEMM clock probe
  size_t f32_reserved = 0;
};

constexpr int64_t kMaxUnits = (int64_t)1 << 22;   // most GEMM tiles / work units of one kind in a launch

int validate(const tlora_problem_t* p) {
  if (!p) return TLORA_ENULL;
  if (p->dtype != TLORA_F32 && p->dtype != TLORA_BF16) return TLORA_EDTYPE;
  if (p->num_jobs < 1 || p->d_in < 8 || p->d_out < 8 || (p->d_in % 8) || (p->d_out % 8)) return TLORA_EINVAL;
  if (p->num_jobs > TLORA_MAX_JOBS || p->d_in > TLORA_MAX_FEATURES || p->d_out > TLORA_MAX_FEATURES) return TLORA_EINVAL;
  if (!p->ranks || !p->offsets || !p->scales) return TLORA_ENULL;
  if (p->offsets[0] != 0) return TLORA_EINVAL;
  for (int j = 0; j < p->num_jobs; ++j) {
    if (p->offsets[j + 1] < p->offsets[j]) return TLORA_EINVAL;
    if (p->ranks[j] < 0 || p->ranks[j] > TLORA_MAX_RANK) return TLORA_EINVAL;
  }
  if (p->offsets[p->num_jobs] > TLORA_MAX_TOKENS) return TLORA_EINVAL;
  {   // one workgroup per GEMM tile: the grid (and the 32-bit tile index arithmetic) must hold them all
    const int64_t tiles_m = (p->offsets[p->num_jobs] + kGemmBM - 1) / kGemmBM;
    const int64_t tiles_n = (std::max(p->d_in, p->d_out) + kGemmBN - 1) / kGemmBN;
    if (tiles_m * tiles_n > kMaxUnits) return TLORA_EINVAL;
  }
  return TLORA_OK;
}

// Work units of the dA / dB token reductions (rank-aware nano-batches of one job's tokens).  A job's rank
// rows are cut into blocks of 128, of which a unit multiplies only the live 32-row sub-blocks.  A token
// chunk streams chunk * 256 * 2 bytes of the activation and leaves a partial tile of live_rows * 256 * 4
// bytes that is written and read once more, so the default chunk is 32 * live_rows tokens (partial traffic
// <= ~12 %).  If that gives too few units to fill the GPU the chunks are shortened (not below `grad_tokens`).
// Units are issued longest first.
bool build_grad_units(const Plan& pl, int D, std::vector<GradUnit>& units, std::vector<GradGroup>& groups,
                      int64_t& partial_floats) {
  const int ncb = (D + kGradCols - 1) / kGradCols;
  const int pb_rows = kGradMaxBlocks * kGradRanks;
  auto live_blocks = [&](const JobDev& jb, int pb) {
    return std::min(kGradMaxBlocks, (jb.rpad - pb * pb_rows + kGradRanks - 1) / kGradRanks);
  };
  auto chunk_of = [&](int live, double shrink) {
    int chunk = std::max(g_opt.grad_tokens, (int)(32 * kGradRanks * live * shrink));
    chunk = (chunk + kGradStep - 1) / kGradStep * kGradStep;
    return std::min(chunk, kGradMaxTokens);          // the kernel stages at most that many row indices per unit
  };
  auto count_units = [&](double shrink) {
    int64_t n = 0;
    for (const JobDev& jb : pl.jobs) {
      if (jb.rank == 0 || jb.row1 == jb.row0) continue;
      for (int pb = 0; pb * pb_rows < jb.rpad; ++pb) {
        const int chunk = chunk_of(live_blocks(jb, pb), shrink);
        n += (int64_t)((jb.row1 - jb.row0 + chunk - 1) / chunk) * ncb;
      }
    }
    return n;
  };
  double shrink = 1.0;
  const int64_t want = 1024;
  while (shrink > 1.0 / 64 && count_units(shrink) < want) shrink *= 0.5;
  if (count_units(shrink) > kMaxUnits) return false;      // refused before the tables are built
  partial_floats = 0;
  for (int j = 0; j < pl.J; ++j) {
    const JobDev& jb = pl.jobs[j];
    if (jb.rank == 0) continue;
    const int Tj = jb.row1 - jb.row0;
    for (int pb = 0; pb * pb_rows < jb.rpad; ++pb) {
      const int mb = live_blocks(jb, pb);
      const int chunk = chunk_of(mb, shrink);
      const int nchunks = Tj > 0 ? (Tj + chunk - 1) / chunk : 0;
      for (int cb = 0; cb < ncb; ++cb) {
        GradGroup g{};
        g.job = j;  g.cb = cb;  g.pb = pb;  g.mb = mb;  g.nunits = nchunks;  g.part_off = partial_floats;
        for (int c = 0; c < nchunks; ++c) {
          GradUnit u{};
          u.job = j;  u.t0 = jb.row0 + c * chunk;  u.t1 = std::min(jb.row1, u.t0 + chunk);  u.cb = cb;  u.pb = pb;
          u.mb = mb;  u.part_off = partial_floats;
          partial_floats += (int64_t)mb * kGradRanks * kGradCols;
          units.push_back(u);
        }
        groups.push_back(g);
      }
    }
  }
  // longest (then heaviest) first: the tail of the launch is made of the short units
  std::stable_sort(units.begin(), units.end(), [](const GradUnit& a, const GradUnit& b) {
    const int64_t ca = (int64_t)(a.t1 - a.t0) * (4 + a.mb), cb = (int64_t)(b.t1 - b.t0) * (4 + b.mb);
    return ca > cb;
  });
  return true;
}

// fwd_only: tables and workspace of the forward alone (no transposed W, no dS, no dA / dB units or partial tiles)
int build_plan(const tlora_problem_t* p, Plan& pl, bool fwd_only = false) {
  const int rc = validate(p);
  if (rc != TLORA_OK) return rc;
  pl.J = p->num_jobs;  pl.T = (int)p->offsets[p->num_jobs];  pl.d_in = p->d_in;  pl.d_out = p->d_out;
  pl.dtype = p->dtype;
  pl.jobs.resize(pl.J);
  int64_t soff = 0, atp = 0;
  int64_t roff = 0;
  for (int j = 0; j < pl.J; ++j) {
    JobDev& jb = pl.jobs[j];
    memset(&jb, 0, sizeof(jb));
    jb.row0 = (int32_t)p->offsets[j];  jb.row1 = (int32_t)p->offsets[j + 1];
    jb.rank = p->ranks[j];
    jb.rpad = (jb.rank + kRankGranule - 1) / kRankGranule * kRankGranule;
    jb.scale = p->scales[j];
    jb.soff = soff;  jb.atp_off = atp;  jb.roff = (int32_t)roff;
    // rows of the packed intermediates are padded (with zeros) to the dA / dB kernel's token step
    soff += (int64_t)((jb.row1 - jb.row0 + kGradStep - 1) / kGradStep * kGradStep) * jb.rpad;
    atp += (int64_t)jb.rpad * pl.d_in;
    roff += jb.rpad;
    pl.max_rpad = std::max(pl.max_rpad, jb.rpad);
  }
  if (roff > (int64_t)1 << 22) return TLORA_EINVAL;   // rows of the stacked adapter operands: 256 of them span 32-bit byte offsets
  pl.s_elems = soff;  pl.atp_elems = atp;  pl.r_total = (int)roff;

  // row tiles of the backbone GEMM (nano-batches of the concatenated batch, Sec. 3.3)
  const int tiles_m = (pl.T + kGemmBM - 1) / kGemmBM;
  pl.tile_jobs.resize(tiles_m);
  {
    int j = 0;
    for (int tm = 0; tm < tiles_m; ++tm) {
      const int r0 = tm * kGemmBM, r1 = std::min(pl.T, r0 + kGemmBM);
      while (pl.jobs[j].row1 <= r0) ++j;             // first job with a row at or after r0
      int last = j;
      for (int k = j; k < pl.J && pl.jobs[k].row0 < r1; ++k)
        if (pl.jobs[k].row1 > pl.jobs[k].row0) last = k;
      TileDev& td = pl.tile_jobs[tm];
      td.first = j;  td.last = last;
      // adapter K-extension of the tile: padded ranks of jobs first..last, rounded up to the K-step
      td.roff_first = pl.jobs[j].roff;
      const int span = pl.jobs[last].roff + pl.jobs[last].rpad - td.roff_first;
      td.kext = (span + kGemmBK - 1) / kGemmBK * kGemmBK;
      td.aoff = pl.sx_elems;
      pl.sx_elems += (int64_t)kGemmBM * td.kext;
    }
  }
  if (pl.dtype == TLORA_BF16) {
    // Rows per unit of the streaming shrink: 128 when that still gives enough workgroups for the 256 CUs, else 64, else
    // 32 (a small batch would otherwise stream its activations through a few dozen CUs).  The 32-row kernel exists for
    // K-steps of 64 only, and the units serve both the forward (K = d_in) and the backward (K = d_out) shrink.
    {
      auto count = [&](int rows) {
        int64_t n = 0;
        for (const JobDev& jb : pl.jobs)
          if (jb.rpad > 0) n += (int64_t)((jb.row1 - jb.row0 + rows - 1) / rows) * ((jb.rpad + 127) / 128);
        return n;
      };
      int64_t generic = 0;                           // units of the generic kernel: 64 rows x 64 rank columns
      for (const JobDev& jb : pl.jobs)
        generic += (int64_t)((jb.row1 - jb.row0 + 63) / 64) * ((jb.rpad + kShrinkCols - 1) / kShrinkCols);
      if (generic > kMaxUnits || count(32) > kMaxUnits) return TLORA_EINVAL;
      const bool can32 = pl.d_in % 64 == 0 && pl.d_out % 64 == 0;
      if (g_opt.shrink_rows != 0) pl.shrink_rows = (g_opt.shrink_rows == 32 && !can32) ? 64 : g_opt.shrink_rows;
      else pl.shrink_rows = count(128) >= 192 ? 128 : (count(64) >= 192 || !can32) ? 64 : 32;
    }
    for (int j = 0; j < pl.J; ++j) {
      const JobDev& jb = pl.jobs[j];
      if (jb.rpad == 0) continue;
      const int npb = (jb.rpad + kShrinkCols - 1) / kShrinkCols;
      for (int t0 = jb.row0; t0 < jb.row1; t0 += 64)
        for (int pb = 0; pb < npb; ++pb) {
          ShrinkUnit u;
          u.job = j;  u.t0 = t0;  u.nrows = std::min(64, jb.row1 - t0);  u.pb = pb;
          pl.shrink_units.push_back(u);
        }
      const int npb2 = (jb.rpad + 127) / 128;
      for (int t0 = jb.row0; t0 < jb.row1; t0 += pl.shrink_rows)
        for (int pb = 0; pb < npb2; ++pb) {
          ShrinkUnit u;
          u.job = j;  u.t0 = t0;  u.nrows = std::min(pl.shrink_rows, jb.row1 - t0);  u.pb = pb;
          pl.stream_units.push_back(u);
        }
    }
    if (!fwd_only) {
      if (!build_grad_units(pl, pl.d_out, pl.gradB_units, pl.gradB_groups, pl.gradB_partial) ||
          !build_grad_units(pl, pl.d_in, pl.gradA_units, pl.gradA_groups, pl.gradA_partial))
        return TLORA_EINVAL;
    }
  }

  // table blob
  size_t o = 0;
  auto place = [&](size_t bytes) { const size_t at = o;  o = align_up(o + bytes, 256);  return at; };
  pl.tb_jobs = place(sizeof(JobDev) * pl.jobs.size());
  pl.tb_tiles = place(sizeof(TileDev) * pl.tile_jobs.size());
  pl.tb_shrink = place(sizeof(ShrinkUnit) * pl.shrink_units.size());
  pl.tb_stream = place(sizeof(ShrinkUnit) * pl.stream_units.size());
  pl.tb_gBu = place(sizeof(GradUnit) * pl.gradB_units.size());
  pl.tb_gBg = place(sizeof(GradGroup) * pl.gradB_groups.size());
  pl.tb_gAu = place(sizeof(GradUnit) * pl.gradA_units.size());
  pl.tb_gAg = place(sizeof(GradGroup) * pl.gradA_groups.size());
  if (pl.dtype == TLORA_F32) {
    // the fp32 path needs at most 3 J + 1 products per launch, two launches per pass
    const size_t max_units = 2 * (size_t)(3 * pl.J + 1);
    size_t max_tiles = 0;
    auto tiles_of = [](int64_t m, int64_t n) { return (size_t)(((m + 63) / 64) * ((n + 63) / 64)); };
    max_tiles += 2 * tiles_of(pl.T, std::max(pl.d_in, pl.d_out));
    for (int j = 0; j < pl.J; ++j) {
      const JobDev& jb = pl.jobs[j];
      const int Tj = jb.row1 - jb.row0;
      max_tiles += 2 * tiles_of(Tj, jb.rank) + tiles_of(Tj, std::max(pl.d_in, pl.d_out)) +
                   tiles_of(pl.d_in, jb.rank) + tiles_of(jb.rank, pl.d_out);
    }
    pl.f32_reserved = align_up(sizeof(F32Unit) * max_units, 256) + align_up(sizeof(F32Tile) * max_tiles, 256) + 4 * 256;
    pl.tb_f32 = place(pl.f32_reserved);
  }
  pl.tables_bytes = o;

  // workspace layout
  size_t w = 0;
  auto wplace = [&](size_t bytes) { const size_t at = w;  w = align_up(w + bytes, 256);  return at; };
  // the transposed W first: its place depends on nothing but d_in x d_out, so a copy made by one call is found
  // by later calls on other token batches (nano-batches) that share the workspace
  if (pl.dtype == TLORA_BF16 && !fwd_only) pl.off_wt = wplace(2 * (size_t)pl.d_in * (size_t)pl.d_out);
  pl.off_tables = wplace(pl.tables_bytes);
  pl.off_clock = wplace(64);
  if (pl.dtype == TLORA_F32) {
    pl.off_S = wplace(sizeof(float) * (size_t)pl.s_elems);
    if (!fwd_only) pl.off_dS = wplace(sizeof(float) * (size_t)pl.s_elems);
  }
  if (pl.dtype == TLORA_BF16) {
    pl.off_Shi = wplace(2 * (size_t)pl.s_elems);
    pl.off_Slo = wplace(2 * (size_t)pl.s_elems);
    if (!fwd_only) {
      pl.off_dShi = wplace(2 * (size_t)pl.s_elems);
      pl.off_dSlo = wplace(2 * (size_t)pl.s_elems);
    }
    // + 256: a 64-wide K-step over a last 32-wide slice reads (and ignores) 64 bytes past each operand row
    pl.off_Sx = wplace(2 * (size_t)pl.sx_elems + 256);
    if (!fwd_only) pl.off_dSx = wplace(2 * (size_t)pl.sx_elems + 256);
    pl.off_atp = wplace(2 * ((size_t)pl.atp_elems + 32 * (size_t)pl.d_in));

    pl.off_ap = wplace(2 * (size_t)pl.d_in * (size_t)(pl.r_total + 32));
    pl.off_bp = wplace(2 * (size_t)pl.d_out * (size_t)(pl.r_total + 32));
    if (!fwd_only) pl.off_partial = wplace(sizeof(float) * (size_t)std::max(pl.gradB_partial, pl.gradA_partial));
  }
  pl.total = std::max<size_t>(w, 256);
  return TLORA_OK;
}

// ---- pinned staging for the table upload ----------------------------------------------------------------
// A small ring of pinned host buffers; a slot is reused only after the copy that read it has finished.
struct Slot {
  void* host = nullptr;
  void* dev_view = nullptr;   // the same buffer as the device addresses it (null: not mapped, copy commands are used)
  size_t cap = 0;
  hipEvent_t ev = nullptr;
  bool busy = false;
};
constexpr int kSlots = 16;
Slot g_slots[kSlots];
int g_next_slot = 0;

int upload_tables(const std::vector<uint8_t>& blob, void* dst, hipStream_t st) {
  Slot& s = g_slots[g_next_slot];
  g_next_slot = (g_next_slot + 1) % kSlots;
  if (s.busy) {
    TLORA_HIP(hipEventSynchronize(s.ev));
    s.busy = false;
  }
  if (s.cap < blob.size()) {
    if (s.host) (void)hipHostFree(s.host);
    s.host = nullptr;  s.dev_view = nullptr;  s.cap = 0;
    const size_t cap = align_up(blob.size() * 2, 4096);
    TLORA_HIP(hipHostMalloc(&s.host, cap, hipHostMallocDefault));
    s.cap = cap;
    if (hipHostGetDevicePointer(&s.dev_view, s.host, 0) != hipSuccess) {
      s.dev_view = nullptr;
      (void)hipGetLastError();
    }
  }
  if (!s.ev) TLORA_HIP(hipEventCreateWithFlags(&s.ev, hipEventDisableTiming));
  memcpy(s.host, blob.data(), blob.size());
  if (g_opt.table_copy_kernel && s.dev_view && blob.size() % 16 == 0 && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
    launch_table_copy(s.dev_view, dst, blob.size(), st);
    TLORA_HIP(hipGetLastError());
  } else {
    TLORA_HIP(hipMemcpyAsync(dst, s.host, blob.size(), hipMemcpyHostToDevice, st));
  }
  TLORA_HIP(hipEventRecord(s.ev, st));
  s.busy = true;
  return TLORA_OK;
}

// ---- optional per-kernel event timing ---------------------------------------------------------------------
struct Pending {
  int cls;
  hipEvent_t a, b;
};
bool g_prof_on = false;
bool g_prof_gemm_only = false;   // mode 2: only the two segmented-GEMM classes are bracketed
std::vector<Pending> g_pending;
std::vector<hipEvent_t> g_event_pool;
double g_prof_ms[TLORA_K_COUNT] = {};
unsigned long long* g_clock_slot[2] = {nullptr, nullptr};   // device slots of the last profiled fwd / dX GEMM
int64_t g_prof_n[TLORA_K_COUNT] = {};

hipEvent_t prof_event() {
  if (!g_event_pool.empty()) {
    hipEvent_t e = g_event_pool.back();
    g_event_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Brackets one launch with events when profiling is on.
struct Timed {
  hipStream_t st;
  Pending p{};
  bool on;
  Timed(int cls, hipStream_t s, bool enable = true)
      : st(s), on(g_prof_on && enable && (!g_prof_gemm_only || cls == TLORA_K_GEMM_FWD || cls == TLORA_K_GEMM_BWD)) {
    if (!on) return;
    p.cls = cls;  p.a = prof_event();  p.b = prof_event();
    if (!p.a || !p.b) { on = false; return; }
    (void)hipEventRecord(p.a, st);
  }
  ~Timed() {
    if (!on) return;
    (void)hipEventRecord(p.b, st);
    g_pending.push_back(p);
  }
};

int prof_drain() {
  for (const Pending& p : g_pending) {
    TLORA_HIP(hipEventSynchronize(p.b));
    float ms = 0.f;
    TLORA_HIP(hipEventElapsedTime(&ms, p.a, p.b));
    g_prof_ms[p.cls] += ms;
    g_prof_n[p.cls] += 1;
    g_event_pool.push_back(p.a);
    g_event_pool.push_back(p.b);
  }
  g_pending.clear();
  return TLORA_OK;
}

// S_j = X_j.A_j (or dS_j = dY_j.B_j^T): streaming kernel when the contraction length allows, else generic
void run_shrink(const Plan& pl, const uint8_t* tb, const JobDev* jobs, const TileDev* tiles, const uint16_t* act, int K,
                const uint16_t* packed, bool packed_is_atp, uint16_t* hi, uint16_t* lo, uint16_t* Sx,
                const int32_t* row_index, hipStream_t st) {
  if (K % 32 == 0)
    launch_shrink_stream(jobs, tiles, reinterpret_cast<const ShrinkUnit*>(tb + pl.tb_stream),
                         (int)pl.stream_units.size(), pl.shrink_rows, g_opt.shrink_stages, act, K, packed, packed_is_atp,
                         hi, lo, Sx, row_index, st);
  else
    launch_shrink(jobs, tiles, reinterpret_cast<const ShrinkUnit*>(tb + pl.tb_shrink), (int)pl.shrink_units.size(), 64,
                  act, K, packed, packed_is_atp, hi, lo, Sx, row_index, st);
}

int check_arch() {
  static int cached = 1;   // 1 = unknown
  if (cached != 1) return cached;
  int dev = 0;
  TLORA_HIP(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  TLORA_HIP(hipGetDeviceProperties(&prop, dev));
  cached = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? TLORA_OK : TLORA_EARCH;
  return cached;
}

inline bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

template <class T>
void put(std::vector<uint8_t>& blob, size_t at, const std::vector<T>& v) {
  if (!v.empty()) memcpy(blob.data() + at, v.data(), sizeof(T) * v.size());
}

std::vector<uint8_t> make_blob(const Plan& pl) {
  std::vector<uint8_t> blob(pl.tables_bytes, 0);
  put(blob, pl.tb_jobs, pl.jobs);
  put(blob, pl.tb_tiles, pl.tile_jobs);
  put(blob, pl.tb_shrink, pl.shrink_units);
  put(blob, pl.tb_stream, pl.stream_units);
  put(blob, pl.tb_gBu, pl.gradB_units);
  put(blob, pl.tb_gBg, pl.gradB_groups);
  put(blob, pl.tb_gAu, pl.gradA_units);
  put(blob, pl.tb_gAg, pl.gradA_groups);
  return blob;
}

// ---- plan cache ---------------------------------------------------------------------------------------------
// A plan depends only on (dtype, d_in, d_out, ranks, offsets), the forward-only flag and the tiling options; the
// per-call values (scales, adapter and gradient pointers) live in the job table alone, which every call patches into
// its copy of the cached table blob.  Training loops call with the same few problems step after step, so building
// the plan (vectors, unit sorting) and assembling the blob are paid once per distinct problem.  Entries are kept in
// most-recently-used order; everything here runs under g_mu.
struct PlanEntry {
  std::vector<int64_t> key;
  Plan pl;
  std::vector<uint8_t> blob;     // tables with a job table whose per-call fields are zero
};
constexpr size_t kPlanCacheEntries = 128;
std::list<PlanEntry> g_plans;
PlanEntry g_plan_uncached;       // the plan of the current call when the cache is switched off

void plan_key(const tlora_problem_t* p, bool fwd_only, std::vector<int64_t>& key) {
  key.clear();
  key.reserve(10 + 2 * (size_t)p->num_jobs);
  key.push_back(p->dtype);  key.push_back(p->num_jobs);  key.push_back(p->d_in);  key.push_back(p->d_out);
  key.push_back(fwd_only ? 1 : 0);
  key.push_back(g_opt.shrink_rows);  key.push_back(g_opt.grad_tokens);
  for (int j = 0; j < p->num_jobs; ++j) key.push_back(p->ranks[j]);
  for (int j = 0; j <= p->num_jobs; ++j) key.push_back(p->offsets[j]);
}

// The plan of a problem: from the cache, or built and inserted.
int get_plan(const tlora_problem_t* p, bool fwd_only, const PlanEntry** out) {
  const int rc = validate(p);
  if (rc != TLORA_OK) return rc;
  if (!g_opt.plan_cache) {
    g_plan_uncached = PlanEntry();
    const int rb = build_plan(p, g_plan_uncached.pl, fwd_only);
    if (rb != TLORA_OK) return rb;
    g_plan_uncached.blob = make_blob(g_plan_uncached.pl);
    *out = &g_plan_uncached;
    return TLORA_OK;
  }
  static std::vector<int64_t> key;
  plan_key(p, fwd_only, key);
  for (auto it = g_plans.begin(); it != g_plans.end(); ++it)
    if (it->key == key) {
      if (it != g_plans.begin()) g_plans.splice(g_plans.begin(), g_plans, it);
      *out = &g_plans.front();
      return TLORA_OK;
    }
  PlanEntry e;
  const int rb = build_plan(p, e.pl, fwd_only);
  if (rb != TLORA_OK) return rb;
  e.key = key;
  e.blob = make_blob(e.pl);
  g_plans.push_front(std::move(e));
  if (g_plans.size() > kPlanCacheEntries) g_plans.pop_back();
  *out = &g_plans.front();
  return TLORA_OK;
}

// fp32 path: append the tiles of one product
void f32_add(std::vector<F32Unit>& units, std::vector<F32Tile>& tiles, const F32Unit& u) {
  if (u.M <= 0 || u.N <= 0) return;
  const int id = (int)units.size();
  units.push_back(u);
  for (int tm = 0; tm < (u.M + 63) / 64; ++tm)
    for (int tn = 0; tn < (u.N + 63) / 64; ++tn) tiles.push_back(F32Tile{id, tm, tn, 0});
}
F32Unit f32_unit(const float* A, int64_t a_rs, int64_t a_cs, const float* B, int64_t b_rs, int64_t b_cs, float* C,
                 int64_t c_rs, int M, int N, int K, float alpha, bool accumulate) {
  F32Unit u{};
  u.A = A;  u.B = B;  u.C = C;  u.M = M;  u.N = N;  u.K = K;  u.accumulate = accumulate ? 1 : 0;
  u.a_rs = a_rs;  u.a_cs = a_cs;  u.b_rs = b_rs;  u.b_cs = b_cs;  u.c_rs = c_rs;  u.alpha = alpha;
  return u;
}

// Write the two launches' unit/tile tables into the blob's fp32 area and return their device addresses.
struct F32Launch {
  size_t units_at[2], tiles_at[2];
  int ntiles[2];
  size_t end;               // the blob is used up to here
};
int f32_place(const Plan& pl, std::vector<uint8_t>& blob, std::vector<F32Unit> units[2], std::vector<F32Tile> tiles[2],
              F32Launch& L) {
  size_t o = pl.tb_f32;
  for (int i = 0; i < 2; ++i) {
    // tile indices are per launch: rebase nothing, each launch has its own unit array
    L.units_at[i] = o;
    o = align_up(o + sizeof(F32Unit) * units[i].size(), 256);
    L.tiles_at[i] = o;
    o = align_up(o + sizeof(F32Tile) * tiles[i].size(), 256);
    L.ntiles[i] = (int)tiles[i].size();
  }
  if (o > pl.tb_f32 + pl.f32_reserved) return TLORA_EWORKSPACE;
  L.end = o;
  for (int i = 0; i < 2; ++i) {
    put(blob, L.units_at[i], units[i]);
    put(blob, L.tiles_at[i], tiles[i]);
  }
  return TLORA_OK;
}

// static_scratch: the "workspace" is the library's static scratch array and only the forward will run.
// Gives the (cached) plan and this call's job table: the plan's with the caller's scales and adapter pointers.
int common_checks(const tlora_problem_t* p, const PlanEntry** entry, std::vector<JobDev>& hjobs, void* ws, size_t ws_bytes,
                  bool static_scratch = false) {
  int rc = get_plan(p, static_scratch, entry);
  if (rc != TLORA_OK) return rc;
  const Plan& pl = (*entry)->pl;
  if ((pl.T > 0 && !p->X) || !p->W || !p->A || !p->B) return TLORA_ENULL;
  for (int j = 0; j < pl.J; ++j)
    if (pl.jobs[j].rank > 0 && (!p->A[j] || !p->B[j])) return TLORA_ENULL;
  if (misaligned16(p->X) || misaligned16(p->W)) return TLORA_EALIGN;
  if (static_scratch && ws_bytes < pl.total) return TLORA_ESCRATCH;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || ws_bytes < pl.total) return TLORA_EWORKSPACE;
  hjobs = pl.jobs;
  for (int j = 0; j < pl.J; ++j) {
    hjobs[j].scale = p->scales[j];
    hjobs[j].A = p->A[j];
    hjobs[j].B = p->B[j];
  }
  return TLORA_OK;
}

}  // namespace
}  // namespace tlora

using namespace tlora;

extern "C" {

size_t tlora_workspace_bytes(const tlora_problem_t* p) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  const PlanEntry* e = nullptr;
  if (get_plan(p, false, &e) != TLORA_OK) return 0;
  return e->pl.total;
}

}  // extern "C"

namespace tlora {
namespace {
// The forward's launch sequence.  no_alloc: the workspace is the static device scratch (`workspace` = its address on
// the current device, `ws_bytes` = its size); the plan and the workspace layout are the forward's alone, the tables
// reach the device as kernel arguments (no staging buffer, no copy node), and nothing is timed: no HIP object is
// created and no memory of any kind is allocated on this path.
// Token-indexed calls (bf16): out_index = the batch row of every token row of the job-sorted order -- the GEMM scatters
// its output rows there; in_index = the same list when X is the batch in its own order, fetched through the list
// inside the kernels' loads (null: X already lies in job-sorted order).
int fwd_impl(const tlora_problem_t* p, void* Y, void* workspace, size_t ws_bytes, void* hip_stream, bool no_alloc,
             const int32_t* out_index = nullptr, const int32_t* in_index = nullptr) {
  const PlanEntry* entry = nullptr;
  std::vector<JobDev> hjobs;
  int rc = common_checks(p, &entry, hjobs, workspace, ws_bytes, no_alloc);
  if (rc != TLORA_OK) return rc;
  const Plan& pl = entry->pl;
  if (pl.T > 0 && !Y) return TLORA_ENULL;
  if (misaligned16(Y)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK) return rc;
  if (pl.T == 0) return TLORA_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  uint8_t* tb = ws + pl.off_tables;
  std::vector<uint8_t> blob = entry->blob;          // the cached tables, with this call's job table
  put(blob, pl.tb_jobs, hjobs);
  const JobDev* jobs = reinterpret_cast<const JobDev*>(tb + pl.tb_jobs);
  const bool timed = g_prof_on && !no_alloc;
  auto upload = [&](size_t used) {
    if (!no_alloc) return upload_tables(blob, tb, st);
    if (used > kNoAllocMaxTableBytes) return (int)TLORA_ESCRATCH;
    launch_table_write(blob.data(), used, tb, st);
    return (int)TLORA_OK;
  };

  if (pl.dtype == TLORA_F32) {
    float* S = reinterpret_cast<float*>(ws + pl.off_S);
    const float* X = static_cast<const float*>(p->X);
    const float* W = static_cast<const float*>(p->W);
    float* Yf = static_cast<float*>(Y);
    std::vector<F32Unit> units[2];
    std::vector<F32Tile> tiles[2];
    f32_add(units[0], tiles[0], f32_unit(X, pl.d_in, 1, W, pl.d_out, 1, Yf, pl.d_out, pl.T, pl.d_out, pl.d_in, 1.f, false));
    for (int j = 0; j < pl.J; ++j) {
      const JobDev& jb = hjobs[j];
      const int Tj = jb.row1 - jb.row0;
      if (jb.rank == 0 || Tj == 0) continue;
      const float* Xj = X + (int64_t)jb.row0 * pl.d_in;
      float* Sj = S + jb.soff;
      f32_add(units[0], tiles[0], f32_unit(Xj, pl.d_in, 1, static_cast<const float*>(jb.A), jb.rank, 1, Sj, jb.rpad,
                                           Tj, jb.rank, pl.d_in, 1.f, false));
      f32_add(units[1], tiles[1], f32_unit(Sj, jb.rpad, 1, static_cast<const float*>(jb.B), pl.d_out, 1,
                                           Yf + (int64_t)jb.row0 * pl.d_out, pl.d_out, Tj, pl.d_out, jb.rank, jb.scale,
                                           true));
    }
    F32Launch L;
    rc = f32_place(pl, blob, units, tiles, L);
    if (rc != TLORA_OK) return rc;
    rc = upload(L.end);
    if (rc != TLORA_OK) return rc;
    for (int i = 0; i < 2; ++i) {
      Timed t(TLORA_K_F32, st, timed);
      launch_f32_units(reinterpret_cast<const F32Unit*>(tb + L.units_at[i]),
                       reinterpret_cast<const F32Tile*>(tb + L.tiles_at[i]), L.ntiles[i], st);
    }
    return launches_ok(__LINE__);
  }

  rc = upload(pl.tables_bytes);
  if (rc != TLORA_OK) return rc;
  uint16_t* Sx = reinterpret_cast<uint16_t*>(ws + pl.off_Sx);
  uint16_t* atp = reinterpret_cast<uint16_t*>(ws + pl.off_atp);
  uint16_t* ap = reinterpret_cast<uint16_t*>(ws + pl.off_ap);
  uint16_t* bp = reinterpret_cast<uint16_t*>(ws + pl.off_bp);
  const TileDev* tiles = reinterpret_cast<const TileDev*>(tb + pl.tb_tiles);
  {
    Timed t(TLORA_K_PACK, st, timed);
    launch_pack_adapters(jobs, pl.J, pl.d_in, pl.d_out, pl.max_rpad, pl.r_total, atp, ap, bp, st);
    launch_zero_fill(Sx, 2 * (size_t)pl.sx_elems, st);
  }
  {
    Timed t(TLORA_K_SHRINK, st, timed);
    run_shrink(pl, tb, jobs, tiles, static_cast<const uint16_t*>(p->X), pl.d_in, atp, true,
               reinterpret_cast<uint16_t*>(ws + pl.off_Shi), reinterpret_cast<uint16_t*>(ws + pl.off_Slo), Sx, in_index, st);
  }
  if (timed) launch_zero_fill(ws + pl.off_clock, 16, st);
  Timed tg(TLORA_K_GEMM_FWD, st, timed);
  launch_seg_gemm(true, tiles, static_cast<const uint16_t*>(p->X), static_cast<const uint16_t*>(p->W), Sx, bp,
                  pl.r_total, static_cast<uint16_t*>(Y), out_index, in_index, pl.T, pl.d_in, pl.d_out,
                  timed ? (g_clock_slot[0] = reinterpret_cast<unsigned long long*>(ws + pl.off_clock)) : nullptr, st);
  return launches_ok(__LINE__);
}
}  // namespace
}  // namespace tlora

extern "C" {

int tlora_fwd(const tlora_problem_t* p, void* Y, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  return fwd_impl(p, Y, workspace, ws_bytes, hip_stream, false);
}

int tlora_fwd_noalloc(const tlora_problem_t* p, void* Y, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  uint8_t* ws = nullptr;
  const int rc = scratch_of_current_device(&ws);
  if (rc != TLORA_OK) return rc;
  return fwd_impl(p, Y, ws, TLORA_NOALLOC_SCRATCH_BYTES, hip_stream, true);
}

}  // extern "C"

namespace tlora {
namespace {
// The backward's launch sequence (out_index / in_index as in fwd_impl: dX rows are scattered; X and dY are fetched
// through the list).
int bwd_impl(const tlora_problem_t* p, const void* dY, void* dX, void* const* dA, void* const* dB, int flags,
             void* workspace, size_t ws_bytes, void* hip_stream, const int32_t* out_index, const int32_t* in_index) {
  const PlanEntry* entry = nullptr;
  std::vector<JobDev> hjobs;
  int rc = common_checks(p, &entry, hjobs, workspace, ws_bytes);
  if (rc != TLORA_OK) return rc;
  const Plan& pl = entry->pl;
  if (pl.T > 0 && !dY) return TLORA_ENULL;
  if ((dA == nullptr) != (dB == nullptr)) return TLORA_ENULL;
  if (misaligned16(dY) || (dX && misaligned16(dX))) return TLORA_EALIGN;
  const bool want_grads = dA != nullptr;
  if (want_grads)
    for (int j = 0; j < pl.J; ++j) {
      if (pl.jobs[j].rank > 0 && (!dA[j] || !dB[j])) return TLORA_ENULL;
      hjobs[j].dA = dA[j];
      hjobs[j].dB = dB[j];
    }
  if (flags & ~(TLORA_BWD_REUSE_S | TLORA_BWD_REUSE_WT | TLORA_BWD_ACCUMULATE)) return TLORA_EINVAL;
  const bool accumulate = (flags & TLORA_BWD_ACCUMULATE) != 0;
  rc = check_arch();
  if (rc != TLORA_OK) return rc;
  const bool reuse_S = (flags & TLORA_BWD_REUSE_S) != 0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  uint8_t* tb = ws + pl.off_tables;
  std::vector<uint8_t> blob = entry->blob;          // the cached tables, with this call's job table
  put(blob, pl.tb_jobs, hjobs);
  const JobDev* jobs = reinterpret_cast<const JobDev*>(tb + pl.tb_jobs);

  if (pl.dtype == TLORA_F32) {
    float* S = reinterpret_cast<float*>(ws + pl.off_S);
    float* dS = reinterpret_cast<float*>(ws + pl.off_dS);
    const float* X = static_cast<const float*>(p->X);
    const float* W = static_cast<const float*>(p->W);
    const float* dYf = static_cast<const float*>(dY);
    float* dXf = static_cast<float*>(dX);
    std::vector<F32Unit> units[2];
    std::vector<F32Tile> tiles[2];
    if (dXf)   // dX = dY . W^T : B(k = o, n = i) = W[i, o]
      f32_add(units[0], tiles[0], f32_unit(dYf, pl.d_out, 1, W, 1, pl.d_out, dXf, pl.d_in, pl.T, pl.d_in, pl.d_out, 1.f, false));
    for (int j = 0; j < pl.J; ++j) {
      const JobDev& jb = hjobs[j];
      const int Tj = jb.row1 - jb.row0;
      if (jb.rank == 0) continue;
      const float* Aj = static_cast<const float*>(jb.A);
      const float* Bj = static_cast<const float*>(jb.B);
      const float* Xj = X + (int64_t)jb.row0 * pl.d_in;
      const float* dYj = dYf + (int64_t)jb.row0 * pl.d_out;
      float* Sj = S + jb.soff;
      float* dSj = dS + jb.soff;
      // dS_j = dY_j . B_j^T : B(k = o, n = p) = B_j[p, o]
      f32_add(units[0], tiles[0], f32_unit(dYj, pl.d_out, 1, Bj, 1, pl.d_out, dSj, jb.rpad, Tj, jb.rank, pl.d_out, 1.f, false));
      if (!reuse_S && want_grads)
        f32_add(units[0], tiles[0], f32_unit(Xj, pl.d_in, 1, Aj, jb.rank, 1, Sj, jb.rpad, Tj, jb.rank, pl.d_in, 1.f, false));
      if (dXf)   // dX_j += s_j dS_j . A_j^T : B(k = p, n = i) = A_j[i, p]
        f32_add(units[1], tiles[1], f32_unit(dSj, jb.rpad, 1, Aj, 1, jb.rank, dXf + (int64_t)jb.row0 * pl.d_in, pl.d_in,
                                             Tj, pl.d_in, jb.rank, jb.scale, true));
      if (want_grads) {
        // dA_j = s_j X_j^T . dS_j : A(m = i, k = t) = X_j[t, i]
        f32_add(units[1], tiles[1], f32_unit(Xj, 1, pl.d_in, dSj, jb.rpad, 1, static_cast<float*>(jb.dA), jb.rank,
                                             pl.d_in, jb.rank, Tj, jb.scale, accumulate));
        // dB_j = s_j S_j^T . dY_j : A(m = p, k = t) = S_j[t, p]
        f32_add(units[1], tiles[1], f32_unit(Sj, 1, jb.rpad, dYj, pl.d_out, 1, static_cast<float*>(jb.dB), pl.d_out,
                                             jb.rank, pl.d_out, Tj, jb.scale, accumulate));
      }
    }
    F32Launch L;
    rc = f32_place(pl, blob, units, tiles, L);
    if (rc != TLORA_OK) return rc;
    rc = upload_tables(blob, tb, st);
    if (rc != TLORA_OK) return rc;
    for (int i = 0; i < 2; ++i) {
      Timed t(TLORA_K_F32, st);
      launch_f32_units(reinterpret_cast<const F32Unit*>(tb + L.units_at[i]),
                       reinterpret_cast<const F32Tile*>(tb + L.tiles_at[i]), L.ntiles[i], st);
    }
    return launches_ok(__LINE__);
  }

  rc = upload_tables(blob, tb, st);
  if (rc != TLORA_OK) return rc;
  uint16_t* Sx = reinterpret_cast<uint16_t*>(ws + pl.off_Sx);
  uint16_t* dSx = reinterpret_cast<uint16_t*>(ws + pl.off_dSx);
  uint16_t* Shi = reinterpret_cast<uint16_t*>(ws + pl.off_Shi);
  uint16_t* Slo = reinterpret_cast<uint16_t*>(ws + pl.off_Slo);
  uint16_t* dShi = reinterpret_cast<uint16_t*>(ws + pl.off_dShi);
  uint16_t* dSlo = reinterpret_cast<uint16_t*>(ws + pl.off_dSlo);
  uint16_t* atp = reinterpret_cast<uint16_t*>(ws + pl.off_atp);
  uint16_t* ap = reinterpret_cast<uint16_t*>(ws + pl.off_ap);
  uint16_t* bp = reinterpret_cast<uint16_t*>(ws + pl.off_bp);
  float* partial = reinterpret_cast<float*>(ws + pl.off_partial);
  const TileDev* tiles = reinterpret_cast<const TileDev*>(tb + pl.tb_tiles);
  const uint16_t* Xb = static_cast<const uint16_t*>(p->X);
  const uint16_t* dYb = static_cast<const uint16_t*>(dY);
  const bool redo_S = want_grads && !reuse_S;

  {
    Timed t(TLORA_K_PACK, st);
    // with TLORA_BWD_REUSE_S the forward's packed copies of the (unchanged) adapters are still in the workspace
    if (!reuse_S) launch_pack_adapters(jobs, pl.J, pl.d_in, pl.d_out, pl.max_rpad, pl.r_total, atp, ap, bp, st);
    if (pl.T > 0) {
      launch_zero_fill(dSx, 2 * (size_t)pl.sx_elems, st);
      if (redo_S) launch_zero_fill(Sx, 2 * (size_t)pl.sx_elems, st);
    }
  }
  if (pl.T > 0) {
    if (redo_S) {
      Timed t(TLORA_K_SHRINK, st);
      run_shrink(pl, tb, jobs, tiles, Xb, pl.d_in, atp, true, Shi, Slo, Sx, in_index, st);
    }
    {
      Timed t(TLORA_K_SHRINK, st);
      run_shrink(pl, tb, jobs, tiles, dYb, pl.d_out, bp, false, dShi, dSlo, dSx, in_index, st);
    }
    if (dX) {
      // dX = dY . W^T contracts over W's contiguous dimension.  Against a transposed copy of W the weight tiles
      // are 64 rows of 512 contiguous bytes instead of 256 rows of 128, which the load stream handles markedly
      // better (the copy costs one read and one write of W; W is frozen, so REUSE_WT skips it).
      const bool wt = g_opt.dx_transposed_w != 0;
      uint16_t* Wt = reinterpret_cast<uint16_t*>(ws + pl.off_wt);
      if (wt && !(flags & TLORA_BWD_REUSE_WT)) {
        Timed t(TLORA_K_WT, st);
        launch_transpose_bf16(static_cast<const uint16_t*>(p->W), Wt, pl.d_in, pl.d_out, st);
      }
      if (g_prof_on) launch_zero_fill(ws + pl.off_clock + 16, 16, st);
      Timed t(TLORA_K_GEMM_BWD, st);
      launch_seg_gemm(wt, tiles, dYb, wt ? Wt : static_cast<const uint16_t*>(p->W), dSx, wt ? atp : ap, pl.r_total,
                      static_cast<uint16_t*>(dX), out_index, in_index, pl.T, pl.d_out, pl.d_in,
                      g_prof_on ? (g_clock_slot[1] = reinterpret_cast<unsigned long long*>(ws + pl.off_clock) + 2) : nullptr,
                      st);
    }
  }
  if (want_grads) {
    {
      Timed t(TLORA_K_RANK_GRAD, st);
      launch_rank_grad(jobs, reinterpret_cast<const GradUnit*>(tb + pl.tb_gBu), (int)pl.gradB_units.size(), Shi, Slo,
                       dYb, pl.d_out, partial, in_index, st);
    }
    {
      Timed t(TLORA_K_GRAD_REDUCE, st);
      launch_grad_reduce(jobs, reinterpret_cast<const GradGroup*>(tb + pl.tb_gBg), (int)pl.gradB_groups.size(), partial,
                         pl.d_out, false, accumulate, st);
    }
    {
      Timed t(TLORA_K_RANK_GRAD, st);
      launch_rank_grad(jobs, reinterpret_cast<const GradUnit*>(tb + pl.tb_gAu), (int)pl.gradA_units.size(), dShi, dSlo,
                       Xb, pl.d_in, partial, in_index, st);
    }
    {
      Timed t(TLORA_K_GRAD_REDUCE, st);
      launch_grad_reduce(jobs, reinterpret_cast<const GradGroup*>(tb + pl.tb_gAg), (int)pl.gradA_groups.size(), partial,
                         pl.d_in, true, accumulate, st);
    }
  }
  return launches_ok(__LINE__);
}

}  // namespace
}  // namespace tlora

extern "C" {

int tlora_bwd(const tlora_problem_t* p, const void* dY, void* dX, void* const* dA, void* const* dB, int flags,
              void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  return bwd_impl(p, dY, dX, dA, dB, flags, workspace, ws_bytes, hip_stream, nullptr, nullptr);
}

// ---- adaptive nano-batching (Sec. 3.3) --------------------------------------------------------------------
int tlora_aimd_init(tlora_aimd_t* c, int32_t n0, int32_t alpha, double beta, double tau_rel, int32_t n_max) {
  if (!c) return TLORA_ENULL;
  if (n0 < 1 || alpha < 1 || !(beta > 0.0 && beta < 1.0) || !(tau_rel >= 0.0) || n_max < 0) return TLORA_EINVAL;
  c->n = n_max > 0 ? std::min(n0, n_max) : n0;
  c->alpha = alpha;  c->n_max = n_max;  c->have_prev = 0;
  c->beta = beta;  c->tau_rel = tau_rel;  c->t_prev = 0.0;
  return TLORA_OK;
}

int tlora_aimd_update(tlora_aimd_t* c, double t_step, int32_t* n_next) {
  if (!c) return TLORA_ENULL;
  if (!(t_step >= 0.0) || c->n < 1) return TLORA_EINVAL;
  int64_t n = c->n;
  if (c->have_prev) {
    const double tau = c->tau_rel * c->t_prev;
    if (t_step <= c->t_prev - tau) n = n + c->alpha;                              // additive increase
    else n = std::max<int64_t>(1, (int64_t)std::floor(c->beta * (double)c->n));   // multiplicative decrease
  }
  if (c->n_max > 0) n = std::min<int64_t>(n, c->n_max);
  n = std::min<int64_t>(n, INT32_MAX);
  c->n = (int32_t)n;  c->t_prev = t_step;  c->have_prev = 1;
  if (n_next) *n_next = c->n;
  return TLORA_OK;
}

namespace {
// token boundary n of N nano-batches: whole samples of `granule` tokens, floor(n U / N) of the U samples
int64_t nano_bound(int64_t T, int64_t n, int64_t N, int64_t granule) {
  const int64_t units = (T + granule - 1) / granule;
  return std::min<int64_t>(T, granule * (int64_t)(((__int128)n * units) / N));
}
// sub-problem of one nano-batch: same jobs, the rows of each segment that fall into [b0, b1)
struct NanoSub {
  tlora_problem_t p;
  std::vector<int64_t> off;
  int64_t b0 = 0, b1 = 0;
};
int make_sub(const tlora_problem_t* p, int32_t n_nano, int64_t granule, int32_t n, NanoSub& s) {
  const int rc = validate(p);
  if (rc != TLORA_OK) return rc;
  if (n_nano < 1 || granule < 1 || n < 0 || n >= n_nano) return TLORA_EINVAL;
  const int64_t T = p->offsets[p->num_jobs];
  s.b0 = nano_bound(T, n, n_nano, granule);
  s.b1 = nano_bound(T, n + 1, n_nano, granule);
  s.off.resize(p->num_jobs + 1);
  for (int j = 0; j <= p->num_jobs; ++j) s.off[j] = std::min(std::max(p->offsets[j], s.b0), s.b1) - s.b0;
  s.p = *p;
  s.p.offsets = s.off.data();
  const size_t elt = p->dtype == TLORA_F32 ? 4 : 2;
  s.p.X = p->X ? static_cast<const uint8_t*>(p->X) + (size_t)s.b0 * p->d_in * elt : nullptr;
  return TLORA_OK;
}
}  // namespace

int tlora_nano_split(const tlora_problem_t* p, int32_t n_nano, int64_t granule, int32_t n, int64_t* row0,
                     int64_t* row1, int64_t* sub_offsets) {
  NanoSub s;
  const int rc = make_sub(p, n_nano, granule, n, s);
  if (rc != TLORA_OK) return rc;
  if (row0) *row0 = s.b0;
  if (row1) *row1 = s.b1;
  if (sub_offsets) std::copy(s.off.begin(), s.off.end(), sub_offsets);
  return TLORA_OK;
}

size_t tlora_nano_workspace_bytes(const tlora_problem_t* p, int32_t n_nano, int64_t granule) {
  size_t need = 0;
  for (int32_t n = 0; n < n_nano; ++n) {
    NanoSub s;
    if (make_sub(p, n_nano, granule, n, s) != TLORA_OK) return 0;
    const size_t b = tlora_workspace_bytes(&s.p);
    if (b == 0) return 0;
    need = std::max(need, b);
  }
  return need;
}

int tlora_fwd_nano(const tlora_problem_t* p, int32_t n_nano, int64_t granule, void* Y, void* workspace, size_t ws_bytes,
                   void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  if (!p) return TLORA_ENULL;
  const size_t need = tlora_nano_workspace_bytes(p, n_nano, granule);
  if (need == 0) return validate(p) != TLORA_OK ? validate(p) : TLORA_EINVAL;
  if (!workspace || ws_bytes < need) return TLORA_EWORKSPACE;
  const size_t elt = p->dtype == TLORA_F32 ? 4 : 2;
  for (int32_t n = 0; n < n_nano; ++n) {          // one after the other, on the caller's stream
    NanoSub s;
    int rc = make_sub(p, n_nano, granule, n, s);
    if (rc != TLORA_OK) return rc;
    if (s.b1 == s.b0) continue;
    rc = tlora_fwd(&s.p, Y ? static_cast<uint8_t*>(Y) + (size_t)s.b0 * p->d_out * elt : nullptr, workspace, ws_bytes,
                   hip_stream);
    if (rc != TLORA_OK) return rc;
  }
  return TLORA_OK;
}

int tlora_bwd_nano(const tlora_problem_t* p, int32_t n_nano, int64_t granule, const void* dY, void* dX, void* const* dA,
                   void* const* dB, int flags, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  if (!p) return TLORA_ENULL;
  if (flags & ~(TLORA_BWD_REUSE_WT | TLORA_BWD_ACCUMULATE)) return TLORA_EINVAL;   // S of a nano-batch is not kept
  const size_t need = tlora_nano_workspace_bytes(p, n_nano, granule);
  if (need == 0) return validate(p) != TLORA_OK ? validate(p) : TLORA_EINVAL;
  if (!workspace || ws_bytes < need) return TLORA_EWORKSPACE;
  const size_t elt = p->dtype == TLORA_F32 ? 4 : 2;
  bool first = true, wt_made = (flags & TLORA_BWD_REUSE_WT) != 0;
  for (int32_t n = 0; n < n_nano; ++n) {
    NanoSub s;
    int rc = make_sub(p, n_nano, granule, n, s);
    if (rc != TLORA_OK) return rc;
    if (s.b1 == s.b0 && !(first && n == n_nano - 1)) continue;      // (an all-empty batch still zeroes dA / dB once)
    // the adapter gradients are sums over the job's tokens: the first nano-batch overwrites, the others add
    int f = (first ? (flags & TLORA_BWD_ACCUMULATE) : TLORA_BWD_ACCUMULATE) | (wt_made ? TLORA_BWD_REUSE_WT : 0);
    rc = tlora_bwd(&s.p, dY ? static_cast<const uint8_t*>(dY) + (size_t)s.b0 * p->d_out * elt : nullptr,
                   dX ? static_cast<uint8_t*>(dX) + (size_t)s.b0 * p->d_in * elt : nullptr, dA, dB, f, workspace,
                   ws_bytes, hip_stream);
    if (rc != TLORA_OK) return rc;
    first = false;
    if (dX && s.b1 > s.b0) wt_made = true;
  }
  return TLORA_OK;
}

// ---- per-job optimizer step ---------------------------------------------------------------------------------
size_t tlora_adamw_workspace_bytes(int32_t count) {
  if (count < 0) return 0;
  return std::max<size_t>(256, align_up(sizeof(AdamwDev) * (size_t)count, 256));
}

int tlora_adamw_step(const tlora_adamw_tensor_t* tensors, int32_t count, int32_t dtype, void* workspace, size_t ws_bytes,
                     void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  if (count < 0) return TLORA_EINVAL;
  if (dtype != TLORA_F32 && dtype != TLORA_BF16) return TLORA_EDTYPE;
  if (count > 0 && !tensors) return TLORA_ENULL;
  if (count > 65535) return TLORA_EINVAL;
  std::vector<uint8_t> blob(sizeof(AdamwDev) * (size_t)count);
  AdamwDev* d = reinterpret_cast<AdamwDev*>(blob.data());
  int64_t max_n = 0;
  for (int i = 0; i < count; ++i) {
    const tlora_adamw_tensor_t& t = tensors[i];
    if (t.n < 0 || t.step < 1 || !(t.beta1 >= 0.f && t.beta1 < 1.f) || !(t.beta2 >= 0.f && t.beta2 < 1.f) ||
        !(t.eps >= 0.f) || !(t.lr >= 0.f) || !(t.weight_decay >= 0.f))
      return TLORA_EINVAL;
    if (t.n > 0 && (!t.param || !t.grad || !t.m || !t.v)) return TLORA_ENULL;
    if (t.n > 0 && dtype == TLORA_BF16 && !t.master) return TLORA_ENULL;   // a bf16 tensor cannot carry the update
    d[i].param = t.param;  d[i].master = t.master;  d[i].grad = t.grad;  d[i].m = t.m;  d[i].v = t.v;  d[i].n = t.n;
    d[i].lr = t.lr;  d[i].beta1 = t.beta1;  d[i].beta2 = t.beta2;  d[i].eps = t.eps;  d[i].weight_decay = t.weight_decay;
    d[i].c1 = (float)(1.0 / (1.0 - std::pow((double)t.beta1, (double)t.step)));
    d[i].c2 = (float)(1.0 / (1.0 - std::pow((double)t.beta2, (double)t.step)));
    d[i].param_is_bf16 = dtype == TLORA_BF16;
    max_n = std::max(max_n, t.n);
  }
  if (count == 0 || max_n == 0) return TLORA_OK;
  if (!workspace || ws_bytes < tlora_adamw_workspace_bytes(count) || (reinterpret_cast<uintptr_t>(workspace) & 255))
    return TLORA_EWORKSPACE;
  int rc = check_arch();
  if (rc != TLORA_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  rc = upload_tables(blob, workspace, st);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_OPT, st);
    launch_adamw(static_cast<const AdamwDev*>(workspace), count, max_n, st);
  }
  return launches_ok(__LINE__);
}

// ---- MLP block: RMSNorm -> gate / up (fused multi-LoRA) -> silu(G) * U -> down (fused multi-LoRA) -> + X -------
namespace {
struct MlpLayout {
  tlora_problem_t gate, up, down;      // the three fused layers (X pointers filled in below)
  size_t elt = 2;
  int64_t T = 0;
  size_t off_xn = 0, off_rstd = 0, off_g = 0, off_u = 0, off_z = 0, off_d = 0, off_dz = 0, off_dg = 0, off_du = 0,
         off_dxa = 0, off_dxb = 0, off_ws_gate = 0, off_ws_up = 0, off_ws_down = 0;
  size_t ws_gate = 0, ws_up = 0, ws_down = 0, total = 0;
};
int mlp_layout(const tlora_mlp_t* p, MlpLayout& L) {
  if (!p) return TLORA_ENULL;
  if (p->dtype != TLORA_F32 && p->dtype != TLORA_BF16) return TLORA_EDTYPE;
  if (!(p->eps >= 0.f)) return TLORA_EINVAL;
  auto layer = [&](int d_in, int d_out, const void* W, const void* const* A, const void* const* B) {
    tlora_problem_t q;
    memset(&q, 0, sizeof(q));
    q.dtype = p->dtype;  q.num_jobs = p->num_jobs;  q.d_in = d_in;  q.d_out = d_out;
    q.ranks = p->ranks;  q.offsets = p->offsets;  q.scales = p->scales;
    q.X = nullptr;  q.W = W;  q.A = A;  q.B = B;
    return q;
  };
  L.gate = layer(p->d_model, p->d_ff, p->W_gate, p->A_gate, p->B_gate);
  L.up = layer(p->d_model, p->d_ff, p->W_up, p->A_up, p->B_up);
  L.down = layer(p->d_ff, p->d_model, p->W_down, p->A_down, p->B_down);
  L.gate.X = L.up.X = L.down.X = p->X;          // placeholder so that validation sees a non-null activation
  int rc = validate(&L.gate);
  if (rc == TLORA_OK) rc = validate(&L.up);
  if (rc == TLORA_OK) rc = validate(&L.down);
  if (rc != TLORA_OK) return rc;
  L.T = p->offsets[p->num_jobs];
  if (L.T > 0 && !p->gamma) return TLORA_ENULL;
  L.elt = p->dtype == TLORA_F32 ? 4 : 2;
  size_t w = 0;
  auto place = [&](size_t bytes) { const size_t at = w;  w = align_up(w + bytes, 256);  return at; };
  const size_t td = (size_t)L.T * p->d_model * L.elt, tf = (size_t)L.T * p->d_ff * L.elt;
  L.off_xn = place(td);  L.off_rstd = place(sizeof(float) * (size_t)L.T);
  L.off_g = place(tf);  L.off_u = place(tf);  L.off_z = place(tf);  L.off_d = place(td);
  L.off_dz = place(tf);  L.off_dg = place(tf);  L.off_du = place(tf);  L.off_dxa = place(td);  L.off_dxb = place(td);
  L.ws_gate = tlora_workspace_bytes(&L.gate);  L.ws_up = tlora_workspace_bytes(&L.up);
  L.ws_down = tlora_workspace_bytes(&L.down);
  if (!L.ws_gate || !L.ws_up || !L.ws_down) return TLORA_EINVAL;
  L.off_ws_gate = place(L.ws_gate);  L.off_ws_up = place(L.ws_up);  L.off_ws_down = place(L.ws_down);
  L.total = w;
  return TLORA_OK;
}
}  // namespace

size_t tlora_mlp_workspace_bytes(const tlora_mlp_t* p) {
  MlpLayout L;
  return mlp_layout(p, L) == TLORA_OK ? L.total : 0;
}

int tlora_mlp_fwd(const tlora_mlp_t* p, void* Out, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  MlpLayout L;
  int rc = mlp_layout(p, L);
  if (rc != TLORA_OK) return rc;
  if (!workspace || ws_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return TLORA_EWORKSPACE;
  if (L.T > 0 && (!p->X || !Out)) return TLORA_ENULL;
  if (misaligned16(p->X) || misaligned16(Out) || misaligned16(p->gamma)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK) return rc;
  if (L.T == 0) return TLORA_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  const bool bf = p->dtype == TLORA_BF16;
  {
    Timed t(TLORA_K_GLUE, st);
    launch_rmsnorm_fwd(bf, p->X, p->gamma, p->eps, (int)L.T, p->d_model, ws + L.off_xn,
                       reinterpret_cast<float*>(ws + L.off_rstd), st);
  }
  L.gate.X = L.up.X = ws + L.off_xn;
  rc = tlora_fwd(&L.gate, ws + L.off_g, ws + L.off_ws_gate, L.ws_gate, hip_stream);
  if (rc != TLORA_OK) return rc;
  rc = tlora_fwd(&L.up, ws + L.off_u, ws + L.off_ws_up, L.ws_up, hip_stream);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_GLUE, st);
    launch_swiglu_fwd(bf, ws + L.off_g, ws + L.off_u, ws + L.off_z, L.T * p->d_ff, st);
  }
  L.down.X = ws + L.off_z;
  rc = tlora_fwd(&L.down, ws + L.off_d, ws + L.off_ws_down, L.ws_down, hip_stream);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_GLUE, st);
    launch_residual_add(bf, p->X, ws + L.off_d, Out, L.T * p->d_model, st);
  }
  return launches_ok(__LINE__);
}

int tlora_mlp_bwd(const tlora_mlp_t* p, const void* dOut, void* dX, void* const* dA_gate, void* const* dB_gate,
                  void* const* dA_up, void* const* dB_up, void* const* dA_down, void* const* dB_down, int flags,
                  void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  MlpLayout L;
  int rc = mlp_layout(p, L);
  if (rc != TLORA_OK) return rc;
  if (flags & ~(TLORA_BWD_ACCUMULATE | TLORA_BWD_REUSE_WT)) return TLORA_EINVAL;
  if (!workspace || ws_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return TLORA_EWORKSPACE;
  if (L.T > 0 && (!p->X || !dOut || !dX)) return TLORA_ENULL;
  if (!dA_gate || !dB_gate || !dA_up || !dB_up || !dA_down || !dB_down) return TLORA_ENULL;
  if (misaligned16(p->X) || misaligned16(dOut) || misaligned16(dX) || misaligned16(p->gamma)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  const bool bf = p->dtype == TLORA_BF16;
  // every layer's workspace still holds its S_j from tlora_mlp_fwd
  const int lf = flags | TLORA_BWD_REUSE_S;
  L.gate.X = L.up.X = ws + L.off_xn;
  L.down.X = ws + L.off_z;
  rc = tlora_bwd(&L.down, dOut, ws + L.off_dz, dA_down, dB_down, lf, ws + L.off_ws_down, L.ws_down, hip_stream);
  if (rc != TLORA_OK) return rc;
  if (L.T > 0) {
    Timed t(TLORA_K_GLUE, st);
    launch_swiglu_bwd(bf, ws + L.off_g, ws + L.off_u, ws + L.off_dz, ws + L.off_dg, ws + L.off_du, L.T * p->d_ff, st);
  }
  rc = tlora_bwd(&L.gate, ws + L.off_dg, ws + L.off_dxa, dA_gate, dB_gate, lf, ws + L.off_ws_gate, L.ws_gate, hip_stream);
  if (rc != TLORA_OK) return rc;
  rc = tlora_bwd(&L.up, ws + L.off_du, ws + L.off_dxb, dA_up, dB_up, lf, ws + L.off_ws_up, L.ws_up, hip_stream);
  if (rc != TLORA_OK) return rc;
  if (L.T > 0) {
    Timed t(TLORA_K_GLUE, st);
    launch_rmsnorm_bwd(bf, p->X, p->gamma, reinterpret_cast<const float*>(ws + L.off_rstd), ws + L.off_dxa,
                       ws + L.off_dxb, nullptr, dOut, (int)L.T, p->d_model, dX, st);
  }
  return launches_ok(__LINE__);
}

// ---- attention half: rotary embedding, causal grouped-query attention, and the block around them ----------
namespace {
struct AttnPlan {
  int64_t T = 0;
  std::vector<AttnTile> tiles;
  std::vector<int32_t> pos;
  int64_t max_len = 0;
  size_t off_tiles = 0, off_pos = 0, off_D = 0, off_rope = 0, blob_bytes = 0, total = 0;
};
// tables: [tiles | positions] (uploaded), then D fp32 [T, n_heads] and the rotary (cos, sin) table [longest sequence, 64]
int attn_plan(int32_t num_seqs, const int64_t* seq_offsets, int32_t n_heads, bool want_tables, AttnPlan& A) {
  if (num_seqs < 0 || n_heads < 1) return TLORA_EINVAL;
  if (!seq_offsets) return TLORA_ENULL;
  if (seq_offsets[0] != 0) return TLORA_EINVAL;
  size_t n_tiles = 0;
  for (int32_t s = 0; s < num_seqs; ++s) {
    const int64_t len = seq_offsets[s + 1] - seq_offsets[s];
    if (len < 0 || seq_offsets[s + 1] > (int64_t)INT32_MAX) return TLORA_EINVAL;
    n_tiles += (size_t)((len + 127) / 128);
    A.max_len = std::max(A.max_len, len);
  }
  A.T = seq_offsets[num_seqs];
  if ((int64_t)A.T * n_heads > (int64_t)INT32_MAX) return TLORA_EINVAL;
  if (want_tables) {
    A.tiles.reserve(n_tiles);
    A.pos.resize((size_t)A.T);
    // longest sequences' last tiles first: a tile's work grows with t0, so the heavy ones start early
    for (int32_t s = 0; s < num_seqs; ++s) {
      const int64_t a = seq_offsets[s], len = seq_offsets[s + 1] - a;
      for (int64_t t0 = 0; t0 < len; t0 += 128) A.tiles.push_back(AttnTile{(int32_t)a, (int32_t)len, (int32_t)t0, 0});
      for (int64_t i = 0; i < len; ++i) A.pos[(size_t)(a + i)] = (int32_t)i;
    }
    std::stable_sort(A.tiles.begin(), A.tiles.end(), [](const AttnTile& x, const AttnTile& y) { return x.t0 > y.t0; });
  }
  size_t w = 0;
  auto place = [&](size_t bytes) { const size_t at = w;  w = align_up(w + bytes, 256);  return at; };
  A.off_tiles = place(n_tiles * sizeof(AttnTile));
  A.off_pos = place((size_t)A.T * sizeof(int32_t));
  A.blob_bytes = w;
  A.off_D = place((size_t)A.T * n_heads * sizeof(float));
  A.off_rope = place((size_t)A.max_len * 64 * 2 * sizeof(float));
  A.total = std::max<size_t>(w, 256);
  return TLORA_OK;
}
int attn_upload(const AttnPlan& A, void* ws, hipStream_t st) {
  std::vector<uint8_t> blob(A.blob_bytes, 0);
  if (!A.tiles.empty()) memcpy(blob.data() + A.off_tiles, A.tiles.data(), A.tiles.size() * sizeof(AttnTile));
  if (!A.pos.empty()) memcpy(blob.data() + A.off_pos, A.pos.data(), A.pos.size() * sizeof(int32_t));
  if (blob.empty()) return TLORA_OK;
  return upload_tables(blob, ws, st);
}
int attn_heads_ok(int32_t n_heads, int32_t n_kv, int32_t head_dim) {
  if (head_dim != kAttnHeadDim) return TLORA_EINVAL;
  if (n_heads < 1 || n_kv < 1 || n_heads % n_kv != 0 || n_heads > 4096) return TLORA_EINVAL;   // 32-bit byte offsets inside a tile
  return TLORA_OK;
}
inline bool bad_ws(const void* ws, size_t have, size_t need) {
  return !ws || have < need || (reinterpret_cast<uintptr_t>(ws) & 255);
}
}  // namespace

size_t tlora_attention_workspace_bytes(int32_t num_seqs, const int64_t* seq_offsets, int32_t n_heads) {
  AttnPlan A;
  return attn_plan(num_seqs, seq_offsets, n_heads, false, A) == TLORA_OK ? A.total : 0;
}

int tlora_rope(void* X, int32_t num_seqs, const int64_t* seq_offsets, int32_t heads, int32_t head_dim, float rope_base,
               int32_t inverse, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  if (head_dim != kAttnHeadDim || !(rope_base > 1.f) || heads > 4096) return TLORA_EINVAL;
  AttnPlan A;
  int rc = attn_plan(num_seqs, seq_offsets, heads, true, A);
  if (rc != TLORA_OK) return rc;
  if (bad_ws(workspace, ws_bytes, A.total)) return TLORA_EWORKSPACE;
  if (A.T > 0 && !X) return TLORA_ENULL;
  if (misaligned16(X)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK || A.T == 0) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  rc = attn_upload(A, ws, st);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_ROPE, st);
    launch_rope_table(reinterpret_cast<float*>(ws + A.off_rope), (int)A.max_len, rope_base, st);
    launch_rope(static_cast<uint16_t*>(X), reinterpret_cast<const int32_t*>(ws + A.off_pos),
                reinterpret_cast<const float*>(ws + A.off_rope), A.T, heads, inverse != 0, st);
  }
  return launches_ok(__LINE__);
}

int tlora_attention_fwd(const void* Q, const void* K, const void* V, void* O, float* lse, int32_t num_seqs,
                        const int64_t* seq_offsets, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, void* workspace,
                        size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  int rc = attn_heads_ok(n_heads, n_kv_heads, head_dim);
  if (rc != TLORA_OK) return rc;
  AttnPlan A;
  rc = attn_plan(num_seqs, seq_offsets, n_heads, true, A);
  if (rc != TLORA_OK) return rc;
  if (bad_ws(workspace, ws_bytes, A.total)) return TLORA_EWORKSPACE;
  if (A.T > 0 && (!Q || !K || !V || !O || !lse)) return TLORA_ENULL;
  if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK || A.T == 0) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  rc = attn_upload(A, ws, st);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_ATTN_FWD, st);
    launch_attn_fwd(reinterpret_cast<const AttnTile*>(ws + A.off_tiles), (int)A.tiles.size(), static_cast<const uint16_t*>(Q),
                    static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(V), static_cast<uint16_t*>(O), lse,
                    n_heads, n_kv_heads, st);
  }
  return launches_ok(__LINE__);
}

int tlora_attention_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO, const float* lse,
                        void* dQ, void* dK, void* dV, int32_t num_seqs, const int64_t* seq_offsets, int32_t n_heads,
                        int32_t n_kv_heads, int32_t head_dim, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  int rc = attn_heads_ok(n_heads, n_kv_heads, head_dim);
  if (rc != TLORA_OK) return rc;
  AttnPlan A;
  rc = attn_plan(num_seqs, seq_offsets, n_heads, true, A);
  if (rc != TLORA_OK) return rc;
  if (bad_ws(workspace, ws_bytes, A.total)) return TLORA_EWORKSPACE;
  if (A.T > 0 && (!Q || !K || !V || !O || !dO || !lse || !dQ || !dK || !dV)) return TLORA_ENULL;
  if (misaligned16(Q) || misaligned16(K) || misaligned16(V) || misaligned16(O) || misaligned16(dO) || misaligned16(dQ) ||
      misaligned16(dK) || misaligned16(dV))
    return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK || A.T == 0) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  rc = attn_upload(A, ws, st);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_ATTN_BWD, st);
    launch_attn_bwd(reinterpret_cast<const AttnTile*>(ws + A.off_tiles), (int)A.tiles.size(), static_cast<const uint16_t*>(Q),
                    static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(V), static_cast<const uint16_t*>(O),
                    static_cast<const uint16_t*>(dO), lse, reinterpret_cast<float*>(ws + A.off_D),
                    static_cast<uint16_t*>(dQ), static_cast<uint16_t*>(dK), static_cast<uint16_t*>(dV), A.T, n_heads,
                    n_kv_heads, st);
  }
  return launches_ok(__LINE__);
}

namespace {
struct AttnLayout {
  tlora_problem_t q, k, v, o;
  AttnPlan A;
  int64_t T = 0;
  size_t off_attn = 0, off_xn = 0, off_rstd = 0, off_q = 0, off_k = 0, off_v = 0, off_o = 0, off_lse = 0, off_d = 0,
         off_do = 0, off_dq = 0, off_dk = 0, off_dv = 0, off_dxa = 0, off_dxb = 0, off_dxc = 0, off_ws[4] = {0, 0, 0, 0};
  size_t ws_l[4] = {0, 0, 0, 0}, total = 0;
};
int attn_layout(const tlora_attn_t* p, bool want_tables, AttnLayout& L) {
  if (!p) return TLORA_ENULL;
  if (p->dtype != TLORA_BF16) return TLORA_EDTYPE;
  if (!(p->eps >= 0.f) || !(p->rope_base > 1.f)) return TLORA_EINVAL;
  int rc = attn_heads_ok(p->n_heads, p->n_kv_heads, p->head_dim);
  if (rc != TLORA_OK) return rc;
  if (p->num_jobs < 0 || !p->offsets) return p->offsets ? TLORA_EINVAL : TLORA_ENULL;
  const int dq = p->n_heads * p->head_dim, dkv = p->n_kv_heads * p->head_dim;
  auto layer = [&](int d_in, int d_out, const void* W, const void* const* A, const void* const* B) {
    tlora_problem_t q;
    memset(&q, 0, sizeof(q));
    q.dtype = p->dtype;  q.num_jobs = p->num_jobs;  q.d_in = d_in;  q.d_out = d_out;
    q.ranks = p->ranks;  q.offsets = p->offsets;  q.scales = p->scales;
    q.X = p->X;  q.W = W;  q.A = A;  q.B = B;      // X: placeholder so that validation sees a non-null activation
    return q;
  };
  L.q = layer(p->d_model, dq, p->W_q, p->A_q, p->B_q);
  L.k = layer(p->d_model, dkv, p->W_k, p->A_k, p->B_k);
  L.v = layer(p->d_model, dkv, p->W_v, p->A_v, p->B_v);
  L.o = layer(dq, p->d_model, p->W_o, p->A_o, p->B_o);
  tlora_problem_t* ls[4] = {&L.q, &L.k, &L.v, &L.o};
  for (tlora_problem_t* l : ls) {
    rc = validate(l);
    if (rc != TLORA_OK) return rc;
  }
  L.T = p->offsets[p->num_jobs];
  rc = attn_plan(p->num_seqs, p->seq_offsets, p->n_heads, want_tables, L.A);
  if (rc != TLORA_OK) return rc;
  if (L.A.T != L.T) return TLORA_EINVAL;
  if (L.T > 0 && !p->gamma) return TLORA_ENULL;
  size_t w = 0;
  auto place = [&](size_t bytes) { const size_t at = w;  w = align_up(w + bytes, 256);  return at; };
  const size_t td = (size_t)L.T * p->d_model * 2, tq = (size_t)L.T * dq * 2, tk = (size_t)L.T * dkv * 2;
  L.off_attn = place(L.A.total);
  L.off_xn = place(td);  L.off_rstd = place(sizeof(float) * (size_t)L.T);
  L.off_q = place(tq);  L.off_k = place(tk);  L.off_v = place(tk);  L.off_o = place(tq);
  L.off_lse = place(sizeof(float) * (size_t)L.T * p->n_heads);
  L.off_d = place(td);
  L.off_do = place(tq);  L.off_dq = place(tq);  L.off_dk = place(tk);  L.off_dv = place(tk);
  L.off_dxa = place(td);  L.off_dxb = place(td);  L.off_dxc = place(td);
  for (int i = 0; i < 4; ++i) {
    L.ws_l[i] = tlora_workspace_bytes(ls[i]);
    if (!L.ws_l[i]) return TLORA_EINVAL;
    L.off_ws[i] = place(L.ws_l[i]);
  }
  L.total = w;
  return TLORA_OK;
}
}  // namespace

size_t tlora_attn_workspace_bytes(const tlora_attn_t* p) {
  AttnLayout L;
  return attn_layout(p, false, L) == TLORA_OK ? L.total : 0;
}

int tlora_attn_fwd(const tlora_attn_t* p, void* Out, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  AttnLayout L;
  int rc = attn_layout(p, true, L);
  if (rc != TLORA_OK) return rc;
  if (bad_ws(workspace, ws_bytes, L.total)) return TLORA_EWORKSPACE;
  if (L.T > 0 && (!p->X || !Out)) return TLORA_ENULL;
  if (misaligned16(p->X) || misaligned16(Out) || misaligned16(p->gamma)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK || L.T == 0) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  uint8_t* aw = ws + L.off_attn;
  rc = attn_upload(L.A, aw, st);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_GLUE, st);
    launch_rmsnorm_fwd(true, p->X, p->gamma, p->eps, (int)L.T, p->d_model, ws + L.off_xn,
                       reinterpret_cast<float*>(ws + L.off_rstd), st);
  }
  L.q.X = L.k.X = L.v.X = ws + L.off_xn;
  rc = tlora_fwd(&L.q, ws + L.off_q, ws + L.off_ws[0], L.ws_l[0], hip_stream);
  if (rc == TLORA_OK) rc = tlora_fwd(&L.k, ws + L.off_k, ws + L.off_ws[1], L.ws_l[1], hip_stream);
  if (rc == TLORA_OK) rc = tlora_fwd(&L.v, ws + L.off_v, ws + L.off_ws[2], L.ws_l[2], hip_stream);
  if (rc != TLORA_OK) return rc;
  const int32_t* pos = reinterpret_cast<const int32_t*>(aw + L.A.off_pos);
  {
    Timed t(TLORA_K_ROPE, st);
    float* tab = reinterpret_cast<float*>(aw + L.A.off_rope);
    launch_rope_table(tab, (int)L.A.max_len, p->rope_base, st);
    launch_rope(reinterpret_cast<uint16_t*>(ws + L.off_q), pos, tab, L.T, p->n_heads, false, st);
    launch_rope(reinterpret_cast<uint16_t*>(ws + L.off_k), pos, tab, L.T, p->n_kv_heads, false, st);
  }
  {
    Timed t(TLORA_K_ATTN_FWD, st);
    launch_attn_fwd(reinterpret_cast<const AttnTile*>(aw + L.A.off_tiles), (int)L.A.tiles.size(),
                    reinterpret_cast<const uint16_t*>(ws + L.off_q), reinterpret_cast<const uint16_t*>(ws + L.off_k),
                    reinterpret_cast<const uint16_t*>(ws + L.off_v), reinterpret_cast<uint16_t*>(ws + L.off_o),
                    reinterpret_cast<float*>(ws + L.off_lse), p->n_heads, p->n_kv_heads, st);
  }
  L.o.X = ws + L.off_o;
  rc = tlora_fwd(&L.o, ws + L.off_d, ws + L.off_ws[3], L.ws_l[3], hip_stream);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_GLUE, st);
    launch_residual_add(true, p->X, ws + L.off_d, Out, L.T * p->d_model, st);
  }
  return launches_ok(__LINE__);
}

int tlora_attn_bwd(const tlora_attn_t* p, const void* dOut, void* dX, void* const* const* dA, void* const* const* dB,
                   int flags, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  AttnLayout L;
  int rc = attn_layout(p, true, L);
  if (rc != TLORA_OK) return rc;
  if (flags & ~(TLORA_BWD_ACCUMULATE | TLORA_BWD_REUSE_WT)) return TLORA_EINVAL;
  if (bad_ws(workspace, ws_bytes, L.total)) return TLORA_EWORKSPACE;
  if (L.T > 0 && (!p->X || !dOut || !dX)) return TLORA_ENULL;
  if (!dA || !dB) return TLORA_ENULL;
  for (int i = 0; i < 4; ++i)
    if (!dA[i] || !dB[i]) return TLORA_ENULL;
  if (misaligned16(p->X) || misaligned16(dOut) || misaligned16(dX) || misaligned16(p->gamma)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  uint8_t* aw = ws + L.off_attn;
  const int lf = flags | TLORA_BWD_REUSE_S;            // every projection's workspace still holds its S_j
  L.q.X = L.k.X = L.v.X = ws + L.off_xn;
  L.o.X = ws + L.off_o;
  rc = tlora_bwd(&L.o, dOut, ws + L.off_do, dA[3], dB[3], lf, ws + L.off_ws[3], L.ws_l[3], hip_stream);
  if (rc != TLORA_OK) return rc;
  if (L.T > 0) {
    const int32_t* pos = reinterpret_cast<const int32_t*>(aw + L.A.off_pos);   // tables uploaded by tlora_attn_fwd
    {
      Timed t(TLORA_K_ATTN_BWD, st);
      launch_attn_bwd(reinterpret_cast<const AttnTile*>(aw + L.A.off_tiles), (int)L.A.tiles.size(),
                      reinterpret_cast<const uint16_t*>(ws + L.off_q), reinterpret_cast<const uint16_t*>(ws + L.off_k),
                      reinterpret_cast<const uint16_t*>(ws + L.off_v), reinterpret_cast<const uint16_t*>(ws + L.off_o),
                      reinterpret_cast<const uint16_t*>(ws + L.off_do), reinterpret_cast<const float*>(ws + L.off_lse),
                      reinterpret_cast<float*>(aw + L.A.off_D), reinterpret_cast<uint16_t*>(ws + L.off_dq),
                      reinterpret_cast<uint16_t*>(ws + L.off_dk), reinterpret_cast<uint16_t*>(ws + L.off_dv), L.T,
                      p->n_heads, p->n_kv_heads, st);
    }
    {
      Timed t(TLORA_K_ROPE, st);
      const float* tab = reinterpret_cast<const float*>(aw + L.A.off_rope);     // written by tlora_attn_fwd
      launch_rope(reinterpret_cast<uint16_t*>(ws + L.off_dq), pos, tab, L.T, p->n_heads, true, st);
      launch_rope(reinterpret_cast<uint16_t*>(ws + L.off_dk), pos, tab, L.T, p->n_kv_heads, true, st);
    }
  }
  rc = tlora_bwd(&L.q, ws + L.off_dq, ws + L.off_dxa, dA[0], dB[0], lf, ws + L.off_ws[0], L.ws_l[0], hip_stream);
  if (rc == TLORA_OK) rc = tlora_bwd(&L.k, ws + L.off_dk, ws + L.off_dxb, dA[1], dB[1], lf, ws + L.off_ws[1], L.ws_l[1], hip_stream);
  if (rc == TLORA_OK) rc = tlora_bwd(&L.v, ws + L.off_dv, ws + L.off_dxc, dA[2], dB[2], lf, ws + L.off_ws[2], L.ws_l[2], hip_stream);
  if (rc != TLORA_OK) return rc;
  if (L.T > 0) {
    Timed t(TLORA_K_GLUE, st);
    launch_rmsnorm_bwd(true, p->X, p->gamma, reinterpret_cast<const float*>(ws + L.off_rstd), ws + L.off_dxa,
                       ws + L.off_dxb, ws + L.off_dxc, dOut, (int)L.T, p->d_model, dX, st);
  }
  return launches_ok(__LINE__);
}

// ---- one decoder layer: attention block, then MLP block -----------------------------------------------------
namespace {
struct LayerLayout {
  tlora_attn_t attn;
  tlora_mlp_t mlp;
  int64_t T = 0;
  size_t off_h = 0, off_dh = 0, off_attn = 0, off_mlp = 0, ws_attn = 0, ws_mlp = 0, total = 0;
};
int layer_layout(const tlora_layer_t* p, LayerLayout& L) {
  if (!p) return TLORA_ENULL;
  L.attn = p->attn;
  L.mlp = p->mlp;
  const tlora_attn_t& a = L.attn;
  const tlora_mlp_t& m = L.mlp;
  if (a.dtype != TLORA_BF16 || m.dtype != TLORA_BF16) return TLORA_EDTYPE;
  if (a.num_jobs != m.num_jobs || a.d_model != m.d_model || a.num_jobs < 0) return TLORA_EINVAL;
  if (!a.offsets || !m.offsets) return TLORA_ENULL;
  if (a.num_jobs > 0 && (!a.ranks || !m.ranks || !a.scales || !m.scales)) return TLORA_ENULL;
  for (int j = 0; j < a.num_jobs; ++j)
    if (a.ranks[j] != m.ranks[j] || a.scales[j] != m.scales[j] || a.offsets[j] != m.offsets[j]) return TLORA_EINVAL;
  if (a.offsets[a.num_jobs] != m.offsets[a.num_jobs]) return TLORA_EINVAL;
  L.mlp.X = a.X;                         // placeholder for validation; the real input is H
  L.ws_attn = tlora_attn_workspace_bytes(&L.attn);
  L.ws_mlp = tlora_mlp_workspace_bytes(&L.mlp);
  if (!L.ws_attn || !L.ws_mlp) return TLORA_EINVAL;
  L.T = a.offsets[a.num_jobs];
  size_t w = 0;
  auto place = [&](size_t bytes) { const size_t at = w;  w = align_up(w + bytes, 256);  return at; };
  const size_t td = (size_t)L.T * a.d_model * 2;
  L.off_h = place(td);  L.off_dh = place(td);
  L.off_attn = place(L.ws_attn);  L.off_mlp = place(L.ws_mlp);
  L.total = std::max<size_t>(w, 256);
  return TLORA_OK;
}
}  // namespace

size_t tlora_layer_workspace_bytes(const tlora_layer_t* p) {
  LayerLayout L;
  return layer_layout(p, L) == TLORA_OK ? L.total : 0;
}

int tlora_layer_fwd(const tlora_layer_t* p, void* Out, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  LayerLayout L;
  int rc = layer_layout(p, L);
  if (rc != TLORA_OK) return rc;
  if (bad_ws(workspace, ws_bytes, L.total)) return TLORA_EWORKSPACE;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  rc = tlora_attn_fwd(&L.attn, ws + L.off_h, ws + L.off_attn, L.ws_attn, hip_stream);
  if (rc != TLORA_OK) return rc;
  L.mlp.X = ws + L.off_h;
  return tlora_mlp_fwd(&L.mlp, Out, ws + L.off_mlp, L.ws_mlp, hip_stream);
}

int tlora_layer_bwd(const tlora_layer_t* p, const void* dOut, void* dX, void* const* const* dA, void* const* const* dB,
                    int flags, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  LayerLayout L;
  int rc = layer_layout(p, L);
  if (rc != TLORA_OK) return rc;
  if (bad_ws(workspace, ws_bytes, L.total)) return TLORA_EWORKSPACE;
  if (!dA || !dB) return TLORA_ENULL;
  for (int i = 0; i < 7; ++i)
    if (!dA[i] || !dB[i]) return TLORA_ENULL;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  L.mlp.X = ws + L.off_h;
  rc = tlora_mlp_bwd(&L.mlp, dOut, ws + L.off_dh, dA[4], dB[4], dA[5], dB[5], dA[6], dB[6], flags, ws + L.off_mlp, L.ws_mlp,
                     hip_stream);
  if (rc != TLORA_OK) return rc;
  return tlora_attn_bwd(&L.attn, ws + L.off_dh, dX, dA, dB, flags, ws + L.off_attn, L.ws_attn, hip_stream);
}

// ---- general token -> adapter assignment (Sec. 3.3: tokens of an adapter are gathered, results scattered back) ----
namespace {
struct IndexedLayout {
  size_t inner = 0, off_x = 0, off_y = 0, off_dx = 0, off_idx = 0, total = 0, elt = 2;
  int64_t T = 0;
};
// The kernels that fetch rows through the index list keep 32-bit byte offsets from the tensor's base.
inline bool direct_index_ok(int64_t T, int64_t width) {
  return g_opt.indexed_direct != 0 && T * width * 2 < ((int64_t)1 << 32);
}
int indexed_layout(const tlora_problem_t* p, IndexedLayout& L) {
  const int rc = validate(p);
  if (rc != TLORA_OK) return rc;
  L.inner = tlora_workspace_bytes(p);
  if (L.inner == 0) return TLORA_EINVAL;
  L.T = p->offsets[p->num_jobs];
  L.elt = p->dtype == TLORA_F32 ? 4 : 2;
  L.off_x = align_up(L.inner, 256);
  L.off_y = align_up(L.off_x + (size_t)L.T * p->d_in * L.elt, 256);
  L.off_dx = align_up(L.off_y + (size_t)L.T * p->d_out * L.elt, 256);
  // the fp32 configuration has no scattering epilogue: its sorted dX is staged and scattered by a copy pass
  L.off_idx = align_up(L.off_dx + (p->dtype == TLORA_F32 ? (size_t)L.T * p->d_in * L.elt : 0), 256);
  // the row list as the kernels use it: the caller's, with every entry forced into [0, T)
  L.total = align_up(L.off_idx + (size_t)L.T * sizeof(int32_t), 256);
  return TLORA_OK;
}
// Everything tlora_fwd / tlora_bwd would reject, checked before the first launch of an indexed call.
int indexed_checks(const tlora_problem_t* q, void* workspace, size_t inner, bool backward, void* const* dA,
                   void* const* dB, int flags) {
  const PlanEntry* e = nullptr;
  std::vector<JobDev> hj;
  const int rc = common_checks(q, &e, hj, workspace, inner);
  if (rc != TLORA_OK || !backward) return rc;
  if ((dA == nullptr) != (dB == nullptr)) return TLORA_ENULL;
  if (dA)
    for (int j = 0; j < q->num_jobs; ++j)
      if (q->ranks[j] > 0 && (!dA[j] || !dB[j])) return TLORA_ENULL;
  if (flags & ~(TLORA_BWD_REUSE_S | TLORA_BWD_REUSE_WT | TLORA_BWD_ACCUMULATE)) return TLORA_EINVAL;
  return TLORA_OK;
}
}  // namespace

size_t tlora_indexed_workspace_bytes(const tlora_problem_t* p) {
  IndexedLayout L;
  return indexed_layout(p, L) == TLORA_OK ? L.total : 0;
}

int tlora_fwd_indexed(const tlora_problem_t* p, const int32_t* row_index, void* Y, void* workspace, size_t ws_bytes,
                      void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  IndexedLayout L;
  int rc = indexed_layout(p, L);
  if (rc != TLORA_OK) return rc;
  if (!workspace || ws_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return TLORA_EWORKSPACE;
  if (L.T > 0 && (!row_index || !Y || !p->X)) return TLORA_ENULL;
  if (misaligned16(Y) || misaligned16(p->X)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK) return rc;
  if (L.T == 0) return TLORA_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  int32_t* const index = reinterpret_cast<int32_t*>(ws + L.off_idx);
  // bf16: the kernels fetch the activation rows through the list inside their loads and the GEMM scatters its output
  // rows, so the batch is read and written exactly as often as in a contiguous call (the in-kernel row offsets are 32
  // bits: larger activations take the gathered copy below)
  const bool direct = p->dtype == TLORA_BF16 && direct_index_ok(L.T, p->d_in);
  tlora_problem_t q = *p;
  if (!direct) q.X = ws + L.off_x;
  rc = indexed_checks(&q, workspace, L.inner, false, nullptr, nullptr, 0);
  if (rc != TLORA_OK) return rc;
  {
    Timed t(TLORA_K_PERMUTE, st);
    launch_clamp_index(row_index, index, L.T, st);
  }
  if (direct) return fwd_impl(p, Y, workspace, L.inner, hip_stream, false, index, index);
  {
    Timed t(TLORA_K_PERMUTE, st);
    launch_permute_rows(p->X, ws + L.off_x, index, L.T, (int64_t)p->d_in * L.elt, false, st);
  }
  if (p->dtype == TLORA_BF16) return fwd_impl(&q, Y, workspace, L.inner, hip_stream, false, index);
  rc = tlora_fwd(&q, ws + L.off_y, workspace, L.inner, hip_stream);
  if (rc != TLORA_OK) return rc;
  Timed t(TLORA_K_PERMUTE, st);
  launch_permute_rows(ws + L.off_y, Y, index, L.T, (int64_t)p->d_out * L.elt, true, st);
  return launches_ok(__LINE__);
}

int tlora_bwd_indexed(const tlora_problem_t* p, const int32_t* row_index, const void* dY, void* dX, void* const* dA,
                      void* const* dB, int flags, void* workspace, size_t ws_bytes, void* hip_stream) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  IndexedLayout L;
  int rc = indexed_layout(p, L);
  if (rc != TLORA_OK) return rc;
  if (!workspace || ws_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return TLORA_EWORKSPACE;
  if (L.T > 0 && (!row_index || !dY || !p->X)) return TLORA_ENULL;
  if (misaligned16(dY) || misaligned16(dX) || misaligned16(p->X)) return TLORA_EALIGN;
  rc = check_arch();
  if (rc != TLORA_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  int32_t* const index = reinterpret_cast<int32_t*>(ws + L.off_idx);
  const bool direct = p->dtype == TLORA_BF16 && direct_index_ok(L.T, std::max(p->d_in, p->d_out));
  tlora_problem_t q = *p;
  if (!direct) q.X = ws + L.off_x;
  rc = indexed_checks(&q, workspace, L.inner, true, dA, dB, flags);
  if (rc != TLORA_OK) return rc;
  if (L.T > 0) {   // made again: the region may have been reused since the forward
    Timed t(TLORA_K_PERMUTE, st);
    launch_clamp_index(row_index, index, L.T, st);
  }
  if (direct) return bwd_impl(p, dY, dX, dA, dB, flags, workspace, L.inner, hip_stream, index, index);
  if (L.T > 0) {
    Timed t(TLORA_K_PERMUTE, st);
    // the sorted activations are gathered again: the region may have been reused since the forward
    launch_permute_rows(p->X, ws + L.off_x, index, L.T, (int64_t)p->d_in * L.elt, false, st);
    launch_permute_rows(dY, ws + L.off_y, index, L.T, (int64_t)p->d_out * L.elt, false, st);
  }
  if (p->dtype == TLORA_BF16 || !dX)
    return bwd_impl(&q, ws + L.off_y, dX, dA, dB, flags, workspace, L.inner, hip_stream, index, nullptr);
  rc = tlora_bwd(&q, ws + L.off_y, ws + L.off_dx, dA, dB, flags, workspace, L.inner, hip_stream);
  if (rc != TLORA_OK) return rc;
  Timed t(TLORA_K_PERMUTE, st);
  launch_permute_rows(ws + L.off_dx, dX, index, L.T, (int64_t)p->d_in * L.elt, true, st);
  return launches_ok(__LINE__);
}

int tlora_plan_dump(const tlora_problem_t* p, int32_t* rpad, int64_t* soff, int32_t* tile_rows, int64_t* tile_row0,
                    int32_t* tile_nrows, int32_t* tile_job_first, int32_t* tile_job_last, int64_t* n_tiles) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  const PlanEntry* e = nullptr;
  const int rc = get_plan(p, false, &e);
  if (rc != TLORA_OK) return rc;
  const Plan& pl = e->pl;
  for (int j = 0; j < pl.J; ++j) {
    if (rpad) rpad[j] = pl.jobs[j].rpad;
    if (soff) soff[j] = pl.jobs[j].soff;
  }
  if (soff) soff[pl.J] = pl.s_elems;
  if (tile_rows) *tile_rows = kGemmBM;
  const int64_t nt = (int64_t)pl.tile_jobs.size();
  if (n_tiles) {
    const int64_t cap = *n_tiles;
    *n_tiles = nt;
    if (cap < nt && (tile_row0 || tile_nrows || tile_job_first || tile_job_last)) return TLORA_EINVAL;
  } else if (tile_row0 || tile_nrows || tile_job_first || tile_job_last) {
    return TLORA_ENULL;
  }
  for (int64_t t = 0; t < nt; ++t) {
    if (tile_row0) tile_row0[t] = t * kGemmBM;
    if (tile_nrows) tile_nrows[t] = (int32_t)std::min<int64_t>(kGemmBM, pl.T - t * kGemmBM);
    if (tile_job_first) tile_job_first[t] = pl.tile_jobs[t].first;
    if (tile_job_last) tile_job_last[t] = pl.tile_jobs[t].last;
  }
  return TLORA_OK;
}

// Host-side consistency check of a freshly built plan: every table entry and every workspace region that a kernel
// will index lies where the kernels assume.  Numbered checks; returns the number of the first one that fails.
static int check_plan(const Plan& pl, bool fwd_only) {
  const bool bf16 = pl.dtype == TLORA_BF16;
  // 1x: jobs
  int64_t soff = 0, atp = 0, roff = 0;
  int row = 0;
  for (int j = 0; j < pl.J; ++j) {
    const JobDev& jb = pl.jobs[j];
    if (jb.row0 != row || jb.row1 < jb.row0) return 10;
    row = jb.row1;
    if (jb.rpad < jb.rank || jb.rpad % kRankGranule || jb.rpad - jb.rank >= kRankGranule) return 11;
    if (jb.soff != soff || jb.atp_off != atp || jb.roff != roff) return 12;
    soff += (int64_t)((jb.row1 - jb.row0 + kGradStep - 1) / kGradStep * kGradStep) * jb.rpad;
    atp += (int64_t)jb.rpad * pl.d_in;
    roff += jb.rpad;
  }
  if (row != pl.T || soff != pl.s_elems || atp != pl.atp_elems || roff != pl.r_total) return 13;
  // 2x: row tiles of the GEMM
  if ((int64_t)pl.tile_jobs.size() != ((int64_t)pl.T + kGemmBM - 1) / kGemmBM) return 20;
  int64_t aoff = 0;
  for (size_t tm = 0; tm < pl.tile_jobs.size(); ++tm) {
    const TileDev& td = pl.tile_jobs[tm];
    const int r0 = (int)tm * kGemmBM, r1 = std::min(pl.T, r0 + kGemmBM);
    if (td.first < 0 || td.last < td.first || td.last >= pl.J) return 21;
    for (int j = 0; j < pl.J; ++j) {          // every job with a row inside the tile lies in first..last
      const JobDev& jb = pl.jobs[j];
      const bool inside = std::max(jb.row0, r0) < std::min(jb.row1, r1);
      if (inside && (j < td.first || j > td.last)) return 22;
    }
    if (td.kext < 0 || td.kext % kGemmBK || td.roff_first != pl.jobs[td.first].roff) return 23;
    if (pl.jobs[td.last].roff + pl.jobs[td.last].rpad > td.roff_first + td.kext) return 24;
    if (td.roff_first + td.kext > pl.r_total + 32) return 25;       // the packed adapters carry 32 spare rank rows
    if (td.aoff != aoff) return 26;
    aoff += (int64_t)kGemmBM * td.kext;
  }
  if (aoff != pl.sx_elems) return 27;
  if (bf16) {
    // 3x: shrink work units tile [row0, row1) x [0, rpad) of every job exactly once
    auto check_shrink = [&](const std::vector<ShrinkUnit>& units, int rows, int cols) -> int {
      std::vector<int64_t> covered(pl.J, 0);
      for (const ShrinkUnit& u : units) {
        if (u.job < 0 || u.job >= pl.J) return 30;
        const JobDev& jb = pl.jobs[u.job];
        if (u.nrows < 1 || u.nrows > rows || u.t0 < jb.row0 || u.t0 + u.nrows > jb.row1) return 31;
        if ((u.t0 - jb.row0) % rows) return 32;
        if (u.pb < 0 || u.pb * cols >= jb.rpad) return 33;
        covered[u.job] += (int64_t)u.nrows * std::min(cols, jb.rpad - u.pb * cols);
      }
      for (int j = 0; j < pl.J; ++j)
        if (covered[j] != (int64_t)(pl.jobs[j].row1 - pl.jobs[j].row0) * pl.jobs[j].rpad) return 34;
      return 0;
    };
    if (pl.shrink_rows != 32 && pl.shrink_rows != 64 && pl.shrink_rows != 128) return 35;
    if (pl.shrink_rows == 32 && (pl.d_in % 64 || pl.d_out % 64)) return 36;
    if (int rc = check_shrink(pl.shrink_units, 64, kShrinkCols)) return rc;
    if (int rc = check_shrink(pl.stream_units, pl.shrink_rows, 128)) return rc + 100;
    // 4x: dA / dB work units and their partial tiles
    auto check_grad = [&](const std::vector<GradUnit>& units, const std::vector<GradGroup>& groups, int64_t partial,
                          int D) -> int {
      const int pb_rows = kGradMaxBlocks * kGradRanks;
      std::vector<std::pair<int64_t, int64_t>> spans;
      for (const GradUnit& u : units) {
        if (u.job < 0 || u.job >= pl.J) return 40;
        const JobDev& jb = pl.jobs[u.job];
        if (u.t0 < jb.row0 || u.t1 <= u.t0 || u.t1 > jb.row1 || u.t1 - u.t0 > kGradMaxTokens) return 41;
        if ((u.t0 - jb.row0) % kGradStep) return 42;                 // the packed S rows are padded to the token step
        if (u.cb < 0 || u.cb * kGradCols >= D || u.pb < 0 || u.pb * pb_rows >= jb.rpad) return 43;
        const int mb = std::min(kGradMaxBlocks, (jb.rpad - u.pb * pb_rows + kGradRanks - 1) / kGradRanks);
        if (u.mb != mb || mb < 1) return 44;
        const int64_t n = (int64_t)mb * kGradRanks * kGradCols;
        if (u.part_off < 0 || u.part_off + n > partial) return 45;
        spans.push_back({u.part_off, n});
      }
      std::sort(spans.begin(), spans.end());
      for (size_t i = 1; i < spans.size(); ++i)
        if (spans[i - 1].first + spans[i - 1].second > spans[i].first) return 46;
      // every output tile (job with a rank, column block, rank block) has one group; its partial tiles are the
      // units of the same (job, cb, pb), consecutive in memory and covering the job's tokens
      int64_t want_groups = 0;
      for (const JobDev& jb : pl.jobs)
        if (jb.rank > 0) want_groups += (int64_t)((jb.rpad + pb_rows - 1) / pb_rows) * ((D + kGradCols - 1) / kGradCols);
      if ((int64_t)groups.size() != want_groups) return 47;
      std::map<std::tuple<int, int, int>, std::vector<const GradUnit*>> by_tile;
      for (const GradUnit& u : units) by_tile[{u.job, u.cb, u.pb}].push_back(&u);
      for (const GradGroup& g : groups) {
        if (g.job < 0 || g.job >= pl.J) return 48;
        const JobDev& jb = pl.jobs[g.job];
        auto& us = by_tile[{g.job, g.cb, g.pb}];
        if ((int)us.size() != g.nunits) return 49;
        std::sort(us.begin(), us.end(), [](const GradUnit* a, const GradUnit* b) { return a->t0 < b->t0; });
        int t = jb.row0;
        for (int k = 0; k < g.nunits; ++k) {
          if (us[k]->t0 != t || us[k]->mb != g.mb) return 50;
          if (us[k]->part_off != g.part_off + (int64_t)k * g.mb * kGradRanks * kGradCols) return 51;
          t = us[k]->t1;
        }
        if (t != jb.row1) return 52;
        if (g.nunits == 0 && jb.row1 != jb.row0) return 53;
      }
      return 0;
    };
    if (!fwd_only) {
      if (int rc = check_grad(pl.gradB_units, pl.gradB_groups, pl.gradB_partial, pl.d_out)) return rc;
      if (int rc = check_grad(pl.gradA_units, pl.gradA_groups, pl.gradA_partial, pl.d_in)) return rc + 100;
    } else if (!pl.gradA_units.empty() || !pl.gradB_units.empty()) {
      return 54;
    }
  }
  // 6x: tables inside the blob, regions inside the workspace, nothing overlapping
  {
    std::vector<std::pair<size_t, size_t>> t = {
        {pl.tb_jobs, sizeof(JobDev) * pl.jobs.size()},          {pl.tb_tiles, sizeof(TileDev) * pl.tile_jobs.size()},
        {pl.tb_shrink, sizeof(ShrinkUnit) * pl.shrink_units.size()}, {pl.tb_stream, sizeof(ShrinkUnit) * pl.stream_units.size()},
        {pl.tb_gBu, sizeof(GradUnit) * pl.gradB_units.size()},  {pl.tb_gBg, sizeof(GradGroup) * pl.gradB_groups.size()},
        {pl.tb_gAu, sizeof(GradUnit) * pl.gradA_units.size()},  {pl.tb_gAg, sizeof(GradGroup) * pl.gradA_groups.size()}};
    if (pl.dtype == TLORA_F32) t.push_back({pl.tb_f32, pl.f32_reserved});
    size_t end = 0;
    for (auto& r : t) {
      if (r.first % 256 || r.first < end) return 60;
      end = r.first + r.second;
    }
    if (end > pl.tables_bytes) return 61;
  }
  {
    std::vector<std::pair<size_t, size_t>> w;
    const size_t se = (size_t)pl.s_elems, sx = 2 * (size_t)pl.sx_elems + 256;
    if (bf16 && !fwd_only) w.push_back({pl.off_wt, 2 * (size_t)pl.d_in * (size_t)pl.d_out});
    w.push_back({pl.off_tables, pl.tables_bytes});
    w.push_back({pl.off_clock, 64});
    if (!bf16) {
      w.push_back({pl.off_S, 4 * se});
      if (!fwd_only) w.push_back({pl.off_dS, 4 * se});
    } else {
      w.push_back({pl.off_Shi, 2 * se});
      w.push_back({pl.off_Slo, 2 * se});
      if (!fwd_only) { w.push_back({pl.off_dShi, 2 * se});  w.push_back({pl.off_dSlo, 2 * se}); }
      w.push_back({pl.off_Sx, sx});
      if (!fwd_only) w.push_back({pl.off_dSx, sx});
      w.push_back({pl.off_atp, 2 * ((size_t)pl.atp_elems + 32 * (size_t)pl.d_in)});
      w.push_back({pl.off_ap, 2 * (size_t)pl.d_in * (size_t)(pl.r_total + 32)});
      w.push_back({pl.off_bp, 2 * (size_t)pl.d_out * (size_t)(pl.r_total + 32)});
      if (!fwd_only) w.push_back({pl.off_partial, 4 * (size_t)std::max(pl.gradB_partial, pl.gradA_partial)});
    }
    size_t end = 0;
    for (auto& r : w) {
      if (r.first % 256 || r.first < end) return 62;
      end = r.first + r.second;
    }
    if (end > pl.total) return 63;
  }
  return 0;
}

int tlora_plan_check(const tlora_problem_t* p, int32_t fwd_only, int32_t* failed_check) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  if (failed_check) *failed_check = 0;
  Plan pl;
  const int rc = build_plan(p, pl, fwd_only != 0);
  if (rc != TLORA_OK) return rc;
  const int bad = check_plan(pl, fwd_only != 0);
  if (failed_check) *failed_check = bad;
  return bad ? TLORA_EINVAL : TLORA_OK;
}

int tlora_profile(int enable) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  const int rc = prof_drain();
  if (enable < 0 || enable > 2) return TLORA_EINVAL;
  g_prof_on = enable != 0;
  g_prof_gemm_only = enable == 2;
  if (g_prof_on) g_clock_slot[0] = g_clock_slot[1] = nullptr;
  if (g_prof_on)
    for (int i = 0; i < TLORA_K_COUNT; ++i) {
      g_prof_ms[i] = 0.0;
      g_prof_n[i] = 0;
    }
  return rc;
}

int tlora_profile_read(int kernel_class, double* total_ms, int64_t* launches) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  if (kernel_class < 0 || kernel_class >= TLORA_K_COUNT) return TLORA_EINVAL;
  const int rc = prof_drain();
  if (rc != TLORA_OK) return rc;
  if (total_ms) *total_ms = g_prof_ms[kernel_class];
  if (launches) *launches = g_prof_n[kernel_class];
  return TLORA_OK;
}

int tlora_profile_clock(double* ghz_fwd, double* ghz_bwd) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  double* out[2] = {ghz_fwd, ghz_bwd};
  for (int i = 0; i < 2; ++i) {
    if (!out[i]) continue;
    *out[i] = 0.0;
    if (!g_clock_slot[i]) continue;
    unsigned long long h[2] = {0, 0};
    TLORA_HIP(hipMemcpy(h, g_clock_slot[i], sizeof(h), hipMemcpyDeviceToHost));
    if (h[1] > 0) *out[i] = (double)h[0] / ((double)h[1] * 10.0);     // cycles per 10 ns tick -> GHz
  }
  return TLORA_OK;
}

int tlora_set_option(const char* name, int64_t value) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  if (!name) return TLORA_ENULL;
  const std::string n(name);
  if (n == "shrink_rows") {
    if (value != 0 && value != 32 && value != 64 && value != 128) return TLORA_EINVAL;
    g_opt.shrink_rows = (int)value;
    return TLORA_OK;
  }
  if (n == "shrink_stages") {
    if (value != 4 && value != 8) return TLORA_EINVAL;
    g_opt.shrink_stages = (int)value;
    return TLORA_OK;
  }
  if (n == "dx_transposed_w") {
    if (value != 0 && value != 1) return TLORA_EINVAL;
    g_opt.dx_transposed_w = (int)value;
    return TLORA_OK;
  }
  if (n == "indexed_direct") {
    if (value != 0 && value != 1) return TLORA_EINVAL;
    g_opt.indexed_direct = (int)value;
    return TLORA_OK;
  }
  if (n == "table_copy_kernel") {
    if (value != 0 && value != 1) return TLORA_EINVAL;
    g_opt.table_copy_kernel = (int)value;
    return TLORA_OK;
  }
  if (n == "plan_cache") {
    if (value != 0 && value != 1) return TLORA_EINVAL;
    g_opt.plan_cache = (int)value;
    g_plans.clear();
    return TLORA_OK;
  }
  if (n == "grad_tokens") {
    if (value < 64 || value % 64 || value > kGradMaxTokens) return TLORA_EINVAL;
    g_opt.grad_tokens = (int)value;
    return TLORA_OK;
  }
  return TLORA_EINVAL;
}

const char* tlora_last_hip_error(void) {
  std::lock_guard<std::recursive_mutex> lk(g_mu);
  static char text[160];
  if (g_hip_err == 0) return "none";
  snprintf(text, sizeof(text), "%s (%d) at line %d of tlora_api.hip", hipGetErrorName((hipError_t)g_hip_err), g_hip_err,
           g_hip_line);
  return text;
}

const char* tlora_strerror(int status) {
  switch (status) {
    case TLORA_OK: return "ok";
    case TLORA_EINVAL: return "invalid problem size, offsets, rank or option";
    case TLORA_ENULL: return "a required pointer is null";
    case TLORA_EDTYPE: return "unsupported dtype";
    case TLORA_EWORKSPACE: return "workspace missing, misaligned or too small";
    case TLORA_EARCH: return "the current device is not gfx950";
    case TLORA_EHIP: return "a HIP runtime call failed";
    case TLORA_EALIGN: return "X, W, Y, dY or dX is not 16-byte aligned";
    case TLORA_ESCRATCH: return "problem too large for the static scratch of tlora_fwd_noalloc";
    default: return "unknown status";
  }
}

const char* tlora_version(void) { return "tlora-gfx950 0.1"; }

}  // extern "C"
