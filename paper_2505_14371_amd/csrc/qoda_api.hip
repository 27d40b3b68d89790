// Host side of libqoda: context, argument checks, device tables, and the order in which the kernels of
// qoda_kernels.hip are enqueued for each C-ABI call declared in include/qoda.h.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/qoda.h"
#include "qoda_kernels.h"

using namespace qoda;

struct qoda_ctx {
  int L = 0, M = 0, K = 0, G = 0;
  int scope = 0;   // NormScope
  int kind = kNormL2;   // NormKind
  int device = 0;  // the device that was current at creation: owns every allocation of the context
  uint64_t seed = 0;
  std::vector<LayerMeta> meta;
  std::vector<int> type_points;
  size_t message_bytes = 0, header_bytes = 0;
  int maxS = 0;
  unsigned int planes_mask = 0;   // bit p set when some layer's code width is p bits
  int maxSP = 0;   // largest 2^(1+b) over the layers: entries of a per-node decode table (indexed by code) in LDS
  // device memory owned by the context
  LayerMeta *d_meta = nullptr;
  int2 *d_tiles = nullptr;
  int4 *d_stiles = nullptr;
  int *d_empty = nullptr;
  int n_empty = 0;
  int GS = 0;
  int *d_type_points = nullptr;
  double *d_partial = nullptr, *d_dpartial = nullptr, *d_sumsq = nullptr, *d_delta = nullptr;
  float *d_norm = nullptr, *d_inv = nullptr, *d_lev = nullptr, *d_rgap = nullptr, *d_eta = nullptr;
  unsigned char *d_lut = nullptr;
  unsigned int *d_hist = nullptr, *d_status = nullptr;
  unsigned long long *d_pooled = nullptr;
  int *d_type_exp = nullptr;
  short *d_dp_arg = nullptr;
  long long *d_dp_arg_off = nullptr;
  int *d_type_exp_next = nullptr;   // bucket scope: the weight scales the next gathering pass will use
  int *d_type_skip = nullptr;       // bucket scope: "no scale" for every type (passes that gather no histogram)
  bool gather = true;               // bucket scope: quantize passes gather the fit's histogram
  unsigned long long *d_index_counts = nullptr;   // [M*256], allocated by the first qoda_index_counts
  // device pointer tables (uploaded when their host shadow changes)
  // A few device copies per table, each remembering the host array it was filled from: a caller that alternates
  // between a few pointer sets (two message buffers per node, say) causes no upload after the first use of each set,
  // so a steady-state round enqueues kernels only and can be captured into a graph.
  struct Table {
    static constexpr int kSlots = 4;
    struct Slot {
      void **dev = nullptr;
      std::vector<void *> host;
      size_t n = 0;
      bool valid = false;
      unsigned long long stamp = 0;
    };
    Slot slots[kSlots];
    int cur = 0;
    unsigned long long clock = 0;
    void **dev() const { return slots[cur].dev; }
    const std::vector<void *> &host() const { return slots[cur].host; }
    bool valid() const { return slots[cur].valid; }
  };
  Table t_grad, t_msg, t_prev, t_in, t_x1, t_y, t_xh, t_xn, t_mean;
  void **d_node_tab = nullptr;   // per-node calls: L layer pointers, then the message and the previous message
  // norms kept by qoda_fit_levels_keep_norms for the quantize calls of the same round on the same vectors
  bool norms_valid = false;
  uint32_t norms_round = 0;
  std::vector<const float *> norms_grad;
  // optional per-kernel event timing
  struct ProfRec { int id; hipEvent_t a, b; };
  unsigned int prof_mask = 0;   // bit i: time kernel class i
  std::vector<ProfRec> prof_recs;
  std::vector<hipEvent_t> prof_pool;
  double prof_ms[kNumKernelIds] = {};
  long long prof_n[kNumKernelIds] = {};
  std::string err;
};

// ---- scratch of qoda_quantize_noalloc: one node's per-tile partial sums, per-layer statistics and pointer tables in a
// file-scope device array instead of the context's allocations.  Every GPU the library runs on holds its own copy
// (about 2.1 MiB) until the process ends.
namespace {
constexpr size_t kNoallocMaxTiles = 1u << 17;     // tiles of 16384 coordinates of one node: 2^31 coordinates
constexpr size_t kNoallocMaxLayers = 4096;
constexpr size_t kOffPartial = 0;                                          // double[tiles]   per-tile statistics
constexpr size_t kOffDpartial = kOffPartial + 8 * kNoallocMaxTiles;        // double[tiles]   per-tile squared distances
constexpr size_t kOffSumsq = kOffDpartial + 8 * kNoallocMaxTiles;          // double[layers]
constexpr size_t kOffNorm = kOffSumsq + 8 * kNoallocMaxLayers;             // float[layers]
constexpr size_t kOffInv = kOffNorm + 4 * kNoallocMaxLayers;               // float[layers]
constexpr size_t kOffTab = kOffInv + 4 * kNoallocMaxLayers;                // pointer[layers + 2] the node's layers, its
                                                                           // message, its previous message
constexpr size_t kScratchBytes = kOffTab + 8 * (kNoallocMaxLayers + 2) + 240;
constexpr int kMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
// In host code `scratch` is only a handle for the symbol; the array's address on each device is looked up once, with
// that device current, and only these addresses are ever handed to kernels.
unsigned char *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

hipError_t scratch_setup(int device) {
  if (device < 0 || device >= kMaxDevices) return hipSuccess;   // such a device has no entry: the entry point says so
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device]) return hipSuccess;
  void *ptr = nullptr;
  const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  g_scratch_ptr[device] = static_cast<unsigned char *>(ptr);
  return hipSuccess;
}

int fail(qoda_ctx *c, int code, const char *fmt, ...) {
  if (c) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    c->err = buf;
  }
  return code;
}

// No exception may cross the C boundary: every entry point that can allocate host memory runs its body through this.
template <class F>
int guarded(qoda_ctx *c, F &&body) {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    if (c) c->err.clear();   // no allocation on this path: the code alone says what happened
    return QODA_ENOMEM;
  } catch (...) {
    // nothing in the library throws anything else on purpose; say so rather than leaving the last message standing
    if (c) {
      try { c->err = "internal exception"; } catch (...) { c->err.clear(); }
    }
    return QODA_EHIP;
  }
}

// The context's buffers live on one device; a call made with another device current would launch there.
int check_device(qoda_ctx *c) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return fail(c, QODA_EHIP, "hipGetDevice failed");
  if (dev != c->device) return fail(c, QODA_EINVAL, "the context was created on device %d but device %d is current", c->device, dev);
  return QODA_OK;
}

#define HIP_TRY(c, call)                                                                        \
  do {                                                                                          \
    hipError_t e_ = (call);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return fail((c), e_ == hipErrorOutOfMemory ? QODA_ENOMEM : QODA_EHIP, "%s: %s", #call,    \
                  hipGetErrorString(e_));                                                       \
  } while (0)

hipError_t prof_event(qoda_ctx *c, hipEvent_t *e) {
  if (!c->prof_pool.empty()) { *e = c->prof_pool.back(); c->prof_pool.pop_back(); return hipSuccess; }
  return hipEventCreate(e);
}

// Enqueue one kernel class; with profiling on, bracket it with two events on the same stream.
#define LAUNCH(c, id, s, call) LAUNCH_IF(c, true, id, s, call)
// The same; with may_time false the launch is never timed (the calls that must not create events).
#define LAUNCH_IF(c, may_time, id, s, call)                                      \
  do {                                                                           \
    qoda_ctx::ProfRec r_{(id), nullptr, nullptr};                                \
    const bool timed_ = (may_time) && (((c)->prof_mask >> (id)) & 1u) != 0u;    \
    if (timed_) {                                                                \
      HIP_TRY((c), prof_event((c), &r_.a));                                      \
      HIP_TRY((c), prof_event((c), &r_.b));                                      \
      HIP_TRY((c), hipEventRecord(r_.a, (s)));                                   \
    }                                                                            \
    HIP_TRY((c), (call));                                                        \
    if (timed_) {                                                                \
      HIP_TRY((c), hipEventRecord(r_.b, (s)));                                   \
      (c)->prof_recs.push_back(r_);                                              \
    }                                                                            \
  } while (0)

int index_bits(int S) {
  int b = 1;
  while ((1 << b) < S) ++b;
  return b;
}

size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

template <class T>
hipError_t dev_alloc(T **p, size_t n) {
  return hipMalloc(reinterpret_cast<void **>(p), (n ? n : 1) * sizeof(T));
}

// Make a table of device pointers current on the device if none of its cached copies holds this set already.
int sync_table(qoda_ctx *c, qoda_ctx::Table &t, const void *const *src, size_t n, hipStream_t s) {
  int victim = 0;
  for (int q = 0; q < qoda_ctx::Table::kSlots; ++q) {
    qoda_ctx::Table::Slot &sl = t.slots[q];
    if (sl.valid && sl.n == n && std::memcmp(sl.host.data(), src, n * sizeof(void *)) == 0) {
      t.cur = q;
      sl.stamp = ++t.clock;
      return QODA_OK;
    }
    if (!sl.valid) victim = q;
    else if (t.slots[victim].valid && sl.stamp < t.slots[victim].stamp) victim = q;
  }
  qoda_ctx::Table::Slot &sl = t.slots[victim];
  sl.host.resize(n);
  std::memcpy(sl.host.data(), src, n * sizeof(void *));   // kept only to recognise the same set next time
  sl.n = n;
  sl.valid = false;
  HIP_TRY(c, launch_stage_pointers(sl.dev, src, n, s));   // through kernel arguments: nothing to wait for
  sl.valid = true;
  sl.stamp = ++t.clock;
  t.cur = victim;
  return QODA_OK;
}

Dev base_args(const qoda_ctx *c) {
  Dev a;
  std::memset(&a, 0, sizeof a);
  a.meta = c->d_meta;
  a.tiles = c->d_tiles;
  a.stiles = c->d_stiles;
  a.empty_layers = c->d_empty;
  a.n_empty = c->n_empty;
  a.GS = c->GS;
  a.L = c->L; a.G = c->G; a.K = c->K; a.M = c->M;
  a.scope = c->scope;
  a.kind = c->kind;
  a.type_points = c->d_type_points;
  a.partial = c->d_partial; a.dpartial = c->d_dpartial; a.sumsq = c->d_sumsq;
  a.norm = c->d_norm; a.inv = c->d_inv; a.delta = c->d_delta;
  a.lev = c->d_lev; a.rgap = c->d_rgap; a.lut = c->d_lut;
  a.hist = c->d_hist; a.pooled = c->d_pooled; a.type_exp = c->d_type_exp;
  a.dp_arg = c->d_dp_arg; a.dp_arg_off = c->d_dp_arg_off;
  a.status = c->d_status; a.eta = c->d_eta;
  a.seed = c->seed;
  a.node0 = 0; a.nnodes = c->K;
  a.invK = 1.0f / (float)c->K;
  a.invK2 = 1.0 / ((double)c->K * (double)c->K);
  return a;
}

int check_layer_ptrs(qoda_ctx *c, const void *const *p, size_t n, const char *what, bool allow_null_for_empty) {
  if (!p) return fail(c, QODA_EINVAL, "%s: null pointer array", what);
  for (size_t i = 0; i < n; ++i) {
    const bool empty = c->meta[i % c->L].d == 0;
    if (!p[i]) {
      if (empty && allow_null_for_empty) continue;
      return fail(c, QODA_EINVAL, "%s[%zu] is null", what, i);
    }
    if (reinterpret_cast<uintptr_t>(p[i]) % 16 != 0) return fail(c, QODA_EINVAL, "%s[%zu] is not 16-byte aligned", what, i);
  }
  return QODA_OK;
}

int check_msg_ptrs(qoda_ctx *c, const void *const *p, size_t n, const char *what, bool allow_null) {
  if (!p) return fail(c, QODA_EINVAL, "%s: null pointer array", what);
  for (size_t i = 0; i < n; ++i) {
    if (!p[i]) {
      if (allow_null) continue;
      return fail(c, QODA_EINVAL, "%s[%zu] is null", what, i);
    }
    if (reinterpret_cast<uintptr_t>(p[i]) % 256 != 0) return fail(c, QODA_EINVAL, "%s[%zu] is not 256-byte aligned", what, i);
  }
  return QODA_OK;
}

void free_all(qoda_ctx *c) {
  void *ptrs[] = {c->d_meta, c->d_tiles, c->d_stiles, c->d_empty, c->d_type_points, c->d_partial, c->d_dpartial, c->d_sumsq, c->d_delta,
                  c->d_norm, c->d_inv, c->d_lev, c->d_rgap, c->d_eta, c->d_lut, c->d_hist, c->d_status, c->d_pooled, c->d_index_counts, c->d_type_exp_next,
                  c->d_type_exp, c->d_dp_arg, c->d_dp_arg_off, c->d_node_tab, c->d_type_skip};
  for (void *p : ptrs)
    if (p) (void)hipFree(p);
  qoda_ctx::Table *tabs[] = {&c->t_grad, &c->t_msg, &c->t_prev, &c->t_in, &c->t_x1, &c->t_y, &c->t_xh, &c->t_xn, &c->t_mean};
  for (qoda_ctx::Table *t : tabs)
    for (auto &sl : t->slots)
      if (sl.dev) (void)hipFree(sl.dev);
  for (auto &r : c->prof_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (hipEvent_t e : c->prof_pool) (void)hipEventDestroy(e);
}

// norms of nodes [node0, node0+n) from the gradient table already on the device
int run_norm_pass(qoda_ctx *c, Dev a, bool with_hist, hipStream_t s) {
  LAUNCH(c, with_hist ? kIdSumsqHist : kIdSumsq, s, launch_sumsq(a, with_hist, s));
  LAUNCH(c, kIdNormFinalize, s, launch_norm_finalize(a, s));
  if (c->scope == kScopeVector) LAUNCH(c, kIdNormVector, s, launch_norm_vector(a, s));
  return QODA_OK;
}

// All nodes in one set of launches, from the K-wide tables already on the device.
int quantize_impl(qoda_ctx *c, int node0, int nnodes, const float *const *grad_full /* K*L */, uint32_t round,
                  hipStream_t s, bool have_prev) {
  Dev a = base_args(c);
  a.grad = reinterpret_cast<const float *const *>(c->t_grad.dev());
  a.msg = reinterpret_cast<unsigned char *const *>(c->t_msg.dev());
  a.prev = have_prev ? reinterpret_cast<const unsigned char *const *>(c->t_prev.dev()) : nullptr;
  a.round = round;
  a.node0 = node0;
  a.nnodes = nnodes;
  bool cached = c->norms_valid && c->norms_round == round;
  if (cached)
    for (int k = node0; k < node0 + nnodes && cached; ++k)
      for (int l = 0; l < c->L; ++l)
        if (c->norms_grad[(size_t)k * c->L + l] != grad_full[(size_t)k * c->L + l]) { cached = false; break; }
  if (c->scope == kScopeBucket && !c->gather) a.type_exp = c->d_type_skip;   // running maxima only, no histogram
  if (c->scope == kScopeBucket) {
    cached = true;   // the bucket norms are computed by the quantize kernel itself, which also gathers the fit's
                     // statistics of these nodes: their histograms and running maxima start from zero
    const size_t n0 = (size_t)node0 * c->L, nn = (size_t)nnodes * c->L;
    LAUNCH(c, kIdZero, s, launch_zero_u32(c->d_hist + n0 * kHistBins, nn * kHistBins, s));
    LAUNCH(c, kIdZero, s, launch_zero_u32(reinterpret_cast<unsigned int *>(c->d_sumsq + n0), 2 * nn, s));
  }
  if (!cached) {
    c->norms_valid = false;   // the cached norms of these nodes are about to be overwritten
    int rc = run_norm_pass(c, a, false, s);
    if (rc) return rc;
  }
  LAUNCH(c, kIdQuantize, s, launch_quantize(a, c->planes_mask, s));
  LAUNCH(c, kIdDeltaFinalize, s, launch_delta_finalize(a, s));
  return QODA_OK;
}

}  // namespace

extern "C" {

// Fills a fresh context from the configuration; on failure the caller releases whatever was allocated so far.
static int create_impl(const qoda_config *cfg, qoda_ctx *c) {
  c->L = cfg->num_layers; c->M = cfg->num_types; c->K = cfg->num_nodes; c->seed = cfg->seed;
  c->scope = cfg->norm_scope;
  c->kind = cfg->norm_kind;
  for (int m = 0; m < c->M; ++m) {
    if (cfg->type_points[m] < 2 || cfg->type_points[m] > QODA_MAX_POINTS) return QODA_EINVAL;
    c->type_points.push_back(cfg->type_points[m]);
  }
  size_t hdr = 0;
  long long chunks = 0;
  c->meta.resize(c->L);
  for (int l = 0; l < c->L; ++l) {
    const long long d = cfg->layer_size[l];
    const int ty = cfg->layer_type[l];
    if (d < 0 || d >= (1ll << 34) || ty < 0 || ty >= c->M) return QODA_EINVAL;
    LayerMeta &m = c->meta[l];
    m.d = d;
    m.type = ty;
    m.S = c->type_points[ty];
    m.planes = 1 + index_bits(m.S);
    m.nblk = (d + kBlockCoords - 1) / kBlockCoords;
    m.hdr_off = (int)hdr;
    hdr += 4 * (size_t)(1 + m.S);
    m.first_chunk = (int)chunks;
    m.nchunks = (int)((d + kChunkCoords - 1) / kChunkCoords);
    chunks += m.nchunks;
    if (m.S > c->maxS) c->maxS = m.S;
    if ((1 << m.planes) > c->maxSP) c->maxSP = 1 << m.planes;
    c->planes_mask |= 1u << m.planes;
    // tiles per node: the decode pass launches up to 8 workgroups per tile in one grid dimension
    if (hdr > (1u << 30) || chunks > (1ll << 28)) return QODA_EINVAL;
  }
  if ((size_t)c->K * c->maxSP * sizeof(float) > 64 * 1024) return QODA_EINVAL;   // decode tables must fit LDS
  c->header_bytes = round_up(hdr, 256);
  size_t off = c->header_bytes;
  for (int l = 0; l < c->L; ++l) {
    c->meta[l].body_off = (long long)off;
    // octets of 8 blocks: planes*256 bytes of codes each, plus the octet's 16 bucket norms under bucket scope
    off += (size_t)((c->meta[l].nblk + 7) / 8) * (256 * c->meta[l].planes + (c->scope == kScopeBucket ? 64 : 0));
  }
  c->message_bytes = round_up(off, 256);
  c->G = (int)chunks;

  std::vector<int2> tiles((size_t)c->G);
  for (int l = 0; l < c->L; ++l)
    for (int ch = 0; ch < c->meta[l].nchunks; ++ch) tiles[(size_t)c->meta[l].first_chunk + ch] = make_int2(l, ch);
  // Runs of tiles for the kernels that keep per-run state (histograms, tables): kSuperTile tiles each, except that in
  // large models the runs shorten towards the end of the table (4, 2, then 1 tile), so that the last workgroups of a
  // launch are short ones and it drains evenly instead of waiting for a last wave of full-length runs.  The table is
  // the same for every node and a launch goes through it node after node, so every node pays the extra flushes of its
  // short runs while only the last node's are the launch's tail: the stretch of single tiles is therefore kept to
  // (workgroups the device holds) / K tiles per node, twice and four times that for the pairs and fours.  A launch of fewer than
  // four device-fills of full-length workgroups keeps full runs throughout: there the extra flushes of the short runs
  // cost more than the tail (measured on 0.4 k tiles per node: +20 % on the norm pass).
  std::vector<int4> stiles;
  {
    const bool large = chunks * c->K >= 4ll * kSuperTile * kTaperWorkgroups;
    const long long T = large ? (kTaperWorkgroups + c->K - 1) / c->K : 0;
    long long before = 0;   // tiles of the layers already listed
    for (int l = 0; l < c->L; ++l) {
      const int n = c->meta[l].nchunks;
      for (int ch = 0; ch < n;) {
        const long long left = chunks - (before + ch);   // tiles from here to the end of the table
        const int want = left <= T ? 1 : left <= 3 * T ? 2 : left <= 7 * T ? 4 : kSuperTile;
        const int len = std::min(want, n - ch);
        stiles.push_back(make_int4(l, ch, len, 0));
        ch += len;
      }
      before += n;
    }
  }
  c->GS = (int)stiles.size();
  std::vector<int> empty;
  for (int l = 0; l < c->L; ++l)
    if (c->meta[l].d == 0) empty.push_back(l);
  c->n_empty = (int)empty.size();
  std::vector<long long> arg_off(c->M);
  long long arg_total = 0;
  for (int m = 0; m < c->M; ++m) { arg_off[m] = arg_total; arg_total += (long long)c->type_points[m] * kGridPoints; }

  const size_t KL = (size_t)c->K * c->L, KG = (size_t)c->K * c->G;
  hipError_t e = hipSuccess;
  auto A = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  A(dev_alloc(&c->d_meta, (size_t)c->L));
  A(dev_alloc(&c->d_tiles, (size_t)c->G));
  A(dev_alloc(&c->d_stiles, (size_t)c->GS));
  A(dev_alloc(&c->d_empty, (size_t)c->n_empty));
  A(dev_alloc(&c->d_type_points, (size_t)c->M));
  A(dev_alloc(&c->d_partial, KG));
  A(dev_alloc(&c->d_dpartial, KG));
  A(dev_alloc(&c->d_sumsq, KL));
  A(dev_alloc(&c->d_delta, (size_t)c->K));
  A(dev_alloc(&c->d_norm, KL));
  A(dev_alloc(&c->d_inv, KL));
  A(dev_alloc(&c->d_lev, (size_t)c->M * kMaxPoints));
  A(dev_alloc(&c->d_rgap, (size_t)c->M * kMaxPoints));
  A(dev_alloc(&c->d_eta, 3));
  A(dev_alloc(&c->d_lut, (size_t)c->M * kLutSize));
  A(dev_alloc(&c->d_status, 2));   // the status word, and a word no kernel result depends on
  A(dev_alloc(&c->d_pooled, (size_t)c->M * kGridPoints));
  A(dev_alloc(&c->d_type_exp, (size_t)c->M));
  if (c->scope == kScopeBucket) {   // the quantize pass gathers the fit's statistics itself
    A(dev_alloc(&c->d_type_exp_next, (size_t)c->M));
    A(dev_alloc(&c->d_type_skip, (size_t)c->M));
    A(dev_alloc(&c->d_hist, KL * kHistBins));
  }
  A(dev_alloc(&c->d_dp_arg, (size_t)arg_total));
  A(dev_alloc(&c->d_dp_arg_off, (size_t)c->M));
  qoda_ctx::Table *tabs[] = {&c->t_grad, &c->t_msg, &c->t_prev, &c->t_in, &c->t_x1, &c->t_y, &c->t_xh, &c->t_xn, &c->t_mean};
  const size_t tab_n[] = {KL, (size_t)c->K, (size_t)c->K, (size_t)c->K, (size_t)c->L, (size_t)c->L, (size_t)c->L, (size_t)c->L, (size_t)c->L};
  for (int i = 0; i < 9; ++i)
    for (auto &sl : tabs[i]->slots) A(dev_alloc(&sl.dev, tab_n[i]));
  A(dev_alloc(&c->d_node_tab, (size_t)c->L + 64));
  if (e == hipSuccess) A(hipMemcpy(c->d_meta, c->meta.data(), c->L * sizeof(LayerMeta), hipMemcpyHostToDevice));
  if (e == hipSuccess && c->G) A(hipMemcpy(c->d_tiles, tiles.data(), c->G * sizeof(int2), hipMemcpyHostToDevice));
  if (e == hipSuccess && c->GS) A(hipMemcpy(c->d_stiles, stiles.data(), c->GS * sizeof(int4), hipMemcpyHostToDevice));
  if (e == hipSuccess && c->n_empty) A(hipMemcpy(c->d_empty, empty.data(), c->n_empty * sizeof(int), hipMemcpyHostToDevice));
  if (e == hipSuccess) A(hipMemcpy(c->d_type_points, c->type_points.data(), c->M * sizeof(int), hipMemcpyHostToDevice));
  if (e == hipSuccess) A(hipMemcpy(c->d_dp_arg_off, arg_off.data(), c->M * sizeof(long long), hipMemcpyHostToDevice));
  if (e == hipSuccess) {   // no weight scale yet: nothing is gathered until a fit has produced one
    const std::vector<int> skip((size_t)c->M, kTypeSkip);
    A(hipMemcpy(c->d_type_exp, skip.data(), c->M * sizeof(int), hipMemcpyHostToDevice));
    if (c->d_type_skip) A(hipMemcpy(c->d_type_skip, skip.data(), c->M * sizeof(int), hipMemcpyHostToDevice));
  }
  if (e == hipSuccess) A(hipMemset(c->d_status, 0, sizeof(unsigned int)));
  if (e == hipSuccess) A(hipMemset(c->d_delta, 0, c->K * sizeof(double)));
  if (e == hipSuccess) A(hipMemset(c->d_pooled, 0, (size_t)c->M * kGridPoints * sizeof(unsigned long long)));
  if (e == hipSuccess) {
    const float one[3] = {1.0f, 1.0f, 1.0f};
    A(hipMemcpy(c->d_eta, one, sizeof one, hipMemcpyHostToDevice));
  }
  if (e != hipSuccess) return e == hipErrorOutOfMemory ? QODA_ENOMEM : QODA_EHIP;
  // uniform initial levels l_j = j / (S - 1)
  for (int m = 0; m < c->M; ++m) {
    const int S = c->type_points[m];
    std::vector<float> lev(S);
    for (int j = 0; j < S; ++j) lev[j] = (float)((double)j / (double)(S - 1));
    lev[S - 1] = 1.0f;
    int rc = qoda_set_levels(c, m, lev.data(), nullptr);
    if (rc != QODA_OK) return rc;
  }
  if (hipDeviceSynchronize() != hipSuccess) return QODA_EHIP;
  return QODA_OK;
}


int qoda_create(const qoda_config *cfg, qoda_ctx **out) {
  if (!out) return QODA_EINVAL;
  *out = nullptr;
  if (!cfg || !cfg->layer_size || !cfg->layer_type || !cfg->type_points) return QODA_EINVAL;
  if (cfg->num_layers < 1 || cfg->num_types < 1 || cfg->num_nodes < 1 || cfg->num_nodes > 65535) return QODA_EINVAL;
  if (cfg->norm_kind != QODA_NORM_L2 && cfg->norm_kind != QODA_NORM_L1 && cfg->norm_kind != QODA_NORM_LINF) return QODA_EINVAL;
  if (cfg->norm_scope < QODA_SCOPE_LAYER || cfg->norm_scope > QODA_SCOPE_BUCKET) return QODA_EINVAL;
  qoda_ctx *c = new (std::nothrow) qoda_ctx;
  if (!c) return QODA_ENOMEM;
  int rc = (hipGetDevice(&c->device) == hipSuccess) ? QODA_OK : QODA_EHIP;
  if (rc == QODA_OK && scratch_setup(c->device) != hipSuccess) rc = QODA_EHIP;
  if (rc == QODA_OK) rc = guarded(c, [&]() -> int {
    c->err.reserve(512);   // as long as fail()'s buffer: recording an error later never allocates
    return create_impl(cfg, c);
  });
  if (rc != QODA_OK) {
    free_all(c);
    delete c;
    return rc;
  }
  *out = c;
  return QODA_OK;
}

int qoda_destroy(qoda_ctx *c) {
  if (!c) return QODA_EINVAL;
  (void)hipDeviceSynchronize();
  free_all(c);
  delete c;
  return QODA_OK;
}

size_t qoda_message_bytes(const qoda_ctx *c) { return c ? c->message_bytes : 0; }

int qoda_message_layout(const qoda_ctx *c, int64_t *hdr_off, int64_t *body_off) {
  if (!c) return QODA_EINVAL;
  for (int l = 0; l < c->L; ++l) {
    if (hdr_off) hdr_off[l] = c->meta[l].hdr_off;
    if (body_off) body_off[l] = c->meta[l].body_off;
  }
  return QODA_OK;
}

int qoda_set_levels(qoda_ctx *c, int32_t type, const float *lev, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (type < 0 || type >= c->M || !lev) return fail(c, QODA_EINVAL, "qoda_set_levels: bad type or null levels");
    const int S = c->type_points[type];
    if (lev[0] != 0.0f || lev[S - 1] != 1.0f) return fail(c, QODA_EINVAL, "qoda_set_levels: levels must start at 0 and end at 1");
    for (int j = 0; j + 1 < S; ++j)
      if (!(lev[j] < lev[j + 1])) return fail(c, QODA_EINVAL, "qoda_set_levels: levels must be strictly increasing");
    hipStream_t s = static_cast<hipStream_t>(stream);
    HIP_TRY(c, launch_stage_words(c->d_lev + (size_t)type * kMaxPoints, lev, (size_t)S, s));
    Dev a = base_args(c);
    LAUNCH(c, kIdBuildTables, s, launch_build_tables(a, type, s));
    return QODA_OK;
  });
}

int qoda_get_levels(qoda_ctx *c, int32_t type, float *lev, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (type < 0 || type >= c->M || !lev) return fail(c, QODA_EINVAL, "qoda_get_levels: bad type or null output");
    hipStream_t s = static_cast<hipStream_t>(stream);
    HIP_TRY(c, hipMemcpyAsync(lev, c->d_lev + (size_t)type * kMaxPoints, c->type_points[type] * sizeof(float),
                              hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    return QODA_OK;
  });
}

static int fit_levels_impl(qoda_ctx *c, const float *const *grad_dev, uint32_t round, void *stream, bool keep_norms) {
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    const size_t KL = (size_t)c->K * c->L;
    if (!grad_dev && c->scope == kScopeBucket) {
      // from the statistics the last quantize pass of every node gathered: pool, fit (with the scale they were gathered
      // under), then the scale for the next pass from the gathered maxima
      hipStream_t s = static_cast<hipStream_t>(stream);
      Dev a = base_args(c);
      a.round = round;
      Dev nx = a;
      nx.type_exp = c->d_type_exp_next;
      LAUNCH(c, kIdFitTypemax, s, launch_fit_typemax(nx, s));   // also clears the pooled weights
      LAUNCH(c, kIdFitPool, s, launch_fit_pool_b(a, s));
      LAUNCH(c, kIdFitDp, s, launch_fit_dp(a, s));
      HIP_TRY(c, hipMemcpyAsync(c->d_type_exp, c->d_type_exp_next, c->M * sizeof(int), hipMemcpyDeviceToDevice, s));
      return QODA_OK;
    }
    int rc = check_layer_ptrs(c, reinterpret_cast<const void *const *>(grad_dev), KL, "qoda_fit_levels: grad_dev", true);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!c->d_hist) HIP_TRY(c, dev_alloc(&c->d_hist, KL * kHistBins));
    rc = sync_table(c, c->t_grad, reinterpret_cast<const void *const *>(grad_dev), KL, s);
    if (rc) return rc;
    c->norms_valid = false;
    Dev a = base_args(c);
    a.grad = reinterpret_cast<const float *const *>(c->t_grad.dev());
    a.round = round;
    LAUNCH(c, kIdZero, s, launch_zero_u32(c->d_hist, KL * kHistBins, s));
    if (c->scope == kScopeBucket) {
      // two passes over the gradient: the scale of the weights, then the weighted histogram
      LAUNCH(c, kIdZero, s, launch_zero_u32(reinterpret_cast<unsigned int *>(c->d_sumsq), 2 * KL, s));
      LAUNCH(c, kIdBucketMax, s, launch_bucket_max(a, s));
      LAUNCH(c, kIdFitTypemax, s, launch_fit_typemax(a, s));
      LAUNCH(c, kIdBucketHist, s, launch_bucket_hist(a, s));
      LAUNCH(c, kIdFitDp, s, launch_fit_dp(a, s));
      return QODA_OK;
    }
    rc = run_norm_pass(c, a, true, s);
    if (rc) return rc;
    LAUNCH(c, kIdFitTypemax, s, launch_fit_typemax(a, s));
    LAUNCH(c, kIdFitPool, s, launch_fit_pool(a, s));
    LAUNCH(c, kIdFitDp, s, launch_fit_dp(a, s));
    if (keep_norms) {   // the caller has declared that these are the vectors the round's quantize calls will be given
      c->norms_grad.assign(grad_dev, grad_dev + KL);
      c->norms_round = round;
      c->norms_valid = true;
    }
    return QODA_OK;
  });
}

int qoda_fit_levels(qoda_ctx *c, const float *const *grad_dev, uint32_t round, void *stream) {
  if (!c) return QODA_EINVAL;
  return fit_levels_impl(c, grad_dev, round, stream, false);
}

int qoda_fit_levels_keep_norms(qoda_ctx *c, const float *const *grad_dev, uint32_t round, void *stream) {
  if (!c) return QODA_EINVAL;
  if (!grad_dev) return fail(c, QODA_EINVAL, "qoda_fit_levels_keep_norms: needs the round's vectors");
  return fit_levels_impl(c, grad_dev, round, stream, true);
}

int qoda_quantize_all(qoda_ctx *c, const float *const *grad_dev, uint32_t round, void *const *msg_dev,
                      const void *const *msg_prev_dev, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    const size_t KL = (size_t)c->K * c->L;
    int rc = check_layer_ptrs(c, reinterpret_cast<const void *const *>(grad_dev), KL, "qoda_quantize_all: grad_dev", true);
    if (rc) return rc;
    rc = check_msg_ptrs(c, reinterpret_cast<const void *const *>(msg_dev), c->K, "qoda_quantize_all: msg_dev", false);
    if (rc) return rc;
    if (msg_prev_dev) {
      rc = check_msg_ptrs(c, msg_prev_dev, c->K, "qoda_quantize_all: msg_prev_dev", true);
      if (rc) return rc;
      for (int k = 0; k < c->K; ++k)
        if (msg_prev_dev[k] == msg_dev[k]) return fail(c, QODA_EINVAL, "qoda_quantize_all: msg_prev_dev[%d] aliases msg_dev", k);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = sync_table(c, c->t_grad, reinterpret_cast<const void *const *>(grad_dev), KL, s);
    if (rc) return rc;
    rc = sync_table(c, c->t_msg, reinterpret_cast<const void *const *>(msg_dev), c->K, s);
    if (rc) return rc;
    if (msg_prev_dev) {
      rc = sync_table(c, c->t_prev, msg_prev_dev, c->K, s);
      if (rc) return rc;
    }
    return quantize_impl(c, 0, c->K, grad_dev, round, s, msg_prev_dev != nullptr);
  });
}

// One node through tables and scratch rows of its own (row0 = node): shared by qoda_quantize (rows of the context's
// buffers, norms may be reused, launches may be timed) and qoda_quantize_noalloc (the static array, neither).
struct NodeBuffers {
  void **tab;   // L layer pointers, then the message pointer, then the previous message pointer
  double *partial, *dpartial, *sumsq;
  float *norm, *inv;
};

static int quantize_node(qoda_ctx *c, int32_t node, const float *const *grad_dev, uint32_t round, void *msg_dev,
                         const void *msg_prev_dev, hipStream_t s, const NodeBuffers &nb, bool of_context,
                         const char *who) {
  char what[96];   // names for the error messages, built on the stack: this path must not allocate
  if (node < 0 || node >= c->K) return fail(c, QODA_EINVAL, "%s: node %d out of range", who, node);
  snprintf(what, sizeof what, "%s: grad_dev", who);
  int rc = check_layer_ptrs(c, reinterpret_cast<const void *const *>(grad_dev), c->L, what, true);
  if (rc) return rc;
  const void *mp[1] = {msg_dev};
  snprintf(what, sizeof what, "%s: msg_dev", who);
  rc = check_msg_ptrs(c, mp, 1, what, false);
  if (rc) return rc;
  const void *pp[1] = {msg_prev_dev};
  snprintf(what, sizeof what, "%s: msg_prev_dev", who);
  rc = check_msg_ptrs(c, pp, 1, what, true);
  if (rc) return rc;
  if (msg_prev_dev == msg_dev) return fail(c, QODA_EINVAL, "%s: msg_prev_dev aliases msg_dev", who);
  // the node's pointers reach the device as kernel arguments: no staging buffer, no copy, nothing to wait for
  HIP_TRY(c, launch_stage_pointers(nb.tab, reinterpret_cast<const void *const *>(grad_dev), (size_t)c->L, s));
  HIP_TRY(c, launch_stage_pointers(nb.tab + c->L, mp, 1, s));
  HIP_TRY(c, launch_stage_pointers(nb.tab + c->L + 1, pp, 1, s));
  Dev a = base_args(c);
  a.grad = reinterpret_cast<const float *const *>(nb.tab);
  a.msg = reinterpret_cast<unsigned char *const *>(nb.tab + c->L);
  a.prev = msg_prev_dev ? reinterpret_cast<const unsigned char *const *>(nb.tab + c->L + 1) : nullptr;
  a.partial = nb.partial;
  a.dpartial = nb.dpartial;
  a.round = round;
  a.node0 = node;
  a.nnodes = 1;
  a.row0 = node;   // the tables and scratch rows above are this node's only
  if (c->scope == kScopeBucket && !c->gather) a.type_exp = c->d_type_skip;   // running maxima only, no histogram
  if (c->scope == kScopeBucket) {
    // the bucket norms are computed by the quantize kernel, which also gathers this node's fit statistics into the
    // context (state of the next fit, not scratch): their histograms and running maxima start from zero
    const size_t n0 = (size_t)node * c->L, nn = (size_t)c->L;
    LAUNCH_IF(c, of_context, kIdZero, s, launch_zero_u32(c->d_hist + n0 * kHistBins, nn * kHistBins, s));
    LAUNCH_IF(c, of_context, kIdZero, s, launch_zero_u32(reinterpret_cast<unsigned int *>(c->d_sumsq + n0), 2 * nn, s));
  } else {
    a.sumsq = nb.sumsq;
    a.norm = nb.norm;
    a.inv = nb.inv;
    bool kept = of_context && c->norms_valid && c->norms_round == round;
    for (int l = 0; l < c->L && kept; ++l) kept = c->norms_grad[(size_t)node * c->L + l] == grad_dev[l];
    if (!kept) {
      if (of_context) c->norms_valid = false;   // this node's kept norms are about to be overwritten
      LAUNCH_IF(c, of_context, kIdSumsq, s, launch_sumsq(a, false, s));
      LAUNCH_IF(c, of_context, kIdNormFinalize, s, launch_norm_finalize(a, s));
      if (c->scope == kScopeVector) LAUNCH_IF(c, of_context, kIdNormVector, s, launch_norm_vector(a, s));
    }
  }
  LAUNCH_IF(c, of_context, kIdQuantize, s, launch_quantize(a, c->planes_mask, s));
  LAUNCH_IF(c, of_context, kIdDeltaFinalize, s, launch_delta_finalize(a, s));
  return QODA_OK;
}

int qoda_quantize(qoda_ctx *c, int32_t node, const float *const *grad_dev, uint32_t round, void *msg_dev,
                  const void *msg_prev_dev, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (node < 0 || node >= c->K) return fail(c, QODA_EINVAL, "qoda_quantize: node %d out of range", node);
    const size_t rowL = (size_t)node * c->L, rowG = (size_t)node * c->G;
    const NodeBuffers nb = {c->d_node_tab, c->d_partial + rowG, c->d_dpartial + rowG, c->d_sumsq + rowL,
                            c->d_norm + rowL, c->d_inv + rowL};
    return quantize_node(c, node, grad_dev, round, msg_dev, msg_prev_dev, static_cast<hipStream_t>(stream), nb, true,
                         "qoda_quantize");
  });
}

int qoda_quantize_noalloc(qoda_ctx *c, int32_t node, const float *const *grad_dev, uint32_t round, void *msg_dev,
                          const void *msg_prev_dev, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if ((size_t)c->L > kNoallocMaxLayers || (size_t)c->G > kNoallocMaxTiles)
      return fail(c, QODA_EINVAL,
                  "qoda_quantize_noalloc: %d layers and %d tiles of 16384 coordinates exceed the static scratch "
                  "(at most %zu layers and %zu tiles per node)", c->L, c->G, kNoallocMaxLayers, kNoallocMaxTiles);
    unsigned char *sp = (c->device >= 0 && c->device < kMaxDevices) ? g_scratch_ptr[c->device] : nullptr;
    if (!sp) return fail(c, QODA_EHIP, "qoda_quantize_noalloc: no static scratch on device %d", c->device);
    const NodeBuffers nb = {reinterpret_cast<void **>(sp + kOffTab), reinterpret_cast<double *>(sp + kOffPartial),
                            reinterpret_cast<double *>(sp + kOffDpartial), reinterpret_cast<double *>(sp + kOffSumsq),
                            reinterpret_cast<float *>(sp + kOffNorm), reinterpret_cast<float *>(sp + kOffInv)};
    return quantize_node(c, node, grad_dev, round, msg_dev, msg_prev_dev, static_cast<hipStream_t>(stream), nb, false,
                         "qoda_quantize_noalloc");
  });
}

static int decode_common(qoda_ctx *c, const void *const *msgs_dev, Dev &a, hipStream_t s, const char *who) {
  int rc = check_msg_ptrs(c, msgs_dev, c->K, who, false);
  if (rc) return rc;
  rc = sync_table(c, c->t_in, msgs_dev, c->K, s);
  if (rc) return rc;
  a.msgs_in = reinterpret_cast<const unsigned char *const *>(c->t_in.dev());
  return QODA_OK;
}

int qoda_dequant_aggregate(qoda_ctx *c, const void *const *msgs_dev, float *const *mean_out_dev, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Dev a = base_args(c);
    int rc = decode_common(c, msgs_dev, a, s, "qoda_dequant_aggregate: msgs_dev");
    if (rc) return rc;
    rc = check_layer_ptrs(c, reinterpret_cast<const void *const *>(mean_out_dev), c->L, "qoda_dequant_aggregate: mean_out_dev", true);
    if (rc) return rc;
    rc = sync_table(c, c->t_mean, reinterpret_cast<const void *const *>(mean_out_dev), c->L, s);
    if (rc) return rc;
    a.mean_out = reinterpret_cast<float *const *>(c->t_mean.dev());
    LAUNCH(c, kIdDecodeMean, s, launch_decode(a, kDecodeMean, c->planes_mask, s));
    return QODA_OK;
  });
}

// Shared by the two step entry points: checks and uploads the K message pointers and the four state tables.
static int step_common(qoda_ctx *c, const void *const *msgs_dev, const float *const *x1, float *const *y,
                       float *const *xh, float *const *xn, Dev &a, hipStream_t s, const char *who) {
  const std::string w(who);
  int rc = decode_common(c, msgs_dev, a, s, (w + ": msgs_dev").c_str());
  if (rc) return rc;
  const struct { const void *const *p; qoda_ctx::Table *t; std::string name; bool optional; } tabs[] = {
      {reinterpret_cast<const void *const *>(x1), &c->t_x1, w + ": x1_dev", false},
      {reinterpret_cast<const void *const *>(y), &c->t_y, w + ": y_dev", false},
      {reinterpret_cast<const void *const *>(xh), &c->t_xh, w + ": x_half_dev", false},
      {reinterpret_cast<const void *const *>(xn), &c->t_xn, w + ": x_next_dev", true}};
  for (const auto &t : tabs) {
    if (!t.p && t.optional) continue;
    rc = check_layer_ptrs(c, t.p, c->L, t.name.c_str(), true);
    if (rc) return rc;
    rc = sync_table(c, *t.t, t.p, c->L, s);
    if (rc) return rc;
  }
  a.x1 = reinterpret_cast<const float *const *>(c->t_x1.dev());
  a.y = reinterpret_cast<float *const *>(c->t_y.dev());
  a.x_half = reinterpret_cast<float *const *>(c->t_xh.dev());
  a.x_next = xn ? reinterpret_cast<float *const *>(c->t_xn.dev()) : nullptr;
  return QODA_OK;
}

int qoda_step(qoda_ctx *c, const void *const *msgs_dev, const qoda_state *st, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (!st || !st->acc_dev) return fail(c, QODA_EINVAL, "qoda_step: null state or accumulator");
    hipStream_t s = static_cast<hipStream_t>(stream);
    Dev a = base_args(c);
    const int rc = step_common(c, msgs_dev, st->x1_dev, st->y_dev, st->x_half_dev, st->x_next_dev, a, s, "qoda_step");
    if (rc) return rc;
    a.acc = st->acc_dev;
    a.eta_out = st->eta_dev;
    LAUNCH(c, kIdStepScalars, s, launch_step_scalars(a, s));
    LAUNCH(c, kIdDecodeUpdate, s, launch_decode(a, kDecodeUpdate, c->planes_mask, s));
    return QODA_OK;
  });
}

int qoda_step_rates(qoda_ctx *c, const void *const *msgs_dev, const qoda_state *st, const float *rates_dev, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (!st || !rates_dev) return fail(c, QODA_EINVAL, "qoda_step_rates: null state or rates");
    hipStream_t s = static_cast<hipStream_t>(stream);
    Dev a = base_args(c);
    const int rc = step_common(c, msgs_dev, st->x1_dev, st->y_dev, st->x_half_dev, st->x_next_dev, a, s, "qoda_step_rates");
    if (rc) return rc;
    a.eta = const_cast<float *>(rates_dev);   // the update kernel only reads its two rates
    LAUNCH(c, kIdDecodeUpdate, s, launch_decode(a, kDecodeUpdate, c->planes_mask, s));
    return QODA_OK;
  });
}

int qoda_index_counts(qoda_ctx *c, const void *const *msgs_dev, uint64_t *counts, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (!counts) return fail(c, QODA_EINVAL, "qoda_index_counts: null output");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t n = (size_t)c->M * 256;
    if (!c->d_index_counts) HIP_TRY(c, dev_alloc(&c->d_index_counts, n));
    Dev a = base_args(c);
    int rc = decode_common(c, msgs_dev, a, s, "qoda_index_counts: msgs_dev");
    if (rc) return rc;
    a.index_counts = c->d_index_counts;
    LAUNCH(c, kIdZero, s, launch_zero_u32(reinterpret_cast<unsigned int *>(c->d_index_counts), 2 * n, s));
    LAUNCH(c, kIdIndexHist, s, launch_index_hist(a, c->planes_mask, s));
    static_assert(sizeof(uint64_t) == sizeof(unsigned long long), "64-bit counters");
    HIP_TRY(c, hipMemcpyAsync(counts, c->d_index_counts, n * sizeof(uint64_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    for (int l = 0; l < c->L; ++l) {   // padding coordinates carry index 0
      const LayerMeta &m = c->meta[l];
      const uint64_t pad = (uint64_t)(((m.nblk + 7) / 8) * 2048 - m.d) * (uint64_t)c->K;
      counts[(size_t)m.type * 256] -= pad;
    }
    return QODA_OK;
  });
}

// Total length of an optimal prefix code for the given occurrence counts: the counts are sorted once, then the two
// lightest subtrees are always at the heads of two queues (leaves in sorted order, merged weights in creation order),
// as App. C.3 notes; every merge adds its weight to the total.
static double huffman_total(const uint64_t *cnt, int n) {
  std::vector<double> leaf;
  for (int j = 0; j < n; ++j)
    if (cnt[j]) leaf.push_back((double)cnt[j]);
  if (leaf.empty()) return 0.0;
  if (leaf.size() == 1) return leaf[0];   // a lone symbol still takes one bit per occurrence
  std::sort(leaf.begin(), leaf.end());
  std::vector<double> merged;
  merged.reserve(leaf.size());
  size_t li = 0, mi = 0;
  double total = 0.0;
  auto take = [&]() {
    if (mi >= merged.size() || (li < leaf.size() && leaf[li] <= merged[mi])) return leaf[li++];
    return merged[mi++];
  };
  const size_t merges = leaf.size() - 1;
  for (size_t q = 0; q < merges; ++q) {
    const double a0 = take();
    const double a1 = take();
    merged.push_back(a0 + a1);
    total += a0 + a1;
  }
  return total;
}

int qoda_code_length(qoda_ctx *c, const uint64_t *counts, uint32_t num_messages, qoda_code_length_report *out) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (!counts || !out) return fail(c, QODA_EINVAL, "qoda_code_length: null argument");
    double norms = 0.0;   // 32-bit norms one message carries
    if (c->scope == kScopeVector) norms = 1.0;
    else
      for (int l = 0; l < c->L; ++l) {
        const long long d = c->meta[l].d;
        if (d == 0) continue;
        norms += (c->scope == kScopeBucket) ? (double)((d + kBucketCoords - 1) / kBucketCoords) : 1.0;
      }
    const double cq = 32.0 * norms * (double)num_messages;
    double fixed = cq, paper = cq, entropy = cq, huff = cq, nonzero = 0.0, coords = 0.0;
    for (int m = 0; m < c->M; ++m) {
      const uint64_t *cm = counts + (size_t)m * 256;
      const int Sm = c->type_points[m];
      double n = 0.0;
      for (int j = 0; j < 256; ++j) n += (double)cm[j];
      if (n == 0.0) continue;
      const double nz = n - (double)cm[0];
      double h_all = 0.0, h_int = 0.0;
      for (int j = 0; j < 256; ++j) {
        if (!cm[j]) continue;
        const double p = (double)cm[j] / n;
        const double t = -p * std::log2(p);
        h_all += t;
        if (j >= 1 && j <= Sm - 2) h_int += t;
      }
      fixed += n * (double)(1 + index_bits(Sm));
      paper += nz + n * (1.0 + h_int);
      entropy += nz + n * h_all;
      huff += nz + huffman_total(cm, 256);
      nonzero += nz;
      coords += n;
    }
    out->fixed_bits = fixed;
    out->paper_bits = paper;
    out->entropy_bits = entropy;
    out->huffman_bits = huff;
    out->nonzeros = nonzero;
    out->coordinates = coords;
    out->message_bits = 8.0 * (double)c->message_bytes * (double)num_messages;
    return QODA_OK;
  });
}

int qoda_extrapolate(qoda_ctx *c, const void *const *msgs_dev, const float *const *x_dev, float *const *out_dev,
                     const float *gamma_dev, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (!gamma_dev) return fail(c, QODA_EINVAL, "qoda_extrapolate: null step size");
    hipStream_t s = static_cast<hipStream_t>(stream);
    Dev a = base_args(c);
    int rc = decode_common(c, msgs_dev, a, s, "qoda_extrapolate: msgs_dev");
    if (rc) return rc;
    rc = check_layer_ptrs(c, reinterpret_cast<const void *const *>(x_dev), c->L, "qoda_extrapolate: x_dev", true);
    if (rc) return rc;
    rc = check_layer_ptrs(c, reinterpret_cast<const void *const *>(out_dev), c->L, "qoda_extrapolate: out_dev", true);
    if (rc) return rc;
    rc = sync_table(c, c->t_x1, reinterpret_cast<const void *const *>(x_dev), c->L, s);
    if (rc) return rc;
    rc = sync_table(c, c->t_xh, reinterpret_cast<const void *const *>(out_dev), c->L, s);
    if (rc) return rc;
    a.x1 = reinterpret_cast<const float *const *>(c->t_x1.dev());
    a.x_half = reinterpret_cast<float *const *>(c->t_xh.dev());
    a.gamma_in = gamma_dev;
    LAUNCH(c, kIdDecodeExtrapolate, s, launch_decode(a, kDecodeExtrapolate, c->planes_mask, s));
    return QODA_OK;
  });
}

int qoda_step_alt(qoda_ctx *c, const void *const *msgs_dev, const qoda_alt_state *st, double q_hat, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (!st || !st->sums_dev || !st->eta_dev) return fail(c, QODA_EINVAL, "qoda_step_alt: null state, sums or rates");
    if (!(q_hat > 0.0) || !(q_hat <= 0.25)) return fail(c, QODA_EINVAL, "qoda_step_alt: the exponent must lie in (0, 1/4]");
    const double digits = std::floor(std::ldexp(q_hat, 32));
    if (digits < 1.0) return fail(c, QODA_EINVAL, "qoda_step_alt: the exponent is below 2^-32");
    // this pass keeps a 2 KiB reduction buffer in shared memory beside the K decode tables
    if ((size_t)c->K * c->maxSP * sizeof(float) + kThreads * sizeof(double) > 64 * 1024)
      return fail(c, QODA_EINVAL, "qoda_step_alt: K * 2^(1+b) = %zu exceeds 15872 (decode tables plus the reduction "
                                  "buffer of this pass must fit 64 KiB of shared memory)", (size_t)c->K * c->maxSP);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Dev a = base_args(c);
    const int rc = step_common(c, msgs_dev, st->x1_dev, st->y_dev, st->x_half_dev, st->x_next_dev, a, s, "qoda_step_alt");
    if (rc) return rc;
    a.alt_sums = st->sums_dev;
    a.eta_out = st->eta_dev;
    a.q_digits = (unsigned int)digits;
    LAUNCH(c, kIdAltScalars, s, launch_alt_scalars(a, s));
    LAUNCH(c, kIdDecodeAlt, s, launch_decode(a, kDecodeUpdateAlt, c->planes_mask, s));
    LAUNCH(c, kIdAltFinalize, s, launch_alt_finalize(a, s));
    return QODA_OK;
  });
}

int qoda_read_buffer(qoda_ctx *c, int32_t which, void *dst, size_t bytes, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (!dst) return fail(c, QODA_EINVAL, "qoda_read_buffer: null destination");
    const size_t KL = (size_t)c->K * c->L;
    const void *src = nullptr;
    size_t have = 0;
    switch (which) {
      case QODA_BUF_SUMSQ: src = c->d_sumsq; have = KL * sizeof(double); break;
      case QODA_BUF_NORM: src = c->d_norm; have = KL * sizeof(float); break;
      case QODA_BUF_INV: src = c->d_inv; have = KL * sizeof(float); break;
      case QODA_BUF_DELTA: src = c->d_delta; have = c->K * sizeof(double); break;
      case QODA_BUF_HIST: src = c->d_hist; have = c->d_hist ? KL * kHistBins * sizeof(unsigned int) : 0; break;
      case QODA_BUF_POOLED: src = c->d_pooled; have = (size_t)c->M * kGridPoints * sizeof(unsigned long long); break;
      default: return fail(c, QODA_EINVAL, "qoda_read_buffer: unknown buffer %d", which);
    }
    if (!src || bytes != have) return fail(c, QODA_EINVAL, "qoda_read_buffer: buffer %d holds %zu bytes, asked for %zu", which, have, bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    HIP_TRY(c, hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    return QODA_OK;
  });
}

int qoda_status(qoda_ctx *c, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned int flag = 0;
    HIP_TRY(c, hipMemcpyAsync(&flag, c->d_status, sizeof flag, hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    if (flag) {
      HIP_TRY(c, launch_zero_u32(c->d_status, 1, s));
      if (flag & 1u) return fail(c, QODA_ENONFINITE, "a vector's norm statistic was not a finite number in range");
      return fail(c, QODA_ETINYNORM, "a vector's norm was positive but below 2^-126: its reciprocal is not a float");
    }
    return QODA_OK;
  });
}

int qoda_gather_statistics(qoda_ctx *c, int32_t enable) {
  if (!c) return QODA_EINVAL;
  c->gather = enable != 0;
  return QODA_OK;
}

int qoda_profile_enable(qoda_ctx *c, uint32_t class_mask) {
  if (!c) return QODA_EINVAL;
  c->prof_mask = class_mask;
  return QODA_OK;
}

int qoda_profile_read(qoda_ctx *c, double *ms, int64_t *launches, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (!ms || !launches) return fail(c, QODA_EINVAL, "qoda_profile_read: null output");
    HIP_TRY(c, hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    for (auto &r : c->prof_recs) {
      float t = 0.0f;
      HIP_TRY(c, hipEventSynchronize(r.b));
      HIP_TRY(c, hipEventElapsedTime(&t, r.a, r.b));
      c->prof_ms[r.id] += (double)t;
      c->prof_n[r.id] += 1;
      c->prof_pool.push_back(r.a);
      c->prof_pool.push_back(r.b);
    }
    c->prof_recs.clear();
    for (int i = 0; i < kNumKernelIds; ++i) {
      ms[i] = c->prof_ms[i];
      launches[i] = c->prof_n[i];
      c->prof_ms[i] = 0.0;
      c->prof_n[i] = 0;
    }
    return QODA_OK;
  });
}

const char *qoda_kernel_name(int32_t id) {
  static const char *names[kNumKernelIds] = {"k_zero_u32", "k_sumsq<false>", "k_sumsq<true>", "k_norm_finalize",
                                             "(unused)", "k_quantize", "k_delta_finalize", "k_step_scalars",
                                             "k_decode<false>", "k_decode<true>", "k_fit_typemax", "k_fit_pool",
                                             "k_fit_dp", "k_build_tables", "k_copy_f4", "k_alt_scalars",
                                             "k_decode<alt>", "k_alt_finalize", "k_norm_vector", "k_bucket_max",
                                             "k_bucket_hist", "k_decode<extrapolate>", "k_index_hist", "k_stream"};
  return (id >= 0 && id < kNumKernelIds) ? names[id] : "";
}

int qoda_copy_calibration(qoda_ctx *c, const void *src_dev, void *dst_dev, size_t bytes, void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    if (!src_dev || !dst_dev || bytes % 16 != 0 || reinterpret_cast<uintptr_t>(src_dev) % 16 != 0 ||
        reinterpret_cast<uintptr_t>(dst_dev) % 16 != 0)
      return fail(c, QODA_EINVAL, "qoda_copy_calibration: pointers and size must be multiples of 16 bytes");
    hipStream_t s = static_cast<hipStream_t>(stream);
    LAUNCH(c, kIdCopy, s, launch_copy(src_dev, dst_dev, bytes, s));
    return QODA_OK;
  });
}

int qoda_stream_calibration(qoda_ctx *c, const void *src_dev, void *dst_dev, size_t bytes, int32_t stores_per_16_loads,
                            void *stream) {
  if (!c) return QODA_EINVAL;
  return guarded(c, [&]() -> int {
    if (const int rc_ = check_device(c)) return rc_;
    const int w = stores_per_16_loads;
    if (!src_dev || !dst_dev || bytes % 65536 != 0 || reinterpret_cast<uintptr_t>(src_dev) % 16 != 0 ||
        reinterpret_cast<uintptr_t>(dst_dev) % 16 != 0 || !(w == 0 || w == 1 || w == 2 || w == 4 || w == 8 || w == 16))
      return fail(c, QODA_EINVAL, "qoda_stream_calibration: 16-byte aligned pointers, a multiple of 65536 bytes and "
                                  "0, 1, 2, 4, 8 or 16 stores per 16 loads");
    hipStream_t s = static_cast<hipStream_t>(stream);
    LAUNCH(c, kIdStream, s, launch_stream(src_dev, dst_dev, bytes, w, c->d_status + 1, s));
    return QODA_OK;
  });
}

const char *qoda_last_error(const qoda_ctx *c) { return c ? c->err.c_str() : "null context"; }

}  // extern "C"
