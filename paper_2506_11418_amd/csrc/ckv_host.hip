// Host driver of libckv: argument validation, the rounds schedule (Algorithm 1's loop after
// prefill), workspace carving, kernel sequencing and optional per-kernel timing.
#include <math.h>
#include <string.h>

#include <string>
#include <vector>

#include "ckv_internal.h"

namespace ckv {
namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
int elem_bytes(int dtype) { return dtype == CKV_BF16 ? 2 : 4; }

int check_layout(const ckv_layout* l) {
  if (!l) return CKV_EINVAL;
  if (l->dtype != CKV_F32 && l->dtype != CKV_BF16) return CKV_EINVAL;
  if (l->batch <= 0 || l->heads <= 0 || l->seq <= 0 || l->dim <= 0) return CKV_ESHAPE;
  if (l->stride_s < l->dim || l->stride_h < l->dim || l->stride_b < l->dim) return CKV_ESHAPE;
  if ((int64_t)l->batch * l->heads > (1 << 24)) return CKV_ESHAPE;
  if (l->deg_stride != 0 && l->deg_stride < l->seq) return CKV_ESHAPE;
  const int e = elem_bytes(l->dtype);
  if ((l->stride_s * e) % 16 || (l->stride_h * e) % 16 || (l->stride_b * e) % 16 || (l->dim * e) % 16)
    return CKV_EALIGN;
  return CKV_OK;
}

// bytes spanned by a tensor with this layout, from its base pointer
size_t extent_bytes(const ckv_layout* l, int seq) {
  const int64_t last = (int64_t)(l->batch - 1) * l->stride_b + (int64_t)(l->heads - 1) * l->stride_h +
                       (int64_t)(seq - 1) * l->stride_s + l->dim;
  return (size_t)last * elem_bytes(l->dtype);
}

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + nb && y < x + na;
}

bool dims_supported(int dtype, int dim) {
  if (dtype == CKV_BF16) return dim == 64 || dim == 128;
  return dim == 16 || dim == 32 || dim == 64 || dim == 128;
}

int64_t deg_stride_of(const ckv_layout* l) { return l->deg_stride ? l->deg_stride : l->seq; }
TensorView view_of(const ckv_layout* l) {
  return TensorView{l->stride_b, l->stride_h, l->stride_s, l->heads, deg_stride_of(l)};
}
TensorView compact_view(int heads, int len, int dim) {
  return TensorView{(int64_t)heads * len * dim, (int64_t)len * dim, (int64_t)dim, heads, (int64_t)len};
}

// [lo, hi): the tokens of a cache of `len` tokens that take part in the clustering; the first n_sink
// and the last n_recent are set aside (Sec. 5.2).  Nothing is clustered when len <= n_sink+n_recent.
void clusterable(int len, int n_sink, int n_recent, int* lo, int* hi) {
  if (len <= n_sink + n_recent) { *lo = 0; *hi = 0; return; }
  *lo = n_sink;
  *hi = len - n_recent;
}

int seq_after_round(int len, int chunk, float r, int n_sink, int n_recent, int scope) {
  int lo, hi;
  clusterable(len, n_sink, n_recent, &lo, &hi);
  const int mid = hi - lo;
  const int full = mid / chunk, tail = mid % chunk;
  if (scope == CKV_SCOPE_HEAD) {   // one ranking over the edges of all chunks
    const int edges = full * (chunk / 2) + (tail >= 2 ? (tail + 1) / 2 : 0);
    return len - merge_count(r, edges);
  }
  return (len - mid) + full * chunk_out(chunk, r) + chunk_out(tail, r);
}

// How each round of a schedule runs.  FULL: match + merge writing keys, values and degrees.
// A deferred pair: when round j merges every edge (r = 1) and another round follows, round j may
// write keys and degrees only (KEYS_ONLY) and round j+1 rebuild the value rows it needs from round
// j's value input (ORIGIN); the intermediate value cache is then neither written nor read, and
// the result is the same bit for bit.  A pair is taken at the start of a schedule or at its end,
// not in between: the staging buffers alternate, so the second round of a pair that starts at round
// j >= 1 reads value and degree input from the very buffers (same parity) a non-final round j+1
// writes.  It pays once the second round has enough workgroups (one per chunk, each rebuilding the
// values of 2*chunk original tokens) to fill the chip: from about 4 per CU on MI355X (measured
// crossover at 1024 chunks); smaller jobs run every round in full unless the caller's flags say
// otherwise.
enum RoundMode { ROUND_FULL = 0, ROUND_KEYS_ONLY = 1, ROUND_ORIGIN = 2 };
constexpr int64_t kDeferMinChunks = 1024;

void plan_routes(const ckv_layout* in, const ckv_params* p, const ckv_plan_t* plan, RoundMode (&mode)[CKV_MAX_ROUNDS]) {
  const int64_t n_bh = (int64_t)in->batch * in->heads;
  const bool allow = !(p->flags & CKV_ROUTE_FULL_ROUNDS), force = (p->flags & CKV_ROUTE_DEFER_ALWAYS) != 0;
  for (int j = 0; j < CKV_MAX_ROUNDS; ++j) mode[j] = ROUND_FULL;
  for (int j = 0; j + 1 < plan->n_rounds; ++j) {
    int lo, hi;
    clusterable(plan->round_len[j], p->n_sink, p->n_recent, &lo, &hi);
    int lo2, hi2;   // both rounds must have tokens to cluster (a cache of sinks and recents only is copied)
    clusterable(plan->round_len[j + 1], p->n_sink, p->n_recent, &lo2, &hi2);
    const bool pair = allow && (j == 0 || j + 2 == plan->n_rounds) && plan->round_r[j] == 1.0f &&
                      p->scope == CKV_SCOPE_CHUNK && hi > lo && hi2 > lo2 &&
                      (force || n_bh * div_up(plan->round_len[j + 1], p->chunk) >= kDeferMinChunks);
    if (pair) {
      mode[j] = ROUND_KEYS_ONLY;
      mode[j + 1] = ROUND_ORIGIN;
      ++j;   // the pair's second round cannot open another pair
    }
  }
}

struct Workspace {
  size_t dst, score, sel, lists, map, K[2], V[2], deg[2], total;
};

Workspace carve(const ckv_layout* in, const ckv_params* p, const ckv_plan_t* plan) {
  Workspace w{};
  const int chunk = p->chunk;
  const size_t n_bh = (size_t)in->batch * in->heads;
  const size_t e = elem_bytes(in->dtype);
  RoundMode mode[CKV_MAX_ROUNDS];
  plan_routes(in, p, plan, mode);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t n_src0 = n_sources(in->seq, chunk);
  w.dst = take(n_bh * n_src0 * 4);
  w.score = take(n_bh * n_src0 * 4);
  if (p->scope == CKV_SCOPE_HEAD) w.sel = take(n_bh * (size_t)div_up(in->seq, chunk) * 8);
  const int inter = plan->n_rounds - 1;   // intermediate caches
  if (inter >= 1) w.map = take(n_bh * (size_t)plan->round_len[1] * 4);
  // member lists a keys-only merge hands to the next round (3 int16 per source of a chunk)
  bool any_pair = false;
  for (int j = 0; j < plan->n_rounds; ++j) any_pair |= mode[j] == ROUND_KEYS_ONLY;
  if (any_pair) w.lists = take(n_bh * (size_t)div_up(in->seq, chunk) * 3 * (chunk / 2) * 2);
  // Rounds alternate between two staging caches.  A staging VALUE cache that only keys-only rounds
  // would write holds nothing but the sink / recent rows, which those rounds still copy: without
  // sinks and recents it is left out (at the full-model 128k shape that is 4 GiB).
  for (int k = 0; k < 2 && k < inter; ++k) {
    size_t len = 0;
    bool values = false;
    for (int j = k; j < inter; j += 2) {
      len = len > (size_t)plan->round_len[j + 1] ? len : (size_t)plan->round_len[j + 1];
      values |= mode[j] != ROUND_KEYS_ONLY || p->n_sink + p->n_recent > 0;
    }
    w.K[k] = take(n_bh * len * in->dim * e);
    w.V[k] = values ? take(n_bh * len * in->dim * e) : w.K[k];
    w.deg[k] = take(n_bh * len * 4);
  }
  w.total = off;
  return w;
}

int make_plan(const ckv_layout* in, const ckv_params* p, ckv_plan_t* plan) {
  int st = check_layout(in);
  if (st != CKV_OK) return st;
  if (!p || !plan) return CKV_EINVAL;
  if (p->chunk < 2 || p->chunk > 2048 || (p->chunk & 1)) return CKV_EINVAL;
  if (p->n_sink < 0 || p->n_recent < 0) return CKV_EINVAL;
  if (p->scope != CKV_SCOPE_CHUNK && p->scope != CKV_SCOPE_HEAD) return CKV_EINVAL;
  if (p->flags & ~(uint32_t)(CKV_ROUTE_FULL_ROUNDS | CKV_ROUTE_DEFER_ALWAYS)) return CKV_EINVAL;
  if ((p->flags & CKV_ROUTE_FULL_ROUNDS) && (p->flags & CKV_ROUTE_DEFER_ALWAYS)) return CKV_EINVAL;
  if (p->n_rounds < 0 || p->n_rounds > CKV_MAX_ROUNDS) return CKV_EINVAL;
  memset(plan, 0, sizeof(*plan));
  if (p->n_rounds > 0) {
    plan->n_rounds = p->n_rounds;
    for (int j = 0; j < p->n_rounds; ++j) {
      if (!(p->r[j] >= 0.f && p->r[j] <= 1.f)) return CKV_EINVAL;
      plan->round_r[j] = p->r[j];
    }
  } else {
    const double rho = (double)p->retain_ratio;
    if (!(rho > 0.0 && rho <= 1.0)) return CKV_EINVAL;
    int J = 0;
    while (ldexp(1.0, -J) > rho * (1.0 + 1e-6)) ++J;
    if (J > CKV_MAX_ROUNDS) return CKV_EINVAL;
    plan->n_rounds = J;
    for (int j = 0; j < J; ++j) plan->round_r[j] = 1.0f;
    if (J > 0) plan->round_r[J - 1] = (float)(2.0 * (1.0 - rho * ldexp(1.0, J - 1)));
  }
  plan->round_len[0] = in->seq;
  for (int j = 0; j < plan->n_rounds; ++j)
    plan->round_len[j + 1] = seq_after_round(plan->round_len[j], p->chunk, plan->round_r[j], p->n_sink, p->n_recent,
                                             p->scope);
  plan->out_seq = plan->round_len[plan->n_rounds];
  plan->workspace_bytes = carve(in, p, plan).total;
  return CKV_OK;
}

int hip_status(hipError_t e) {
  if (e == hipSuccess) return CKV_OK;
  (void)hipGetLastError();
  return (e == hipErrorInvalidValue) ? CKV_EUNSUPPORTED : CKV_EHIP;
}

// ---- timing --------------------------------------------------------------------------------
struct TimedLaunch {
  const char* name;
  hipEvent_t a, b;
};
bool g_timing = false;
std::string g_timing_prefix;          // empty: every kernel; else only names that start with it
std::vector<TimedLaunch> g_launches;
std::vector<std::pair<std::string, std::pair<double, int64_t>>> g_totals;

void fold_launches() {
  for (auto& t : g_launches) {
    float ms = 0.f;
    if (hipEventSynchronize(t.b) == hipSuccess && hipEventElapsedTime(&ms, t.a, t.b) == hipSuccess) {
      bool found = false;
      for (auto& kv : g_totals)
        if (kv.first == t.name) { kv.second.first += ms; kv.second.second += 1; found = true; break; }
      if (!found) g_totals.push_back({t.name, {ms, 1}});
    }
    (void)hipEventDestroy(t.a);
    (void)hipEventDestroy(t.b);
  }
  g_launches.clear();
  (void)hipGetLastError();
}


// A paged call: the cache lives in block pools (K, V, deg_in of run_rounds are then the pools) and
// the result goes back into the sequences' own first blocks.  Only the first round reads the pools;
// the last round writes a pool directly when no workgroup of that round still reads it, and into a
// staging tensor (scattered afterwards) otherwise: with a single round everything is staged; when the
// schedule is one deferred pair the last round rebuilds its value rows from the ORIGINAL values and
// degrees, so those two are staged while the keys, which that round takes from the first round's
// output, go straight to their pool.
struct PagedCall {
  PagedSide side;            // table (at the first sequence of the call), max_blocks, shift, n_blocks; tok0 = 0
  void *sK, *sV;             // staging tensors [batch, heads, out_seq, dim] (only those that are needed)
  int32_t* sdeg;
  bool stage_k, stage_v;     // out: which outputs went to staging
};

// The rounds of one compression (Algorithm 1, the loop after prefill), launches only.
int run_rounds(const void* K, const void* V, const int32_t* deg_in, const ckv_layout* in, const ckv_params* p,
               const ckv_plan_t* planp, void* K_out, void* V_out, int32_t* deg_out, const ckv_layout* out,
               int32_t* assign, void* workspace, PagedCall* pc, hipStream_t s) {
  const ckv_plan_t& plan = *planp;
  const int n_bh = in->batch * in->heads;
  const int e = in->dtype == CKV_BF16 ? 2 : 4;
  const Workspace w = carve(in, p, &plan);
  RoundMode mode[CKV_MAX_ROUNDS];
  plan_routes(in, p, &plan, mode);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  int32_t* dst = reinterpret_cast<int32_t*>(ws + w.dst);
  float* score = reinterpret_cast<float*>(ws + w.score);
  const void* curK = K;
  const void* curV = V;
  const int32_t* curDeg = deg_in;
  TensorView curView = view_of(in);
  int16_t* lists = reinterpret_cast<int16_t*>(ws + w.lists);
  ValueOrigin org{};
  const void* edgesV = V;   // where the current cache's sink / recent value rows live
  if (pc) {
    pc->stage_k = plan.n_rounds == 1;
    pc->stage_v = plan.n_rounds == 1 || (plan.n_rounds == 2 && mode[0] == ROUND_KEYS_ONLY);
  }
  for (int j = 0; j < plan.n_rounds; ++j) {
    const int len = plan.round_len[j];
    const int next = plan.round_len[j + 1];
    const bool last = (j == plan.n_rounds - 1);
    int lo, hi;
    clusterable(len, p->n_sink, p->n_recent, &lo, &hi);
    const int mid = hi - lo;
    // which sides of this round's launches are block pools
    PagedSide pin{}, pok{}, pov{}, pin0{}, pok0{}, pov0{};   // (…0: the same with token offset 0, for whole-sequence kernels)
    if (pc && j == 0) { pin = pc->side; pin.tok0 = lo; pin0 = pc->side; }
    if (pc && last && !pc->stage_k) { pok = pc->side; pok.tok0 = lo; pok0 = pc->side; }
    if (pc && last && !pc->stage_v) { pov = pc->side; pov.tok0 = lo; pov0 = pc->side; }
    const TensorView stView = compact_view(in->heads, next, in->dim);
    void* oK = !last ? ws + w.K[j & 1] : !pc ? K_out : pc->stage_k ? pc->sK : const_cast<void*>(K);
    void* oV = !last ? ws + w.V[j & 1] : !pc ? V_out : pc->stage_v ? pc->sV : const_cast<void*>(V);
    int32_t* oDeg = !last ? reinterpret_cast<int32_t*>(ws + w.deg[j & 1])
                    : !pc ? deg_out : pc->stage_v ? pc->sdeg : const_cast<int32_t*>(deg_in);
    const TensorView oView = (last && !pc) ? view_of(out) : stView;
    const int64_t oDegStride = oView.deg_stride;
    int32_t* map = nullptr;
    if (assign) map = (j == 0) ? assign : reinterpret_cast<int32_t*>(ws + w.map);
    const bool keys_only = mode[j] == ROUND_KEYS_ONLY, from_origin = mode[j] == ROUND_ORIGIN;
    hipError_t err = hipSuccess;
    if (mid > 0) {   // cluster tokens [lo, hi): the same kernels on a view that starts at token lo
      const bool in_pool = pin.table != nullptr;
      const unsigned char* mK = static_cast<const unsigned char*>(curK) + (in_pool ? 0 : (size_t)lo * curView.stride_s * e);
      const unsigned char* mV = static_cast<const unsigned char*>(curV) + (in_pool ? 0 : (size_t)lo * curView.stride_s * e);
      const int32_t* mDeg = !curDeg ? nullptr : in_pool ? curDeg : curDeg + lo;
      err = launch_match(mK, in->dtype, in->dim, curView, n_bh, mid, p->chunk, dst, score, s, pin);
      if (err != hipSuccess) return hip_status(err);
      int32_t* sel = nullptr;
      if (p->scope == CKV_SCOPE_HEAD) {
        sel = reinterpret_cast<int32_t*>(ws + w.sel);
        err = launch_global_select(score, n_bh, mid, p->chunk, plan.round_r[j], sel, s);
        if (err != hipSuccess) return hip_status(err);
      }
      unsigned char* moK = static_cast<unsigned char*>(oK) + (pok.table ? 0 : (size_t)lo * oView.stride_s * e);
      unsigned char* moV = static_cast<unsigned char*>(oV) + (pov.table ? 0 : (size_t)lo * oView.stride_s * e);
      int32_t* moDeg = pov.table ? oDeg : oDeg + lo;
      err = launch_merge(mK, mV, mDeg, in->dtype, in->dim, curView, n_bh, mid, p->chunk, plan.round_r[j], dst, score,
                         moK, moV, moDeg, oView, oDegStride, map ? map + lo : nullptr, curView.deg_stride, len, lo, sel,
                         keys_only ? lists : nullptr, from_origin ? &org : nullptr, s, pin, pok, pov);
      if (err != hipSuccess) return hip_status(err);
    }
    if (mid < len)   // sinks and recents (or a cache too short to cluster): straight copy
      err = launch_edges(curK, edgesV, curDeg, curView, len, oK, oV, oDeg, oView, oDegStride, next, map,
                         mid > 0 ? lo : len, mid > 0 ? len - hi : 0, n_bh, in->dim * e, e, s, pin0, pok0, pov0);
    if (err != hipSuccess) return hip_status(err);
    if (assign && j > 0) {
      err = launch_compose(assign, map, n_bh, in->seq, len, s);
      if (err != hipSuccess) return hip_status(err);
    }
    if (keys_only) {   // the clustered values stay where they are; the next round reads them through the lists
      const bool in_pool = pin.table != nullptr;
      org = ValueOrigin{static_cast<const unsigned char*>(curV) + (in_pool ? 0 : (size_t)lo * curView.stride_s * e), curView,
                        !curDeg ? nullptr : in_pool ? curDeg : curDeg + lo, lists, mid, div_up(mid, p->chunk), pin};
    } else {
      curV = oV;
    }
    edgesV = oV;       // sinks and recents are copied in every round, deferred or not
    curK = oK; curDeg = oDeg; curView = oView;
  }
  return CKV_OK;
}

}  // namespace

bool timing_begin(const char* name, hipStream_t st) {
  if (!g_timing) return false;
  if (!g_timing_prefix.empty() && strncmp(name, g_timing_prefix.c_str(), g_timing_prefix.size()) != 0) return false;
  TimedLaunch t{name, nullptr, nullptr};
  if (hipEventCreate(&t.a) != hipSuccess) return false;
  if (hipEventCreate(&t.b) != hipSuccess) {
    (void)hipEventDestroy(t.a);
    return false;
  }
  (void)hipEventRecord(t.a, st);
  g_launches.push_back(t);
  return true;
}

void timing_end(hipStream_t st) {
  if (g_launches.empty()) return;
  (void)hipEventRecord(g_launches.back().b, st);
}

}  // namespace ckv

using namespace ckv;

extern "C" {

const char* ckv_version(void) { return "ckv 0.1 (gfx950)"; }

const char* ckv_strerror(int status) {
  switch (status) {
    case CKV_OK: return "ok";
    case CKV_EINVAL: return "invalid argument";
    case CKV_ESHAPE: return "invalid shape or stride";
    case CKV_EALIGN: return "pointer or stride not 16-byte aligned";
    case CKV_EWORKSPACE: return "workspace too small";
    case CKV_EUNSUPPORTED: return "unsupported configuration";
    case CKV_EHIP: return "HIP runtime error";
  }
  return "unknown status";
}

int ckv_plan(const ckv_layout* in, const ckv_params* p, ckv_plan_t* plan) { return make_plan(in, p, plan); }

int ckv_match(const void* K, const ckv_layout* in, int32_t chunk, int32_t* dst, float* score, void* hip_stream) {
  int st = check_layout(in);
  if (st != CKV_OK) return st;
  if (!K || !dst || !score) return CKV_EINVAL;
  if (chunk < 2 || chunk > 2048 || (chunk & 1)) return CKV_EINVAL;
  if (((uintptr_t)K) % 16 || ((uintptr_t)dst) % 4 || ((uintptr_t)score) % 4) return CKV_EALIGN;
  if (!dims_supported(in->dtype, in->dim)) return CKV_EUNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int n_bh = in->batch * in->heads;
  hipError_t e = launch_match(K, in->dtype, in->dim, view_of(in), n_bh, in->seq, chunk, dst, score, s);
  if (e != hipSuccess) return hip_status(e);
  return hip_status(launch_dst_positions(dst, dst, n_bh, in->seq, chunk, s));
}

int ckv_compress(const void* K, const void* V, const int32_t* deg_in, const ckv_layout* in, const ckv_params* p,
                 void* K_out, void* V_out, int32_t* deg_out, const ckv_layout* out, int32_t* assign,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  ckv_plan_t plan;
  int st = make_plan(in, p, &plan);
  if (st != CKV_OK) return st;
  st = check_layout(out);
  if (st != CKV_OK) return st;
  if (!K || !V || !K_out || !V_out || !deg_out) return CKV_EINVAL;
  if (out->batch != in->batch || out->heads != in->heads || out->dim != in->dim || out->dtype != in->dtype)
    return CKV_ESHAPE;
  if (out->seq < plan.out_seq) return CKV_ESHAPE;
  if (((uintptr_t)K) % 16 || ((uintptr_t)V) % 16 || ((uintptr_t)K_out) % 16 || ((uintptr_t)V_out) % 16 ||
      ((uintptr_t)deg_out) % 4 || ((uintptr_t)deg_in) % 4 || ((uintptr_t)assign) % 4)
    return CKV_EALIGN;
  if (!dims_supported(in->dtype, in->dim)) return CKV_EUNSUPPORTED;
  if (plan.workspace_bytes > 0) {
    if (!workspace) return CKV_EINVAL;
    if (((uintptr_t)workspace) % 256) return CKV_EALIGN;
    if (workspace_bytes < plan.workspace_bytes) return CKV_EWORKSPACE;
  }
  {
    const size_t in_b = extent_bytes(in, in->seq), out_b = extent_bytes(out, plan.out_seq);
    const void* ins[2] = {K, V};
    const void* outs[2] = {K_out, V_out};
    for (auto o : outs) {
      for (auto i : ins)
        if (overlaps(o, out_b, i, in_b)) return CKV_EINVAL;
      if (plan.workspace_bytes && overlaps(o, out_b, workspace, plan.workspace_bytes)) return CKV_EINVAL;
    }
    if (overlaps(K_out, out_b, V_out, out_b)) return CKV_EINVAL;
    if (plan.workspace_bytes)
      for (auto i : ins)
        if (overlaps(workspace, plan.workspace_bytes, i, in_b)) return CKV_EINVAL;
  }

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int n_bh = in->batch * in->heads;
  const int e = in->dtype == CKV_BF16 ? 2 : 4;
  if (plan.n_rounds == 0) {
    hipError_t err = launch_copy_rows(K, view_of(in), K_out, view_of(out), n_bh, in->seq, in->dim * e, e, s);
    if (err == hipSuccess)
      err = launch_copy_rows(V, view_of(in), V_out, view_of(out), n_bh, in->seq, in->dim * e, e, s);
    if (err == hipSuccess)
      err = launch_fill_deg(deg_in, deg_stride_of(in), deg_out, deg_stride_of(out), assign, n_bh, in->seq, s);
    return hip_status(err);
  }

  return run_rounds(K, V, deg_in, in, p, &plan, K_out, V_out, deg_out, out, assign, workspace, nullptr, s);
}

int32_t ckv_n_sources(int32_t seq, int32_t chunk) {
  if (seq < 0) return CKV_ESHAPE;
  if (chunk < 2 || chunk > 2048 || (chunk & 1)) return CKV_EINVAL;
  return n_sources(seq, chunk);
}

int32_t ckv_budget_tokens(float cache_ratio, int32_t n) {
  if (!(cache_ratio > 0.f && cache_ratio <= 1.f)) return CKV_EINVAL;
  if (n < 0) return CKV_ESHAPE;
  return (int32_t)((double)cache_ratio * (double)n + 1e-9);
}

int ckv_schedule_annealed(int32_t seq, int32_t chunk, int32_t n_sink, int32_t n_recent, int32_t scope,
                          int32_t budget, float r_init, float delta_r, float r_floor, ckv_params* out) {
  if (scope != CKV_SCOPE_CHUNK && scope != CKV_SCOPE_HEAD) return CKV_EINVAL;
  if (!out || seq <= 0 || budget < 0 || n_sink < 0 || n_recent < 0) return CKV_EINVAL;
  if (chunk < 2 || chunk > 2048 || (chunk & 1)) return CKV_EINVAL;
  if (!(r_init >= 0.f && r_init <= 1.f) || !(delta_r >= 0.f) || !(r_floor >= 0.f && r_floor <= 1.f)) return CKV_EINVAL;
  memset(out, 0, sizeof(*out));
  out->chunk = chunk;
  out->retain_ratio = 1.0f;
  out->n_sink = n_sink;
  out->n_recent = n_recent;
  out->scope = scope;
  int len = seq, j = 0;
  while (len > budget) {
    if (j == CKV_MAX_ROUNDS) return CKV_EUNSUPPORTED;
    const double want = (double)r_init - (double)j * (double)delta_r;
    const float r = (float)(want > (double)r_floor ? want : (double)r_floor);
    const int next = seq_after_round(len, chunk, r, n_sink, n_recent, scope);
    if (next == len) return CKV_EUNSUPPORTED;   // the schedule has run dry above the budget
    out->r[j++] = r;
    len = next;
  }
  out->n_rounds = j;
  return CKV_OK;
}

int ckv_append(const void* k_new, const void* v_new, void* K, void* V, int32_t* deg, const ckv_layout* cache,
               int32_t* lens, int32_t pos, void* hip_stream) {
  int st = check_layout(cache);
  if (st != CKV_OK) return st;
  if (!k_new || !v_new || !K || !V) return CKV_EINVAL;
  if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)K | (uintptr_t)V) % 16) return CKV_EALIGN;
  if (!lens && (pos < 0 || pos >= cache->seq)) return CKV_ESHAPE;
  const int e = elem_bytes(cache->dtype);
  return hip_status(launch_append(k_new, v_new, K, V, deg, view_of(cache), cache->batch, cache->seq, lens, pos,
                                  cache->dim * e, e, static_cast<hipStream_t>(hip_stream)));
}

int ckv_decode_attn_workspace(const ckv_layout* kv, int32_t q_heads, size_t* bytes) {
  int st = check_layout(kv);
  if (st != CKV_OK) return st;
  if (!bytes) return CKV_EINVAL;
  if (q_heads <= 0 || q_heads % kv->heads) return CKV_ESHAPE;
  *bytes = align_up(attn_workspace_bytes(kv->batch, kv->heads, q_heads, kv->dim, kv->seq, 0), 256);
  return CKV_OK;
}

int ckv_decode_attn(const void* q, int32_t q_heads, const void* K, const void* V, const ckv_layout* kv,
                    const int32_t* lens, const int32_t* deg, float scale, void* o, int32_t o_dtype,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  size_t need = 0;
  int st = ckv_decode_attn_workspace(kv, q_heads, &need);
  if (st != CKV_OK) return st;
  if (!q || !K || !V || !o || !workspace) return CKV_EINVAL;
  if (o_dtype != CKV_F32 && o_dtype != CKV_BF16) return CKV_EINVAL;
  if (((uintptr_t)q) % 16 || ((uintptr_t)K) % 16 || ((uintptr_t)V) % 16 || ((uintptr_t)o) % 4 ||
      ((uintptr_t)workspace) % 16 || ((uintptr_t)lens) % 4 || ((uintptr_t)deg) % 4)
    return CKV_EALIGN;
  if (workspace_bytes < need) return CKV_EWORKSPACE;
  const int G = q_heads / kv->heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return CKV_EUNSUPPORTED;
  if (kv->dtype == CKV_BF16 ? !(kv->dim == 64 || kv->dim == 128)
                            : !(kv->dim == 32 || kv->dim == 64 || kv->dim == 128))
    return CKV_EUNSUPPORTED;
  if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)kv->dim);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  return hip_status(launch_decode_attn(q, q_heads, K, V, kv->dtype, kv->dim, view_of(kv), kv->batch, kv->heads,
                                       kv->seq, lens, deg, scale, o, o_dtype, workspace, PagedView{nullptr, 0, 0, 0},
                                       s));
}

// ---- block-paged caches ------------------------------------------------------------------------
namespace {
int check_paged(const ckv_paged_layout* pl, int* shift) {
  if (!pl) return CKV_EINVAL;
  if (pl->dtype != CKV_F32 && pl->dtype != CKV_BF16) return CKV_EINVAL;
  if (pl->batch <= 0 || pl->heads <= 0 || pl->dim <= 0 || pl->max_blocks <= 0 || pl->n_blocks <= 0) return CKV_ESHAPE;
  if (pl->block_size < 1 || pl->block_size > 1024 || (pl->block_size & (pl->block_size - 1))) return CKV_ESHAPE;
  if ((int64_t)pl->max_blocks * pl->block_size > INT32_MAX) return CKV_ESHAPE;
  if ((pl->dim * ckv::elem_bytes(pl->dtype)) % 16) return CKV_EALIGN;
  int sh = 0;
  while ((1 << sh) < pl->block_size) ++sh;
  *shift = sh;
  return CKV_OK;
}
// the strided layout of a compact [batch, heads, seq, dim] staging tensor
ckv_layout staging_layout(const ckv_paged_layout* pl, int seq) {
  ckv_layout l{};
  l.batch = pl->batch; l.heads = pl->heads; l.seq = seq; l.dim = pl->dim; l.dtype = pl->dtype;
  l.stride_s = pl->dim; l.stride_h = (int64_t)seq * pl->dim; l.stride_b = (int64_t)pl->heads * seq * pl->dim;
  l.deg_stride = 0;
  return l;
}
ckv::TensorView pool_view(const ckv_paged_layout* pl) {
  return ckv::TensorView{0, (int64_t)pl->block_size * pl->dim, (int64_t)pl->dim, pl->heads, 0};
}
}  // namespace

int ckv_paged_decode_attn_workspace(const ckv_paged_layout* pl, int32_t q_heads, int32_t max_len, size_t* bytes) {
  int shift;
  int st = check_paged(pl, &shift);
  if (st != CKV_OK) return st;
  if (!bytes) return CKV_EINVAL;
  if (max_len <= 0 || q_heads <= 0 || q_heads % pl->heads) return CKV_ESHAPE;
  const int limit = ckv::attn_paged_span_limit(pl->block_size);
  if ((int64_t)limit * 1024 < max_len) return CKV_EUNSUPPORTED;   // more table entries per slice than the kernel holds
  if ((int64_t)pl->n_blocks * pl->heads * pl->block_size > INT32_MAX) return CKV_EUNSUPPORTED;   // pool rows are indexed in 32 bits
  *bytes = ckv::align_up(ckv::attn_workspace_bytes(pl->batch, pl->heads, q_heads, pl->dim, max_len, limit), 256);
  return CKV_OK;
}

int ckv_paged_decode_attn(const void* q, int32_t q_heads, const void* K_pool, const void* V_pool,
                          const int32_t* deg_pool, const int32_t* block_table, const int32_t* lens,
                          const ckv_paged_layout* pl, int32_t max_len, float scale, void* o, int32_t o_dtype,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  size_t need = 0;
  int st = ckv_paged_decode_attn_workspace(pl, q_heads, max_len, &need);
  if (st != CKV_OK) return st;
  if (!q || !K_pool || !V_pool || !block_table || !lens || !o || !workspace) return CKV_EINVAL;
  if (o_dtype != CKV_F32 && o_dtype != CKV_BF16) return CKV_EINVAL;
  if (((uintptr_t)q) % 16 || ((uintptr_t)K_pool) % 16 || ((uintptr_t)V_pool) % 16 || ((uintptr_t)o) % 4 ||
      ((uintptr_t)workspace) % 16 || ((uintptr_t)lens) % 4 || ((uintptr_t)deg_pool) % 4 ||
      ((uintptr_t)block_table) % 4)
    return CKV_EALIGN;
  if (workspace_bytes < need) return CKV_EWORKSPACE;
  const int G = q_heads / pl->heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return CKV_EUNSUPPORTED;
  if (pl->dtype == CKV_BF16 ? !(pl->dim == 64 || pl->dim == 128) : !(pl->dim == 32 || pl->dim == 64 || pl->dim == 128))
    return CKV_EUNSUPPORTED;
  if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)pl->dim);
  int shift;
  check_paged(pl, &shift);
  const int64_t cap = (int64_t)pl->max_blocks * pl->block_size;
  const int seq = (int)(max_len < cap ? max_len : cap);
  return ckv::hip_status(ckv::launch_decode_attn(q, q_heads, K_pool, V_pool, pl->dtype, pl->dim, pool_view(pl), pl->batch,
                                                 pl->heads, seq, lens, deg_pool, scale, o, o_dtype, workspace,
                                                 ckv::PagedView{block_table, pl->max_blocks, shift, pl->n_blocks},
                                                 static_cast<hipStream_t>(hip_stream)));
}

int ckv_paged_append(const void* k_new, const void* v_new, void* K_pool, void* V_pool, int32_t* deg_pool,
                     const int32_t* block_table, int32_t* lens, const ckv_paged_layout* pl, void* hip_stream) {
  int shift;
  int st = check_paged(pl, &shift);
  if (st != CKV_OK) return st;
  if (!k_new || !v_new || !K_pool || !V_pool || !block_table || !lens) return CKV_EINVAL;
  if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)K_pool | (uintptr_t)V_pool) % 16) return CKV_EALIGN;
  const int e = ckv::elem_bytes(pl->dtype);
  return ckv::hip_status(ckv::launch_paged_append(k_new, v_new, K_pool, V_pool, deg_pool,
                                                  ckv::PagedView{block_table, pl->max_blocks, shift, pl->n_blocks},
                                                  pl->batch, pl->heads, pl->dim * e, lens,
                                                  static_cast<hipStream_t>(hip_stream)));
}

int ckv_paged_gather(const void* K_pool, const void* V_pool, const int32_t* deg_pool, const int32_t* block_table,
                     const ckv_paged_layout* pl, int32_t seq, void* K, void* V, int32_t* deg,
                     const ckv_layout* out, void* hip_stream) {
  int shift;
  int st = check_paged(pl, &shift);
  if (st == CKV_OK) st = ckv::check_layout(out);
  if (st != CKV_OK) return st;
  if (!K_pool || !V_pool || !block_table || !K || !V) return CKV_EINVAL;
  if (out->batch != pl->batch || out->heads != pl->heads || out->dim != pl->dim || out->dtype != pl->dtype) return CKV_ESHAPE;
  if (seq <= 0 || seq > out->seq || (int64_t)seq > (int64_t)pl->max_blocks * pl->block_size) return CKV_ESHAPE;
  if (((uintptr_t)K_pool | (uintptr_t)V_pool | (uintptr_t)K | (uintptr_t)V) % 16) return CKV_EALIGN;
  const int e = ckv::elem_bytes(pl->dtype);
  return ckv::hip_status(ckv::launch_paged_gather(K_pool, V_pool, deg_pool,
                                                  ckv::PagedView{block_table, pl->max_blocks, shift, pl->n_blocks},
                                                  pl->batch, pl->heads, seq, pl->dim * e, K, V, deg, ckv::view_of(out), e,
                                                  static_cast<hipStream_t>(hip_stream)));
}

int ckv_paged_scatter(const void* K, const void* V, const int32_t* deg, const ckv_layout* in, void* K_pool,
                      void* V_pool, int32_t* deg_pool, int32_t* block_table, const ckv_paged_layout* pl,
                      int32_t old_seq, int32_t* freed, int32_t* lens, void* hip_stream) {
  int shift;
  int st = check_paged(pl, &shift);
  if (st == CKV_OK) st = ckv::check_layout(in);
  if (st != CKV_OK) return st;
  if (!K_pool || !V_pool || !block_table || !K || !V) return CKV_EINVAL;
  if (in->batch != pl->batch || in->heads != pl->heads || in->dim != pl->dim || in->dtype != pl->dtype) return CKV_ESHAPE;
  const int64_t cap = (int64_t)pl->max_blocks * pl->block_size;
  if (old_seq < in->seq || old_seq > cap) return CKV_ESHAPE;
  if (((uintptr_t)K_pool | (uintptr_t)V_pool | (uintptr_t)K | (uintptr_t)V) % 16) return CKV_EALIGN;
  const int e = ckv::elem_bytes(pl->dtype);
  const int keep = ckv::div_up(in->seq, pl->block_size), old_blocks = ckv::div_up(old_seq, pl->block_size);
  return ckv::hip_status(ckv::launch_paged_scatter(K, V, deg, ckv::view_of(in), pl->batch, pl->heads, in->seq, pl->dim * e, e,
                                                   K_pool, V_pool, deg_pool, block_table, pl->max_blocks, shift,
                                                   pl->n_blocks, keep, old_blocks, freed, old_blocks - keep, lens,
                                                   static_cast<hipStream_t>(hip_stream)));
}

int32_t ckv_paged_freed_blocks(const ckv_paged_layout* pl, int32_t old_seq, int32_t new_seq) {
  int shift;
  int st = check_paged(pl, &shift);
  if (st != CKV_OK) return st;
  if (new_seq < 0 || old_seq < new_seq || (int64_t)old_seq > (int64_t)pl->max_blocks * pl->block_size) return CKV_ESHAPE;
  return ckv::div_up(old_seq, pl->block_size) - ckv::div_up(new_seq, pl->block_size);
}

namespace {
// Workspace of a paged compression: staging for the outputs the last round cannot write in place
// (see PagedCall), then ckv_compress's own workspace.  Sequences are processed in runs of equal
// length, one after the other, so the sizes are those of the largest run.
struct PagedWs { size_t sK, sV, sdeg, inner, total; };
struct PagedRun { int b0, n, seq; };

// maximal runs of neighbouring sequences with equal length
int paged_runs(const ckv_paged_layout* pl, int32_t seq, const int32_t* seq_lens, PagedRun* runs) {
  int n = 0;
  for (int b = 0; b < pl->batch; ++b) {
    const int len = seq_lens ? seq_lens[b] : seq;
    if (n > 0 && runs[n - 1].seq == len) ++runs[n - 1].n;
    else runs[n++] = PagedRun{b, 1, len};
  }
  return n;
}

ckv_paged_layout run_layout(const ckv_paged_layout* pl, const PagedRun& r) {
  ckv_paged_layout x = *pl;
  x.batch = r.n;
  return x;
}

int paged_run_plan(const ckv_paged_layout* pl, const PagedRun& run, const ckv_params* p, ckv_plan_t* plan, PagedWs* w) {
  if (run.seq <= 0 || (int64_t)run.seq > (int64_t)pl->max_blocks * pl->block_size) return CKV_ESHAPE;
  const ckv_paged_layout rl = run_layout(pl, run);
  const ckv_layout in = staging_layout(&rl, run.seq);
  int st = ckv_plan(&in, p, plan);
  if (st != CKV_OK) return st;
  RoundMode mode[CKV_MAX_ROUNDS];
  plan_routes(&in, p, plan, mode);
  const bool stage_k = plan->n_rounds == 1;
  const bool stage_v = plan->n_rounds == 1 || (plan->n_rounds == 2 && mode[0] == ROUND_KEYS_ONLY);
  const size_t e = ckv::elem_bytes(pl->dtype), n_bh = (size_t)run.n * pl->heads;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = ckv::align_up(off + bytes, 256); return o; };
  w->sK = take(stage_k ? n_bh * plan->out_seq * pl->dim * e : 0);
  w->sV = take(stage_v ? n_bh * plan->out_seq * pl->dim * e : 0);
  w->sdeg = take(stage_v ? n_bh * plan->out_seq * 4 : 0);
  w->inner = take(plan->workspace_bytes);
  w->total = off;
  return CKV_OK;
}

int check_paged_compress(const ckv_paged_layout* pl, int32_t seq, const int32_t* seq_lens) {
  int shift;
  int st = check_paged(pl, &shift);
  if (st != CKV_OK) return st;
  if (pl->block_size < 8) return CKV_EUNSUPPORTED;          // the kernels' block tables hold blocks of 8 tokens or more
  if ((int64_t)pl->n_blocks * pl->heads * pl->block_size > INT32_MAX) return CKV_EUNSUPPORTED;   // pool rows are indexed in 32 bits
  if (pl->batch > 4096) return CKV_ESHAPE;
  if (!seq_lens && (seq <= 0 || (int64_t)seq > (int64_t)pl->max_blocks * pl->block_size)) return CKV_ESHAPE;
  return CKV_OK;
}
}  // namespace

int ckv_paged_compress_plan(const ckv_paged_layout* pl, int32_t seq, const int32_t* seq_lens, const ckv_params* p,
                            int32_t* out_seq, int32_t* n_freed, size_t* workspace_bytes) {
  int st = check_paged_compress(pl, seq, seq_lens);
  if (st != CKV_OK) return st;
  std::vector<PagedRun> runs(pl->batch);
  const int n_runs = paged_runs(pl, seq, seq_lens, runs.data());
  size_t need = 0;
  int freed_max = 0;
  for (int i = 0; i < n_runs; ++i) {
    ckv_plan_t plan;
    PagedWs w;
    st = paged_run_plan(pl, runs[i], p, &plan, &w);
    if (st != CKV_OK) return st;
    need = w.total > need ? w.total : need;
    const int nf = ckv::div_up(runs[i].seq, pl->block_size) - ckv::div_up(plan.out_seq, pl->block_size);
    freed_max = nf > freed_max ? nf : freed_max;
    if (out_seq) {
      if (seq_lens) for (int b = 0; b < runs[i].n; ++b) out_seq[runs[i].b0 + b] = plan.out_seq;
      else out_seq[0] = plan.out_seq;
    }
  }
  if (n_freed) *n_freed = freed_max;
  if (workspace_bytes) *workspace_bytes = need;
  return CKV_OK;
}

int ckv_paged_compress(void* K_pool, void* V_pool, int32_t* deg_pool, int32_t* block_table, int32_t* lens,
                       const ckv_paged_layout* pl, int32_t seq, const int32_t* seq_lens, const ckv_params* p,
                       int32_t* freed, int32_t freed_stride, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = check_paged_compress(pl, seq, seq_lens);
  if (st != CKV_OK) return st;
  if (!K_pool || !V_pool || !deg_pool || !block_table || !workspace) return CKV_EINVAL;
  if (((uintptr_t)K_pool | (uintptr_t)V_pool) % 16 || ((uintptr_t)deg_pool | (uintptr_t)block_table | (uintptr_t)freed |
                                                        (uintptr_t)lens) % 4)
    return CKV_EALIGN;
  if (((uintptr_t)workspace) % 256) return CKV_EALIGN;
  if (!dims_supported(pl->dtype, pl->dim)) return CKV_EUNSUPPORTED;
  int32_t n_freed_max = 0;
  size_t need = 0;
  st = ckv_paged_compress_plan(pl, seq, seq_lens, p, nullptr, &n_freed_max, &need);
  if (st != CKV_OK) return st;
  if (workspace_bytes < need) return CKV_EWORKSPACE;
  if (freed && freed_stride < n_freed_max) return CKV_ESHAPE;
  int shift;
  check_paged(pl, &shift);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  std::vector<PagedRun> runs(pl->batch);
  const int n_runs = paged_runs(pl, seq, seq_lens, runs.data());
  const int e = ckv::elem_bytes(pl->dtype);
  for (int i = 0; i < n_runs; ++i) {
    const PagedRun& run = runs[i];
    ckv_plan_t plan;
    PagedWs w;
    st = paged_run_plan(pl, run, p, &plan, &w);
    if (st != CKV_OK) return st;
    int32_t* table = block_table + (size_t)run.b0 * pl->max_blocks;
    int32_t* run_freed = freed ? freed + (size_t)run.b0 * freed_stride : nullptr;
    int32_t* run_lens = lens ? lens + run.b0 : nullptr;
    const ckv_paged_layout rl = run_layout(pl, run);
    const ckv_layout in = staging_layout(&rl, run.seq), stg = staging_layout(&rl, plan.out_seq);
    PagedCall pc{};
    pc.side.table = table;
    pc.side.max_blocks = pl->max_blocks;
    pc.side.shift = shift;
    pc.side.n_blocks = pl->n_blocks;
    pc.sK = ws + w.sK;
    pc.sV = ws + w.sV;
    pc.sdeg = reinterpret_cast<int32_t*>(ws + w.sdeg);
    if (plan.n_rounds > 0) {
      st = run_rounds(K_pool, V_pool, deg_pool, &in, p, &plan, nullptr, nullptr, nullptr, &stg, nullptr, ws + w.inner, &pc, s);
      if (st != CKV_OK) return st;
    }
    // staged outputs into the sequences' first blocks, then the blocks behind the new length are released
    const int keep = ckv::div_up(plan.out_seq, pl->block_size), old_blocks = ckv::div_up(run.seq, pl->block_size);
    hipError_t err = ckv::launch_paged_scatter(
        (plan.n_rounds > 0 && pc.stage_k) ? pc.sK : nullptr, (plan.n_rounds > 0 && pc.stage_v) ? pc.sV : nullptr,
        (plan.n_rounds > 0 && pc.stage_v) ? pc.sdeg : nullptr, ckv::view_of(&stg), run.n, pl->heads, plan.out_seq, pl->dim * e, e,
        K_pool, V_pool, deg_pool, table, pl->max_blocks, shift, pl->n_blocks, keep, old_blocks, run_freed, freed_stride,
        run_lens, s);
    if (err != hipSuccess) return ckv::hip_status(err);
  }
  return CKV_OK;
}

int ckv_timing_enable(int on) {
  if (!on) fold_launches();
  g_timing = on != 0;
  return CKV_OK;
}

int ckv_timing_select(const char* prefix) {
  g_timing_prefix = prefix ? prefix : "";
  return CKV_OK;
}

int ckv_timing_reset(void) {
  fold_launches();
  g_totals.clear();
  return CKV_OK;
}

int ckv_timing_read(ckv_kernel_time* out, int max) {
  fold_launches();
  int n = 0;
  for (auto& kv : g_totals) {
    if (out && n < max) {
      memset(&out[n], 0, sizeof(out[n]));
      strncpy(out[n].name, kv.first.c_str(), sizeof(out[n].name) - 1);
      out[n].total_ms = kv.second.first;
      out[n].launches = kv.second.second;
    }
    ++n;
  }
  return n;
}

}  // extern "C"
