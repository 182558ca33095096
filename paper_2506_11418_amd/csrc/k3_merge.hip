// Top-r selection, degree-weighted merge and order-preserving compaction of one clustering round
// (Sec. 5.3: candidate edges are ranked by similarity and only the best fraction r is merged; the
// centroid equation; values merged with the same weights).
//
// One workgroup per (sequence, chunk).  Integer bookkeeping lives in LDS:
//   keep[i]      source i is among the m = floor(r*|A|) best edges (score desc, index asc);
//   members[]    kept sources grouped by destination, ascending inside a group (rank by counting:
//                no atomics decide an order, so results are run-to-run identical);
//   local_out[]  prefix sum over retained tokens (all B tokens, unkept A tokens).
// Rows are then produced gather-style: 16-byte pieces, one row per group of row_bytes/16 lanes,
// fp32 accumulation for bf16 (fp64 for fp32 storage), one rounding to the storage type.
#include <type_traits>

#include "ckv_internal.h"
#include "ckv_device.h"

namespace ckv {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxHalf = 1024;  // max |A| = |B| (chunk <= 2048); chunks up to 1024 tokens take half the LDS

__device__ inline int block_exclusive_scan(int v, int* s_wave_tot, int* total) {
  // 256 threads = 4 waves
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  if (lane == 63) s_wave_tot[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int t = s_wave_tot[w];
    if (w < wave) base += t;
    tot += t;
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

template <typename T>
struct Row;  // per-lane 16-byte piece arithmetic

template <>
struct Row<__bf16> {
  static constexpr int E = 8;
  typedef float Acc;
  typedef uint4 Raw;
  __device__ static Raw load_raw(const __bf16* p) { return ldg16_stream(p); }
  __device__ static void store_raw(__bf16* p, const Raw& r) { stg16_stream(p, r); }
  template <bool WIDE>
  __device__ static void fma_into(Acc* acc, const Raw& u, int w) { fma_bf16x8_t<WIDE>(acc, u, w); }
  __device__ static Raw div_raw(const Acc* acc, int n) { return round_div_pack_bf16(acc, n); }
  __device__ static void store_div(__bf16* p, const Acc* acc, int n) { stg16_stream(p, div_raw(acc, n)); }
};

template <>
struct Row<float> {
  static constexpr int E = 4;
  typedef double Acc;
  typedef float4 Raw;
  __device__ static Raw load_raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static void store_raw(float* p, const Raw& r) { *reinterpret_cast<float4*>(p) = r; }
  template <bool WIDE>
  __device__ static void fma_into(Acc* acc, const Raw& u, int wi) {
    const double w = (double)wi;
    acc[0] += w * (double)u.x; acc[1] += w * (double)u.y; acc[2] += w * (double)u.z; acc[3] += w * (double)u.w;
  }
  __device__ static Raw div_raw(const Acc* acc, int n) {
    const double dn = (double)n;
    return make_float4((float)(acc[0] / dn), (float)(acc[1] / dn), (float)(acc[2] / dn), (float)(acc[3] / dn));
  }
  __device__ static void store_div(float* p, const Acc* acc, int n) { *reinterpret_cast<float4*>(p) = div_raw(acc, n); }
};

constexpr int kRowsInFlight = 1;   // output rows of a row group per batch (two batches are in flight)
constexpr int kRowsInFlightOrigin = 2;   // ... when every value row is itself rebuilt from several rows

// MODE (two consecutive rounds whose first merges every edge, r = 1, can skip the intermediate
// VALUE cache: a round-0 chunk then keeps exactly its B tokens, so a round-1 chunk is fed by two
// round-0 chunks):
//   kMergeFull    keys and values of this round's input -> this round's output;
//   kMergeKeys    first round of such a pair: keys and degrees only, and the member lists of
//                 every chunk are exported (lists_out: per chunk cnt | start | members, int16);
//   kMergeOrigin  second round of the pair: keys as usual, while every value row of the input
//                 (a round-0 centroid that was never written) is rebuilt from the ORIGINAL values
//                 through the exported lists, in the same fp32 order and with the same single
//                 rounding the first round would have used, so the results are bit-identical.
enum { kMergeFull = 0, kMergeKeys = 1, kMergeOrigin = 2 };

// PAGED: some side of the launch lives in a block pool (PagedSide): the input rows (K, V, deg_in),
// the original values of kMergeOrigin (org.paged), the output keys (out_k_paged) or the output values
// and degrees (out_v_paged), each decided by its table pointer / flag at run time; the pool rows of the
// blocks a workgroup touches are staged in LDS (blocks of 8 tokens or more).
template <typename T, int D, int MODE, int MH, bool PAGED>   // MH: capacity of the per-chunk LDS arrays (|A| = |B| <= MH)
__global__ __launch_bounds__(kThreads) void merge_kernel(
    const T* __restrict__ K, const T* __restrict__ V, const int32_t* __restrict__ deg_in, TensorView in,
    int seq, int chunk, int n_chunks, float r, const int32_t* __restrict__ dst_local,
    const float* __restrict__ score, T* __restrict__ K_out, T* __restrict__ V_out,
    int32_t* __restrict__ deg_out, TensorView out, int64_t deg_out_stride, int32_t* __restrict__ map_out,
    int64_t deg_in_stride, int64_t map_stride, int map_offset, const int2* __restrict__ sel_table,
    int16_t* __restrict__ lists_out, ValueOrigin org, int parts, PagedSide pin, PagedSide pout, int out_k_paged,
    int out_v_paged) {
  constexpr int E = Row<T>::E;
  constexpr int LPR = D / E;                 // lanes per row
  constexpr int NRG = kThreads / LPR;        // row groups per workgroup
  constexpr int U = (MODE == kMergeOrigin) ? kRowsInFlightOrigin : kRowsInFlight;
  typedef typename Row<T>::Acc Acc;
  typedef typename Row<T>::Raw Raw;

  // s_dstk[i]: destination (B index) of source i if its edge is kept, -1 otherwise
  __shared__ __attribute__((aligned(16))) int16_t s_dstk[MH];
  __shared__ __attribute__((aligned(16))) float s_score[MH];
  __shared__ int32_t s_cnt[MH];
  __shared__ int32_t s_fill[MH];
  __shared__ int16_t s_start[MH];
  __shared__ int16_t s_members[MH];
  __shared__ int16_t s_local_out[2 * MH];
  __shared__ int16_t s_src_of_out[2 * MH];
  __shared__ int s_wave_tot[4];
  // kMergeOrigin, chunks up to 1024 tokens: per output row, everything the emit loop would look up
  // through the lists, resolved once (three 8-byte words: the row's own sources, then where the
  // value rows of its own token and of its first merged source come from)
  constexpr bool DESC = (MODE == kMergeOrigin) && (MH <= 512);
  __shared__ uint2 s_desc[DESC ? 3 * 2 * MH : 1];
  __shared__ int32_t s_rb_in[PAGED ? 2 * MH / 8 + 2 : 1];
  __shared__ int32_t s_rb_org[(PAGED && MODE == kMergeOrigin) ? 4 * MH / 8 + 2 : 1];
  __shared__ int32_t s_rb_out[PAGED ? 2 * MH / 8 + 2 : 1];

  // `parts` workgroups share a chunk when the launch would otherwise leave most of the chip idle:
  // each repeats the (cheap) bookkeeping and emits every parts-th group of output rows.
  const int part = blockIdx.x % parts, wg = blockIdx.x / parts;
  const int g = wg % n_chunks, bh = wg / n_chunks;
  const int tid = threadIdx.x;
  const int g0 = g * chunk, L = min(chunk, seq - g0);
  const int half = chunk >> 1;
  const int nA = (L + 1) >> 1, nB = L >> 1;
  // edges merged in this chunk and its first output row: fixed by r alone for per-chunk selection,
  // read from the table of the sequence-wide selection otherwise
  int m, out_base;
  if (sel_table) {
    const int2 e = sel_table[(int64_t)bh * n_chunks + g];
    m = e.x;
    out_base = e.y;
  } else {
    m = (nB > 0) ? merge_count(r, nA) : 0;
    out_base = g * chunk_out(chunk, r);
  }
  const int n_out = L - m;
  RowBases rb_in{}, rb_org{}, rb_out{};
  const bool in_paged = PAGED && pin.table != nullptr;
  const bool org_paged = PAGED && MODE == kMergeOrigin && org.paged.table != nullptr;
  const bool ok_paged = PAGED && out_k_paged, ov_paged = PAGED && out_v_paged;
  if (PAGED) {   // (the barriers of the bookkeeping below come before the first use)
    const int b = bh / in.heads, h = bh % in.heads;
    if (in_paged && L > 0) rb_in = stage_row_bases(s_rb_in, pin, b, h, in.heads, pin.tok0 + g0, pin.tok0 + g0 + L - 1, tid, kThreads);
    if (org_paged) {
      const int t_lo = 2 * g * chunk, t_hi = min(org.seq0, t_lo + 2 * chunk);
      if (t_hi > t_lo)
        rb_org = stage_row_bases(s_rb_org, org.paged, b, h, in.heads, org.paged.tok0 + t_lo, org.paged.tok0 + t_hi - 1, tid, kThreads);
    }
    if ((ok_paged || ov_paged) && n_out > 0)
      rb_out = stage_row_bases(s_rb_out, pout, b, h, in.heads, pout.tok0 + out_base, pout.tok0 + out_base + n_out - 1, tid, kThreads);
  }
  const int n_src = n_sources(seq, chunk);
  const int64_t src_base = (int64_t)bh * n_src + (int64_t)g * (chunk >> 1);
  const int nA_pad = (nA + 7) & ~7;

  for (int i = tid; i < nA_pad; i += kThreads) {
    s_dstk[i] = (i < nA && m > 0) ? (int16_t)dst_local[src_base + i] : (int16_t)-1;
    if (m > 0 && m < nA) s_score[i] = (i < nA) ? score[src_base + i] : -INFINITY;
  }
  for (int j = tid; j < nB; j += kThreads) s_cnt[j] = 0;
  __syncthreads();

  // ---- top-r: rank by counting (score descending, index ascending) ----------------------------
  if (m > 0 && m < nA) {
    bool drop[MH / kThreads];
#pragma unroll
    for (int it = 0; it < MH / kThreads; ++it) {
      const int i = tid + it * kThreads;
      drop[it] = false;
      if (i < nA) {
        const float si = s_score[i];
        int rank = 0;
        for (int o4 = 0; o4 < nA_pad; o4 += 4) {
          const float4 so = *reinterpret_cast<const float4*>(&s_score[o4]);
          rank += (so.x > si) || (so.x == si && o4 < i);
          rank += (so.y > si) || (so.y == si && o4 + 1 < i);
          rank += (so.z > si) || (so.z == si && o4 + 2 < i);
          rank += (so.w > si) || (so.w == si && o4 + 3 < i);
        }
        drop[it] = rank >= m;
      }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < MH / kThreads; ++it)
      if (drop[it]) s_dstk[tid + it * kThreads] = -1;
    __syncthreads();
  }

  // ---- kept sources grouped by destination, ascending within a group --------------------------
  // counts by integer atomics (order-free), then slots handed out by atomics in arbitrary order
  // and every destination's short list sorted: the final order is unique, so results stay
  // run-to-run identical.  Lists longer than kSortMax (degenerate inputs: many identical keys)
  // are placed by rank counting instead.
  constexpr int kSortMax = 8;
#pragma unroll
  for (int it = 0; it < MH / kThreads; ++it) {
    const int i = tid + it * kThreads;
    const int d = (i < nA) ? (int)s_dstk[i] : -1;
    if (d >= 0) atomicAdd(&s_cnt[d], 1);
  }
  __syncthreads();
  int longest = 0;
  {
    int c[4], sum = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = tid * 4 + e;
      c[e] = (j < nB) ? s_cnt[j] : 0;
      sum += c[e];
      longest = max(longest, c[e]);
    }
    int tot;
    int base = block_exclusive_scan(sum, s_wave_tot, &tot);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = tid * 4 + e;
      if (j < nB) { s_start[j] = (int16_t)base; s_fill[j] = 0; }
      base += c[e];
    }
  }
  const bool any_long = __syncthreads_or(longest > kSortMax);
#pragma unroll
  for (int it = 0; it < MH / kThreads; ++it) {
    const int i = tid + it * kThreads;
    const int d = (i < nA) ? (int)s_dstk[i] : -1;
    if (d >= 0) {
      int pos;
      if (any_long && s_cnt[d] > kSortMax) {        // rank among earlier sources of the same list
        pos = 0;
        for (int o = 0; o < i; ++o) pos += ((int)s_dstk[o] == d);
      } else {
        pos = atomicAdd(&s_fill[d], 1);
      }
      s_members[s_start[d] + pos] = (int16_t)i;
    }
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 4; ++e) {                     // insertion sort of the short lists
    const int j = tid * 4 + e;
    const int n = (j < nB) ? s_cnt[j] : 0;
    if (n > 1 && n <= kSortMax) {
      int16_t* lst = &s_members[s_start[j]];
      for (int a = 1; a < n; ++a) {
        const int16_t v = lst[a];
        int b2 = a - 1;
        while (b2 >= 0 && lst[b2] > v) { lst[b2 + 1] = lst[b2]; --b2; }
        lst[b2 + 1] = v;
      }
    }
  }

  // ---- retained tokens: prefix sum over the chunk --------------------------------------------
  {
    int flags = 0, cnt = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int u = tid * 8 + e;
      const bool ret = (u < L) && ((u & 1) || s_dstk[u >> 1] < 0);
      flags |= (int)ret << e;
      cnt += ret;
    }
    int tot;
    int base = block_exclusive_scan(cnt, s_wave_tot, &tot);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int u = tid * 8 + e;
      if ((flags >> e) & 1) {
        s_local_out[u] = (int16_t)base;
        s_src_of_out[base] = (int16_t)u;
        ++base;
      }
    }
  }
  __syncthreads();

  if (MODE == kMergeKeys && part == 0) {   // member lists of this chunk for the next round's value rebuild
    int16_t* lst = lists_out + ((int64_t)bh * n_chunks + g) * 3 * half;
    for (int i = tid; i < half; i += kThreads) {
      lst[i] = (i < nB) ? (int16_t)s_cnt[i] : (int16_t)0;
      lst[half + i] = (i < nB) ? s_start[i] : (int16_t)0;
      lst[2 * half + i] = (i < m) ? s_members[i] : (int16_t)0;
    }
  }

  // ---- assignment map of this round ----------------------------------------------------------
  if (map_out != nullptr && part == 0) {
    int32_t* mp = map_out + (int64_t)bh * map_stride + g0;
    for (int u = tid; u < L; u += kThreads) {
      const int d = (u & 1) ? -1 : (int)s_dstk[u >> 1];
      const int slot = (d < 0) ? s_local_out[u] : s_local_out[2 * d + 1];
      mp[u] = map_offset + out_base + slot;
    }
  }

  // kMergeOrigin: the member lists of the two previous-round chunks that feed this chunk, staged in
  // LDS arrays the bookkeeping above no longer needs (scores, fill counters, local output slots)
  int16_t (*s0_cnt)[MH] = reinterpret_cast<int16_t (*)[MH]>(s_score);
  int16_t (*s0_start)[MH] = reinterpret_cast<int16_t (*)[MH]>(s_fill);
  int16_t (*s0_mem)[MH] = reinterpret_cast<int16_t (*)[MH]>(s_local_out);
  if (MODE == kMergeOrigin) {
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c0 = 2 * g + h;
      if (c0 < org.n_chunks0) {
        const int16_t* lst = org.lists + ((int64_t)bh * org.n_chunks0 + c0) * 3 * half;
        for (int i = tid; i < half; i += kThreads) {
          s0_cnt[h][i] = lst[i];
          s0_start[h][i] = lst[half + i];
          s0_mem[h][i] = lst[2 * half + i];
        }
      }
    }
    __syncthreads();
    if constexpr (DESC) {
      // token indices are kept relative to the first token of previous-round chunk 2g
      auto value_words = [&](int p) -> uint2 {
        const int h = (p >= half) ? 1 : 0, jj = p - h * half;
        const bool single = (org.seq0 - (2 * g + h) * chunk) == 1;
        const int tb = h * chunk + (single ? 0 : 2 * jj + 1);
        const int n = single ? 0 : (int)s0_cnt[h][jj];
        const int off = h * MH + (int)s0_start[h][jj];
        const int ta = (n > 0) ? h * chunk + 2 * (int)(&s0_mem[0][0])[off] : tb;
        return make_uint2((uint32_t)tb | ((uint32_t)ta << 16), (uint32_t)n | ((uint32_t)off << 16));
      };
      for (int o = tid; o < n_out; o += kThreads) {
        const int tok = s_src_of_out[o];
        const bool isB = tok & 1;
        const int nmem = isB ? s_cnt[tok >> 1] : 0;
        const int first = isB ? (int)s_start[tok >> 1] : 0;
        const int mem0 = (nmem > 0) ? 2 * (int)s_members[first] : tok;
        s_desc[3 * o] = make_uint2((uint32_t)tok | ((uint32_t)mem0 << 16), (uint32_t)nmem | ((uint32_t)first << 16));
        s_desc[3 * o + 1] = value_words(tok);
        s_desc[3 * o + 2] = value_words(mem0);
      }
      __syncthreads();
    }
  }

  // ---- emit rows: every row group works on U output rows at once; the loads of their own rows
  // and of their first merged source are all in flight before anything is consumed ---------------
  const int rg = tid / LPR, piece = tid % LPR;
  const T* Kin = in_paged ? K + piece * E : K + in.seq_base(bh) + (int64_t)g0 * in.stride_s + piece * E;
  const T* Vin = (MODE != kMergeFull) ? nullptr
                 : in_paged ? V + piece * E : V + in.seq_base(bh) + (int64_t)g0 * in.stride_s + piece * E;
  T* Ko = ok_paged ? K_out + piece * E : K_out + out.seq_base(bh) + (int64_t)out_base * out.stride_s + piece * E;
  T* Vo = (MODE == kMergeKeys) ? nullptr
          : ov_paged ? V_out + piece * E : V_out + out.seq_base(bh) + (int64_t)out_base * out.stride_s + piece * E;
  const int32_t* dseq = !deg_in ? nullptr : in_paged ? deg_in : deg_in + (int64_t)bh * deg_in_stride + g0;
  int32_t* dout = ov_paged ? deg_out : deg_out + (int64_t)bh * deg_out_stride + out_base;
  // element offset of input row u / output row o of this chunk from Kin, Vin / Ko, Vo, and the index
  // of their degrees in dseq / dout.  An output row whose block lies outside the pool is not written.
  const int u_in0 = pin.tok0 + g0, u_out0 = pout.tok0 + out_base;
  auto in_off = [&](int u) -> int64_t { return in_paged ? (int64_t)rb_in.row(u_in0 + u) * D : (int64_t)u * in.stride_s; };
  auto in_deg = [&](int u) -> int { return in_paged ? dseq[rb_in.row(u_in0 + u)] : dseq[u]; };
  auto ok_off = [&](int o) -> int64_t { return ok_paged ? (int64_t)rb_out.row(u_out0 + o) * D : (int64_t)o * out.stride_s; };
  auto ov_off = [&](int o) -> int64_t { return ov_paged ? (int64_t)rb_out.row(u_out0 + o) * D : (int64_t)o * out.stride_s; };
  auto out_ok = [&](int o) -> bool { return !(ok_paged || ov_paged) || rb_out.base_of(u_out0 + o) >= 0; };
  auto put_deg = [&](int o, int d) {
    if (ov_paged) dout[rb_out.row(u_out0 + o)] = d;
    else dout[o] = d;
  };

  // The value row of input row p of this chunk.  kMergeFull: a load.  kMergeOrigin: the previous
  // round's centroid p, rebuilt: p is B token j of previous-round chunk 2g+h (a one-token tail chunk
  // kept its only token); its own row and its first member are loaded at once, the rest on demand.
  const T* V0p = (MODE != kMergeOrigin) ? nullptr
                 : org_paged ? static_cast<const T*>(org.V0) + piece * E
                             : static_cast<const T*>(org.V0) + org.view0.seq_base(bh) + piece * E;
  const int32_t* d0p = (MODE == kMergeOrigin && org.deg0)
                           ? (org_paged ? org.deg0 : org.deg0 + (int64_t)bh * org.view0.deg_stride) : nullptr;
  // original value row / degree of token t of the first round's clustered range
  auto v0_off = [&](int t) -> int64_t {
    return org_paged ? (int64_t)rb_org.row(org.paged.tok0 + t) * D : (int64_t)t * org.view0.stride_s;
  };
  auto d0_at = [&](int t) -> int { return org_paged ? d0p[rb_org.row(org.paged.tok0 + t)] : d0p[t]; };
  constexpr int kEager = 1;   // members of a previous-round cluster loaded together with its own row
  struct VLoad {
    Raw b, m[kEager];
    int db, dm[kEager], n, base;
    const int16_t* mem;
  };
  struct NoVLoad {};   // keys-only mode carries no value rows
  auto v_issue = [&](int p) -> VLoad {
    VLoad x;
    if (MODE == kMergeFull) {
      x.b = Row<T>::load_raw(Vin + in_off(p));
      x.n = 0;
    } else if (MODE == kMergeOrigin) {
      const int h = (p >= half) ? 1 : 0, jj = p - h * half;
      x.base = (2 * g + h) * chunk;
      const bool single = (org.seq0 - x.base) == 1;
      const int tb = x.base + (single ? 0 : 2 * jj + 1);
      x.n = single ? 0 : (int)s0_cnt[h][jj];
      x.mem = &s0_mem[h][s0_start[h][jj]];
      x.b = Row<T>::load_raw(V0p + v0_off(tb));
      x.db = d0p ? d0_at(tb) : 1;
#pragma unroll
      for (int q = 0; q < kEager; ++q) {
        if (q < x.n) {
          const int ta = x.base + 2 * (int)x.mem[q];
          x.m[q] = Row<T>::load_raw(V0p + v0_off(ta));
          x.dm[q] = d0p ? d0_at(ta) : 1;
        }
      }
    }
    return x;
  };
  auto v_issue_resolved = [&](uint2 w) -> VLoad {
    VLoad x;
    if constexpr (MODE == kMergeOrigin) {
      const int t0 = 2 * g * chunk;
      const int tb_rel = (int)(w.x & 0xffffu);
      const int tb = t0 + tb_rel, ta = t0 + (int)(w.x >> 16);
      x.base = t0 + ((tb_rel >= chunk) ? chunk : 0);
      x.n = (int)(w.y & 0xffffu);
      x.mem = &s0_mem[0][0] + (w.y >> 16);
      x.b = Row<T>::load_raw(V0p + v0_off(tb));
      x.db = d0p ? d0_at(tb) : 1;
      static_assert(kEager == 1, "one resolved member per cluster");
      if (x.n > 0) {
        x.m[0] = Row<T>::load_raw(V0p + v0_off(ta));
        x.dm[0] = d0p ? d0_at(ta) : 1;
      }
    }
    return x;
  };
  auto v_finish = [&](auto wide_c, const VLoad& x) -> Raw {
    constexpr bool WIDE = decltype(wide_c)::value;
    if (MODE != kMergeOrigin || x.n == 0) return x.b;
    Acc a[E];
#pragma unroll
    for (int e = 0; e < E; ++e) a[e] = 0;
    Row<T>::template fma_into<WIDE>(a, x.b, x.db);
    int nd = x.db;
#pragma unroll
    for (int q = 0; q < kEager; ++q)
      if (q < x.n) {
        Row<T>::template fma_into<WIDE>(a, x.m[q], x.dm[q]);
        nd += x.dm[q];
      }
    for (int q = kEager; q < x.n; ++q) {
      const int ta = x.base + 2 * (int)x.mem[q];
      const int da = d0p ? d0_at(ta) : 1;
      Row<T>::template fma_into<WIDE>(a, Row<T>::load_raw(V0p + v0_off(ta)), da);
      nd += da;
    }
    return Row<T>::div_raw(a, nd);
  };

  // One batch = U output rows per row group: where they come from (LDS lookups) and the loads of
  // their own rows and first merged sources, all issued before anything is consumed.
  struct Batch {
    int ob;
    int tok[U], nmem[U], first[U], du[U], dm[U];
    bool valid[U];
    Raw kb[U], km[U];
    typename std::conditional<MODE == kMergeKeys, NoVLoad, VLoad>::type vb[U], vm[U];
  };
  struct Where {
    int ob;
    int tok[U], mem0[U], nmem[U], first[U];
    bool valid[U];
    uint2 wb[U], wm[U];
  };
  auto lookup = [&](int ob) -> Where {
    Where w;
    w.ob = ob;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int o = ob + u * NRG + rg;
      w.valid[u] = o < n_out;
      const int oo = w.valid[u] ? o : n_out - 1;
      if constexpr (DESC) {
        const uint2 k = s_desc[3 * oo];
        w.wb[u] = s_desc[3 * oo + 1];
        w.wm[u] = s_desc[3 * oo + 2];
        w.tok[u] = (int)(k.x & 0xffffu);
        w.mem0[u] = (int)(k.x >> 16);
        w.nmem[u] = (int)(k.y & 0xffffu);
        w.first[u] = (int)(k.y >> 16);
      } else {
        w.tok[u] = s_src_of_out[oo];
        const bool isB = w.tok[u] & 1;
        w.nmem[u] = isB ? s_cnt[w.tok[u] >> 1] : 0;
        w.first[u] = isB ? (int)s_start[w.tok[u] >> 1] : 0;
        w.mem0[u] = (w.nmem[u] > 0) ? 2 * (int)s_members[w.first[u]] : w.tok[u];   // no source: re-read own row
      }
    }
    return w;
  };
  auto issue = [&](const Where& w) -> Batch {
    Batch x;
    x.ob = w.ob;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      x.valid[u] = w.valid[u];
      x.tok[u] = w.tok[u];
      x.nmem[u] = w.nmem[u];
      x.first[u] = w.first[u];
      x.kb[u] = Row<T>::load_raw(Kin + in_off(w.tok[u]));
      x.km[u] = Row<T>::load_raw(Kin + in_off(w.mem0[u]));
      if constexpr (DESC) {
        x.vb[u] = v_issue_resolved(w.wb[u]);
        x.vm[u] = v_issue_resolved(w.wm[u]);
      } else if constexpr (MODE != kMergeKeys) {
        x.vb[u] = v_issue(w.tok[u]);
        x.vm[u] = v_issue(w.mem0[u]);
      }
      x.du[u] = dseq ? in_deg(w.tok[u]) : 1;
      x.dm[u] = dseq ? in_deg(w.mem0[u]) : 1;
    }
    return x;
  };
  auto fetch = [&](int ob) -> Batch { return issue(lookup(ob)); };
  auto finish = [&](auto wide_c, const Batch& x) {
    constexpr bool WIDE = decltype(wide_c)::value;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!x.valid[u]) continue;
      const int o = x.ob + u * NRG + rg;
      if (PAGED && !out_ok(o)) continue;
      if (x.nmem[u] == 0) {  // untouched token: bit copy
        Row<T>::store_raw(Ko + ok_off(o), x.kb[u]);
        if constexpr (MODE != kMergeKeys) Row<T>::store_raw(Vo + ov_off(o), v_finish(wide_c, x.vb[u]));
        if (piece == 0) put_deg(o, x.du[u]);
        continue;
      }
      Acc ak[E], av[E];
#pragma unroll
      for (int e = 0; e < E; ++e) { ak[e] = 0; av[e] = 0; }
      Row<T>::template fma_into<WIDE>(ak, x.kb[u], x.du[u]);
      Row<T>::template fma_into<WIDE>(ak, x.km[u], x.dm[u]);
      if constexpr (MODE != kMergeKeys) {
        Row<T>::template fma_into<WIDE>(av, v_finish(wide_c, x.vb[u]), x.du[u]);
        Row<T>::template fma_into<WIDE>(av, v_finish(wide_c, x.vm[u]), x.dm[u]);
      }
      int ndeg = x.du[u] + x.dm[u];
      for (int q = 1; q < x.nmem[u]; ++q) {
        const int ua = 2 * (int)s_members[x.first[u] + q];
        const int da = dseq ? in_deg(ua) : 1;
        const Raw kx = Row<T>::load_raw(Kin + in_off(ua));
        Row<T>::template fma_into<WIDE>(ak, kx, da);
        if constexpr (MODE != kMergeKeys) Row<T>::template fma_into<WIDE>(av, v_finish(wide_c, v_issue(ua)), da);
        ndeg += da;
      }
      Row<T>::store_div(Ko + ok_off(o), ak, ndeg);
      if constexpr (MODE != kMergeKeys) Row<T>::store_div(Vo + ov_off(o), av, ndeg);
      if (piece == 0) put_deg(o, ndeg);
    }
  };
  // kMergeOrigin: the same sums in the same order as v_finish, for several clusters in lock step.
  // A row group that walks one cluster after the other waits a full memory latency per extra member
  // while the rest of its wave idles; here the q-th extra member of every cluster handed in is
  // requested at once, so the wave waits as often as the longest of them has members, not the sum.
  // Called per output row with its two clusters (own token, first merged source): handing in all
  // four of a batch measured the same and needs 15 more registers.
  auto v_finish_all = [&](auto wide_c, auto count_c, const VLoad* cl, const bool* on, Raw* res) {
    constexpr bool WIDE = decltype(wide_c)::value;
    constexpr int C = decltype(count_c)::value;
    Acc a[C][E];
    int nd[C], n[C], longest = 0;
#pragma unroll
    for (int c = 0; c < C; ++c) {
      n[c] = on[c] ? cl[c].n : 0;
      nd[c] = 0;
#pragma unroll
      for (int e = 0; e < E; ++e) a[c][e] = 0;
      if (n[c] > 0) {
        Row<T>::template fma_into<WIDE>(a[c], cl[c].b, cl[c].db);
        Row<T>::template fma_into<WIDE>(a[c], cl[c].m[0], cl[c].dm[0]);
        nd[c] = cl[c].db + cl[c].dm[0];
      }
      longest = max(longest, n[c]);
    }
    for (int q = kEager; q < longest; ++q) {
      Raw r[C];
      int d[C];
#pragma unroll
      for (int c = 0; c < C; ++c)
        if (q < n[c]) {
          const int ta = cl[c].base + 2 * (int)cl[c].mem[q];
          r[c] = Row<T>::load_raw(V0p + v0_off(ta));
          d[c] = d0p ? d0_at(ta) : 1;
        }
#pragma unroll
      for (int c = 0; c < C; ++c)
        if (q < n[c]) {
          Row<T>::template fma_into<WIDE>(a[c], r[c], d[c]);
          nd[c] += d[c];
        }
    }
#pragma unroll
    for (int c = 0; c < C; ++c)
      if (on[c]) res[c] = (n[c] == 0) ? cl[c].b : Row<T>::div_raw(a[c], nd[c]);
  };
  auto finish_origin = [&](auto wide_c, const Batch& x) {
    constexpr bool WIDE = decltype(wide_c)::value;
    if constexpr (MODE == kMergeOrigin) {
      bool on[2 * U];
      Raw vr[2 * U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const VLoad cl[2] = {x.vb[u], x.vm[u]};
        on[2 * u] = x.valid[u];
        on[2 * u + 1] = x.valid[u] && x.nmem[u] > 0;
        v_finish_all(wide_c, std::integral_constant<int, 2>{}, cl, on + 2 * u, vr + 2 * u);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (!x.valid[u]) continue;
        const int o = x.ob + u * NRG + rg;
        if (PAGED && !out_ok(o)) continue;
        if (x.nmem[u] == 0) {  // untouched token: bit copy of the key; its value row is one cluster
          Row<T>::store_raw(Ko + ok_off(o), x.kb[u]);
          Row<T>::store_raw(Vo + ov_off(o), vr[2 * u]);
          if (piece == 0) put_deg(o, x.du[u]);
          continue;
        }
        Acc ak[E], av[E];
#pragma unroll
        for (int e = 0; e < E; ++e) { ak[e] = 0; av[e] = 0; }
        Row<T>::template fma_into<WIDE>(ak, x.kb[u], x.du[u]);
        Row<T>::template fma_into<WIDE>(ak, x.km[u], x.dm[u]);
        Row<T>::template fma_into<WIDE>(av, vr[2 * u], x.du[u]);
        Row<T>::template fma_into<WIDE>(av, vr[2 * u + 1], x.dm[u]);
        int ndeg = x.du[u] + x.dm[u];
        for (int q = 1; q < x.nmem[u]; ++q) {
          const int ua = 2 * (int)s_members[x.first[u] + q];
          const int da = dseq ? in_deg(ua) : 1;
          const Raw kx = Row<T>::load_raw(Kin + in_off(ua));
          Row<T>::template fma_into<WIDE>(ak, kx, da);
          Row<T>::template fma_into<WIDE>(av, v_finish(wide_c, v_issue(ua)), da);
          ndeg += da;
        }
        Row<T>::store_div(Ko + ok_off(o), ak, ndeg);
        Row<T>::store_div(Vo + ov_off(o), av, ndeg);
        if (piece == 0) put_deg(o, ndeg);
      }
    }
  };
  // The loop over batches is software-pipelined (the next batch's loads are in flight while this
  // one is merged and stored) except in origin mode, whose batches are too large to hold twice.
  auto emit = [&](auto wide_c) {
    const int step = parts * NRG * U;
    int ob = part * NRG * U;
    if (ob >= n_out) return;
    if (MODE == kMergeOrigin) {
      for (; ob < n_out; ob += step) finish_origin(wide_c, fetch(ob));
      return;
    }
    Batch a = fetch(ob);
    for (;;) {
      ob += step;
      if (ob >= n_out) { finish(wide_c, a); break; }
      Batch b2 = fetch(ob);
      finish(wide_c, a);
      ob += step;
      if (ob >= n_out) { finish(wide_c, b2); break; }
      a = fetch(ob);
      finish(wide_c, b2);
    }
  };
  // Two versions of the emit loop: weights up to 256 ride in a packed bf16 operand (one v_dot2 per
  // element); a chunk that holds a larger degree takes the general route.  Same bits either way.
  bool wide;
  {
    int big = 0;
    if (deg_in) {
      for (int u = tid; u < L; u += kThreads) big |= in_deg(u) > 256;
    }
    if (MODE == kMergeOrigin && d0p) {
      const int t_lo = 2 * g * chunk, t_hi = min(org.seq0, t_lo + 2 * chunk);
      for (int t = t_lo + tid; t < t_hi; t += kThreads) big |= d0_at(t) > 256;
    }
    wide = __syncthreads_or(big) != 0;
  }
  if (wide) emit(std::true_type{});
  else emit(std::false_type{});
}

// assign[bh][t] <- map[bh][assign[bh][t]]: four consecutive tokens per thread (one 16-byte access when
// the rows allow it), one workgroup per piece of 1024 tokens of one sequence
__global__ void compose_kernel(int32_t* __restrict__ assign, const int32_t* __restrict__ map, int seq0,
                               int map_len, int pieces, int vec) {
  const int bh = blockIdx.x / pieces, pc = blockIdx.x % pieces;
  int32_t* a = assign + (int64_t)bh * seq0;
  const int32_t* m = map + (int64_t)bh * map_len;
  const int t = (pc * (int)blockDim.x + (int)threadIdx.x) * 4;
  if (t >= seq0) return;
  if (vec && t + 4 <= seq0) {
    int4 v = *reinterpret_cast<const int4*>(a + t);
    v.x = m[v.x];
    v.y = m[v.y];
    v.z = m[v.z];
    v.w = m[v.w];
    *reinterpret_cast<int4*>(a + t) = v;
  } else {
    for (int i = t; i < min(t + 4, seq0); ++i) a[i] = m[a[i]];
  }
}

__global__ void copy_rows_kernel(const unsigned char* __restrict__ src, TensorView in,
                                 unsigned char* __restrict__ dst, TensorView out, int seq, int pieces_per_row,
                                 int elem_bytes, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int piece = (int)(e % pieces_per_row);
  const int64_t row = e / pieces_per_row;
  const int t = (int)(row % seq), bh = (int)(row / seq);
  const int64_t so = (in.seq_base(bh) + (int64_t)t * in.stride_s) * elem_bytes + piece * 16;
  const int64_t dof = (out.seq_base(bh) + (int64_t)t * out.stride_s) * elem_bytes + piece * 16;
  *reinterpret_cast<uint4*>(dst + dof) = *reinterpret_cast<const uint4*>(src + so);
}

// Tokens that bypass the clustering (Sec. 5.2: attention sinks and recent tokens are set aside
// before partitioning; Sec. 5.3: they are concatenated back): the first n_head and the last n_tail
// tokens of every sequence are copied to the head / tail of the output (keys, values, degree), and
// their entries of the round's assignment map are written.
__global__ void edges_kernel(const unsigned char* __restrict__ K, const unsigned char* __restrict__ V,
                             const int32_t* __restrict__ deg_in, TensorView in, int in_len,
                             unsigned char* __restrict__ K_out, unsigned char* __restrict__ V_out,
                             int32_t* __restrict__ deg_out, TensorView out, int64_t deg_out_stride, int out_len,
                             int32_t* __restrict__ map_out, int n_head, int n_tail, int pieces_per_row,
                             int elem_bytes, int64_t total, PagedSide pin, PagedSide pok, PagedSide pov) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int piece = (int)(e % pieces_per_row);
  const int64_t row = e / pieces_per_row;
  const int n_edge = n_head + n_tail;
  const int k = (int)(row % n_edge), bh = (int)(row / n_edge);
  const int t_in = k < n_head ? k : in_len - n_tail + (k - n_head);
  const int t_out = k < n_head ? k : out_len - n_tail + (k - n_head);
  const int b = bh / in.heads, h = bh % in.heads;
  // pool row of token u of this (batch, head) through a side's block table; -1 outside the pool
  auto pool_row = [&](const PagedSide& pg, int u) -> int64_t {
    const int blk = ((u >> pg.shift) < pg.max_blocks) ? pg.table[(int64_t)b * pg.max_blocks + (u >> pg.shift)] : -1;
    if ((unsigned)blk >= (unsigned)pg.n_blocks) return -1;
    return (((int64_t)blk * in.heads + h) << pg.shift) + (u & ((1 << pg.shift) - 1));
  };
  const int64_t row_bytes = (int64_t)pieces_per_row * 16;
  int64_t ri = 0, rk = 0, rv = 0;
  if (pin.table) ri = pool_row(pin, pin.tok0 + t_in);
  if (pok.table) rk = pool_row(pok, pok.tok0 + t_out);
  if (pov.table) rv = pool_row(pov, pov.tok0 + t_out);
  if (ri < 0) ri = 0;                      // a block outside the pool reads as row 0 and is not written
  const int64_t so = pin.table ? ri * row_bytes + piece * 16
                               : (in.seq_base(bh) + (int64_t)t_in * in.stride_s) * elem_bytes + piece * 16;
  const int64_t dof = (out.seq_base(bh) + (int64_t)t_out * out.stride_s) * elem_bytes + piece * 16;
  const int64_t dk = pok.table ? rk * row_bytes + piece * 16 : dof;
  const int64_t dv = pov.table ? rv * row_bytes + piece * 16 : dof;
  if (rk >= 0) *reinterpret_cast<uint4*>(K_out + dk) = *reinterpret_cast<const uint4*>(K + so);
  if (rv >= 0) *reinterpret_cast<uint4*>(V_out + dv) = *reinterpret_cast<const uint4*>(V + so);
  if (piece == 0) {
    const int d = !deg_in ? 1 : pin.table ? deg_in[ri] : deg_in[(int64_t)bh * in.deg_stride + t_in];
    if (pov.table) { if (rv >= 0) deg_out[rv] = d; }
    else deg_out[(int64_t)bh * deg_out_stride + t_out] = d;
    if (map_out) map_out[(int64_t)bh * in_len + t_in] = t_out;
  }
}

// Cache update of a decode step (Algorithm 1, decoding part): the new token of every (batch, head)
// goes to row lens[b] (or `pos`) with degree 1.  A sequence already at capacity is left alone.
// One workgroup per sequence: all of its threads read lens[b], meet, write the rows of all heads, and
// one of them then advances lens[b] - no other workgroup reads or writes that entry, so the update
// needs no launch of its own.
__global__ void append_kernel(const unsigned char* __restrict__ k_new, const unsigned char* __restrict__ v_new,
                              unsigned char* __restrict__ K, unsigned char* __restrict__ V,
                              int32_t* __restrict__ deg, TensorView cache, int capacity,
                              int32_t* __restrict__ lens, int pos, int pieces_per_row, int elem_bytes) {
  const int b = blockIdx.x;
  const int t = lens ? lens[b] : pos;
  __syncthreads();
  if (t < 0 || t >= capacity) return;      // the same for every thread of the workgroup
  const int per_seq = cache.heads * pieces_per_row;
  for (int e = threadIdx.x; e < per_seq; e += blockDim.x) {
    const int piece = e % pieces_per_row, bh = b * cache.heads + e / pieces_per_row;
    const int64_t so = ((int64_t)bh * pieces_per_row + piece) * 16;
    const int64_t dof = (cache.seq_base(bh) + (int64_t)t * cache.stride_s) * elem_bytes + piece * 16;
    *reinterpret_cast<uint4*>(K + dof) = *reinterpret_cast<const uint4*>(k_new + so);
    *reinterpret_cast<uint4*>(V + dof) = *reinterpret_cast<const uint4*>(v_new + so);
    if (piece == 0 && deg) deg[(int64_t)bh * cache.deg_stride + t] = 1;
  }
  if (lens && threadIdx.x == 0) lens[b] = t + 1;
}

__global__ void fill_deg_kernel(const int32_t* __restrict__ deg_in, int64_t in_stride, int32_t* __restrict__ deg_out,
                                int64_t out_stride, int32_t* __restrict__ assign, int seq, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int t = (int)(e % seq);
  const int64_t bh = e / seq;
  deg_out[bh * out_stride + t] = deg_in ? deg_in[bh * in_stride + t] : 1;
  if (assign) assign[e] = t;
}

template <typename T, int D>
hipError_t launch_merge_t(const void* K, const void* V, const int32_t* deg_in, TensorView in, int n_bh,
                          int seq, int chunk, float r, const int32_t* dst_local, const float* score,
                          void* K_out, void* V_out, int32_t* deg_out, TensorView out,
                          int64_t deg_out_stride, int32_t* map_out, int64_t deg_in_stride, int64_t map_stride,
                          int map_offset, const int32_t* sel_table, int16_t* lists_out, const ValueOrigin* org,
                          hipStream_t st, PagedSide pin, PagedSide pok, PagedSide pov) {
  const int n_chunks = div_up(seq, chunk);
  const int64_t total = (int64_t)n_bh * n_chunks;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  const ValueOrigin o = org ? *org : ValueOrigin{};
  // small launches: split every chunk's rows over several workgroups, aiming at 4 workgroups per CU
  int parts = 1;
  while (parts < 8 && total * parts < 1024) parts *= 2;
  // any side in a block pool: the kernel variant that stages block tables (blocks of 8 tokens or more)
  const bool any_paged = pin.table || pok.table || pov.table || o.paged.table;
  if (any_paged && ((pin.table && pin.shift < 3) || (pok.table && pok.shift < 3) || (pov.table && pov.shift < 3) ||
                    (o.paged.table && o.paged.shift < 3)))
    return hipErrorInvalidValue;
  const PagedSide pout = pok.table ? pok : pov;
#define CKV_LAUNCH_MH(MODE, MH, PG)                                                                           \
  hipLaunchKernelGGL((merge_kernel<T, D, MODE, MH, PG>), dim3((int)(total * parts)), dim3(kThreads), 0, st,  \
                     static_cast<const T*>(K), static_cast<const T*>(V), deg_in, in, seq, chunk, n_chunks, r, \
                     dst_local, score, static_cast<T*>(K_out), static_cast<T*>(V_out), deg_out, out,          \
                     deg_out_stride, map_out, deg_in_stride, map_stride, map_offset,                          \
                     reinterpret_cast<const int2*>(sel_table), lists_out, o, parts, pin, pout,                \
                     pok.table != nullptr, pov.table != nullptr)
  // smaller LDS arrays for chunks of up to 1024 tokens: more workgroups per CU
#define CKV_LAUNCH(MODE)                                                    \
  do {                                                                      \
    if (any_paged) {                                                        \
      if (chunk <= kMaxHalf) CKV_LAUNCH_MH(MODE, kMaxHalf / 2, true);       \
      else CKV_LAUNCH_MH(MODE, kMaxHalf, true);                             \
    } else {                                                                \
      if (chunk <= kMaxHalf) CKV_LAUNCH_MH(MODE, kMaxHalf / 2, false);      \
      else CKV_LAUNCH_MH(MODE, kMaxHalf, false);                            \
    }                                                                       \
  } while (0)
  if (org) {
    ScopedTimer t(sizeof(T) == 2 ? "merge_origin_bf16" : "merge_origin_f32", st);
    CKV_LAUNCH(kMergeOrigin);
  } else if (lists_out) {
    ScopedTimer t(sizeof(T) == 2 ? "merge_keys_bf16" : "merge_keys_f32", st);
    CKV_LAUNCH(kMergeKeys);
  } else {
    ScopedTimer t(sizeof(T) == 2 ? "merge_bf16" : "merge_f32", st);
    CKV_LAUNCH(kMergeFull);
  }
#undef CKV_LAUNCH
  return hipGetLastError();
}

}  // namespace

hipError_t launch_merge(const void* K, const void* V, const int32_t* deg_in, int dtype, int dim,
                        TensorView in, int n_bh, int seq, int chunk, float r,
                        const int32_t* dst_local, const float* score, void* K_out, void* V_out,
                        int32_t* deg_out, TensorView out, int64_t deg_out_stride, int32_t* map_out,
                        int64_t deg_in_stride, int64_t map_stride, int map_offset, const int32_t* sel_table,
                        int16_t* lists_out, const ValueOrigin* org, hipStream_t st, PagedSide paged_in,
                        PagedSide paged_out_k, PagedSide paged_out_v) {
#define CKV_MERGE(T, DD)                                                                             \
  return launch_merge_t<T, DD>(K, V, deg_in, in, n_bh, seq, chunk, r, dst_local, score, K_out, V_out, \
                               deg_out, out, deg_out_stride, map_out, deg_in_stride, map_stride, map_offset, \
                               sel_table, lists_out, org, st, paged_in, paged_out_k, paged_out_v)
  if (dtype == CKV_BF16) {
    if (dim == 128) CKV_MERGE(__bf16, 128);
    if (dim == 64) CKV_MERGE(__bf16, 64);
  } else {
    if (dim == 128) CKV_MERGE(float, 128);
    if (dim == 64) CKV_MERGE(float, 64);
    if (dim == 32) CKV_MERGE(float, 32);
    if (dim == 16) CKV_MERGE(float, 16);
  }
#undef CKV_MERGE
  return hipErrorInvalidValue;
}

hipError_t launch_compose(int32_t* assign, const int32_t* map, int n_bh, int seq0, int map_len,
                          hipStream_t st) {
  if (n_bh <= 0 || seq0 <= 0) return hipSuccess;
  const int vec = (seq0 % 4 == 0) && (reinterpret_cast<uintptr_t>(assign) % 16 == 0);
  ScopedTimer t("compose_assign", st);
  const int pieces = (seq0 + 1023) / 1024;
  if ((int64_t)n_bh * pieces > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(compose_kernel, dim3((unsigned)(n_bh * pieces)), dim3(256), 0, st, assign, map, seq0,
                     map_len, pieces, vec);
  return hipGetLastError();
}

hipError_t launch_copy_rows(const void* src, TensorView in, void* dst, TensorView out, int n_bh, int seq,
                            int row_bytes, int elem_bytes, hipStream_t st) {
  const int ppr = row_bytes / 16;
  const int64_t total = (int64_t)n_bh * seq * ppr;
  ScopedTimer t("copy_rows", st);
  hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     static_cast<const unsigned char*>(src), in, static_cast<unsigned char*>(dst), out, seq,
                     ppr, elem_bytes, total);
  return hipGetLastError();
}

hipError_t launch_edges(const void* K, const void* V, const int32_t* deg_in, TensorView in, int in_len, void* K_out,
                        void* V_out, int32_t* deg_out, TensorView out, int64_t deg_out_stride, int out_len,
                        int32_t* map_out, int n_head, int n_tail, int n_bh, int row_bytes, int elem_bytes,
                        hipStream_t st, PagedSide paged_in, PagedSide paged_out_k, PagedSide paged_out_v) {
  const int ppr = row_bytes / 16;
  const int64_t total = (int64_t)n_bh * (n_head + n_tail) * ppr;
  if (total == 0) return hipSuccess;
  ScopedTimer t("edges_copy", st);
  hipLaunchKernelGGL(edges_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     static_cast<const unsigned char*>(K), static_cast<const unsigned char*>(V), deg_in, in, in_len,
                     static_cast<unsigned char*>(K_out), static_cast<unsigned char*>(V_out), deg_out, out,
                     deg_out_stride, out_len, map_out, n_head, n_tail, ppr, elem_bytes, total, paged_in, paged_out_k,
                     paged_out_v);
  return hipGetLastError();
}

hipError_t launch_append(const void* k_new, const void* v_new, void* K, void* V, int32_t* deg, TensorView cache,
                         int batch, int capacity, int32_t* lens, int pos, int row_bytes, int elem_bytes,
                         hipStream_t st) {
  const int ppr = row_bytes / 16;
  ScopedTimer t("append", st);
  hipLaunchKernelGGL(append_kernel, dim3((unsigned)batch), dim3(256), 0, st,
                     static_cast<const unsigned char*>(k_new), static_cast<const unsigned char*>(v_new),
                     static_cast<unsigned char*>(K), static_cast<unsigned char*>(V), deg, cache, capacity, lens,
                     pos, ppr, elem_bytes);
  return hipGetLastError();
}

hipError_t launch_fill_deg(const int32_t* deg_in, int64_t in_stride, int32_t* deg_out, int64_t out_stride,
                           int32_t* assign, int n_bh, int seq, hipStream_t st) {
  const int64_t total = (int64_t)n_bh * seq;
  ScopedTimer t("fill_deg", st);
  hipLaunchKernelGGL(fill_deg_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, deg_in,
                     in_stride, deg_out, out_stride, assign, seq, total);
  return hipGetLastError();
}

}  // namespace ckv
