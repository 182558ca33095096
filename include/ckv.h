/*
 * ckv.h - C ABI of libckv: CentroidKV's KV-cache compression (Chunked Soft Matching +
 * degree-weighted merge) and decode attention over the compressed cache, as hand-written
 * gfx950 (MI355X) HIP kernels.  Paper: arXiv 2506.11418.
 *
 * Conventions for every function
 *   - returns CKV_OK (0) or a negative ckv_status; never throws, aborts or prints;
 *   - pointers named K, V, q, o, deg, lens, assign, dst, score, freed, block_table, workspace
 *     and the *_pool / *_new / *_out buffers are DEVICE pointers (HIP global memory of the current
 *     device); ckv_layout / ckv_paged_layout / ckv_params / ckv_plan_t and other struct or
 *     scalar-result pointers are HOST pointers;
 *   - the caller owns every buffer; the library allocates and frees no device memory;
 *   - work is enqueued on `hip_stream` (a hipStream_t, NULL = the default stream) and the call
 *     returns without synchronising; argument errors are detected on the host before any launch;
 *   - buffers passed through const pointers are never written; outputs and workspace must not
 *     overlap inputs (CKV_EINVAL where the host can tell); ckv_append and the ckv_paged_* calls
 *     update the cache they are given in place, as stated with each of them;
 *   - base pointers and row strides (in bytes) of K/V tensors are multiples of 16 (CKV_EALIGN);
 *   - the library reads no environment variable and keeps no state between calls apart from the
 *     timing hooks at the end of this file (a single benchmarking thread) and a per-device note,
 *     taken under a lock, of which kernels have been set up: calls from several threads, each on
 *     its own stream and buffers, do not disturb one another.
 *
 * Tensor layout ("layout"): element (b, h, t, :) of a [batch, heads, seq, dim] tensor lives at
 * base + b*stride_b + h*stride_h + t*stride_s (strides in ELEMENTS); dim is contiguous.  This
 * covers [B,H,S,D] and [B,S,H,D] storage.  `heads` are KV heads; layers are folded into batch
 * or heads by the caller, every (batch, head) sequence is compressed independently (Sec. 3:
 * the method is stated per attention head).
 */
#ifndef CKV_H
#define CKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CKV_OK = 0,
  CKV_EINVAL = -1,       /* null pointer, bad enum, bad ratio, overlapping buffers            */
  CKV_ESHAPE = -2,       /* non-positive size, stride smaller than the extent it spans         */
  CKV_EALIGN = -3,       /* pointer or row stride not a multiple of 16 bytes                   */
  CKV_EWORKSPACE = -4,   /* workspace smaller than ckv_plan / ckv_decode_attn_workspace said   */
  CKV_EUNSUPPORTED = -5, /* valid request this build has no kernel for (see each function)     */
  CKV_EHIP = -6          /* a HIP call failed; the HIP error state has been cleared            */
} ckv_status;

typedef enum { CKV_F32 = 0, CKV_BF16 = 1 } ckv_dtype;

typedef struct {
  int32_t batch, heads, seq, dim;
  int64_t stride_b, stride_h, stride_s; /* in elements */
  int32_t dtype;                        /* ckv_dtype */
  int64_t deg_stride;                   /* elements between the rows of consecutive (batch, head)
                                           sequences in the int32 degree array that goes with this
                                           tensor; 0 = seq (a packed [batch, heads, seq] array).  A
                                           cache with spare capacity sets it to the capacity.      */
} ckv_layout;

#define CKV_MAX_ROUNDS 8

/* Parameters of CentroidKV(K, V, N, s, n1, n2, r, c) (Algorithm 1, Sec. 5). */
typedef struct {
  int32_t chunk;        /* c: chunk size in tokens, even, 2..2048 (Sec. 5.2)                     */
  float retain_ratio;   /* rho in (0,1]: fraction of tokens kept; used when n_rounds == 0.
                           Schedule: J = ceil(log2(1/rho)) rounds (a round removes at most half,
                           Sec. 5.1), r = 1 for the first J-1 and r = 2(1 - rho*2^(J-1)) last.  */
  int32_t n_rounds;     /* > 0: run exactly these rounds with merge fractions r[0..n_rounds)     */
  float r[CKV_MAX_ROUNDS]; /* r_j in [0,1]: fraction of a chunk's candidate edges merged (5.3)   */
  int32_t n_sink, n_recent; /* n1, n2 of Algorithm 1 (Sec. 5.2), >= 0: in every round the first n1
                               and the last n2 tokens of the current cache are set aside before
                               chunking and copied unchanged (degree kept) to the head / tail of
                               the round's output (Sec. 5.3); chunks, merge fractions and
                               retain_ratio's schedule apply to the tokens between them.  A cache
                               of at most n1+n2 tokens passes through a round unchanged.          */
  int32_t scope;        /* how the top-r edges are chosen (Sec. 5.2-5.3 leave both readings open):
                           CKV_SCOPE_CHUNK (0): the floor(r*|A|) best edges of every chunk;
                           CKV_SCOPE_HEAD  (1): the edges of all chunks of a (batch, head)
                           sequence ranked together, the floor(r*edges) best merged, ties to the
                           lower position.  Equal at r = 1.                                     */
  uint32_t flags;       /* CKV_ROUTE_* bits; 0 = let the library choose.  They pick between kernel
                           routes that give the same result bit for bit (see ckv_compress).     */
} ckv_params;

enum { CKV_SCOPE_CHUNK = 0, CKV_SCOPE_HEAD = 1 };
enum {
  CKV_ROUTE_FULL_ROUNDS = 1u,   /* every round writes its value cache                            */
  CKV_ROUTE_DEFER_ALWAYS = 2u   /* leave values to the next round wherever that is possible,
                                   whatever the size of the job                                  */
};

typedef struct {
  int32_t out_seq;                       /* tokens per (batch, head) after the last round        */
  int32_t n_rounds;
  int32_t round_len[CKV_MAX_ROUNDS + 1]; /* round_len[0] = seq, round_len[j+1] after round j     */
  float round_r[CKV_MAX_ROUNDS];         /* the merge fraction each round uses                   */
  size_t workspace_bytes;                /* device scratch ckv_compress needs                    */
} ckv_plan_t;

const char* ckv_version(void);
const char* ckv_strerror(int status);

/* Host only.  Resolves the rounds schedule and the sequence length after every round.
 * One round (Sec. 5.2-5.3): chunks of `chunk` consecutive tokens (last may be shorter); inside a
 * chunk of L tokens set A = 1st, 3rd, ... token (ceil(L/2) sources), B = 2nd, 4th, ...; the
 * m = floor(r*|A| + 1e-9) best edges are merged, so the chunk keeps L - m tokens (a chunk with
 * L < 2 keeps all).  Lengths depend only on (seq, chunk, schedule), never on data. */
int ckv_plan(const ckv_layout* in, const ckv_params* p, ckv_plan_t* plan);

/* Host only.  Number of A tokens (sources) of a sequence of `seq` tokens cut into chunks of `chunk`
 * tokens (Sec. 5.2): ceil(L/2) per chunk of L tokens.  Negative status for bad arguments. */
int32_t ckv_n_sources(int32_t seq, int32_t chunk);

/* Host only.  The cache budget B = floor(R * n) of Algorithm 1 for a prompt of n tokens and cache
 * ratio R in (0,1] (R carried as float, widened, + 1e-9 so that exact products stay exact).
 * Negative status for bad arguments. */
int32_t ckv_budget_tokens(float cache_ratio, int32_t n);

/* Similarity + matching stage alone (Sec. 5.2; Eq. 2): for every A token its most similar B
 * token of the same chunk under cosine similarity of the keys (lowest B index on ties).
 *   dst   [batch, heads, n_src] int32: position in the sequence of the matched B token (-1 when the
 *         chunk has no B token);  n_src = number of A tokens = sum over chunks of ceil(L/2),
 *         sources ordered by position.
 *   score [batch, heads, n_src] fp32: cosine similarity of that edge.
 * bf16 keys: dot products of the stored values on bf16 MFMA with fp32 accumulation, inverse norms
 * in fp32 applied afterwards (keys are not re-rounded).  Supported: bf16 dim 64 or 128; fp32 dim
 * 16, 32, 64 or 128 (plain fp32 FMA through LDS: a correctness path for small caches, not tuned
 * against a roofline). */
int ckv_match(const void* K, const ckv_layout* in, int32_t chunk, int32_t* dst, float* score,
              void* hip_stream);

/* Compress a KV cache (Algorithm 1, the loop after prefill; Sec. 5.2-5.3).
 *   K, V     inputs, layout `in`;  deg_in [batch, heads, seq] int32 cluster degrees (row stride
 *            in->deg_stride) or NULL (= 1).
 *   K_out, V_out  layout `out` (same batch/heads/dim/dtype; out->seq >= plan.out_seq); rows
 *            [0, plan.out_seq) of every (batch, head) are written: the retained tokens in their
 *            original order, each B token replaced by the degree-weighted mean of itself and the
 *            A tokens merged into it (keys and values alike), rounded to nearest-even.
 *   deg_out  [batch, heads, out->seq] int32 degrees of the output tokens (row stride out->deg_stride).
 *   assign   [batch, heads, seq] int32 or NULL: output index of the centroid each INPUT token
 *            ended up in (composition over rounds).
 *   workspace  >= plan.workspace_bytes, 256-byte aligned.
 * Every round re-chunks the current sequence with the same chunk size.
 * Routes (p->flags; none of them changes a result bit): by default a round with r = 1 that opens
 * or closes the schedule together with its successor leaves the values to that successor, which
 * rebuilds them from the round's input, once the job is large enough for that to pay;
 * CKV_ROUTE_FULL_ROUNDS makes every round write its value cache, CKV_ROUTE_DEFER_ALWAYS defers
 * whatever the size.  ckv_plan sizes the workspace for the route the same flags select. */
int ckv_compress(const void* K, const void* V, const int32_t* deg_in, const ckv_layout* in,
                 const ckv_params* p, void* K_out, void* V_out, int32_t* deg_out,
                 const ckv_layout* out, int32_t* assign, void* workspace, size_t workspace_bytes,
                 void* hip_stream);

/* Host only.  The annealed schedule of merge fractions (Eq. 4) run as Algorithm 1's loop after
 * prefill: starting from `seq` tokens, rounds j = 0, 1, ... with r_j = max(r_init - j*delta_r,
 * r_floor) are added while the cache is longer than `budget` tokens (budget = R*n in Algorithm 1).
 * Fills *out (chunk, n_sink, n_recent, scope, n_rounds, r[]) for ckv_plan / ckv_compress; zero rounds
 * (budget already met) gives the identity.  The paper states no floor: r_floor = 0 is Eq. 4 as
 * printed, and then CKV_EUNSUPPORTED is returned when a round removes nothing while the cache is
 * still above the budget, or when more than CKV_MAX_ROUNDS rounds would be needed. */
int ckv_schedule_annealed(int32_t seq, int32_t chunk, int32_t n_sink, int32_t n_recent, int32_t scope,
                          int32_t budget, float r_init, float delta_r, float r_floor, ckv_params* out);

/* Cache update of one decode step (Algorithm 1, decoding part: K = [K, k], V = [V, v], N = [N, 1]).
 *   k_new, v_new [batch, heads, dim] contiguous, the cache's dtype, device.
 *   K, V     the cache, layout `cache` with cache->seq = its CAPACITY in tokens; deg [batch, heads,
 *            capacity] int32 (row stride cache->deg_stride) or NULL.
 *   lens     device int32 [batch] or NULL.  With lens: the token of sequence b is written to row
 *            lens[b] of every head, its degree set to 1, and lens[b] is incremented on the stream
 *            afterwards; a sequence with lens[b] already at capacity is left untouched.  Without:
 *            row `pos` of every sequence (CKV_ESHAPE when pos is outside [0, capacity)).
 * To re-cluster (Algorithm 1: once the cache holds budget + g tokens), call ckv_compress with a
 * layout whose seq is the current length, deg_in = deg, and one round. */
int ckv_append(const void* k_new, const void* v_new, void* K, void* V, int32_t* deg, const ckv_layout* cache,
               int32_t* lens, int32_t pos, void* hip_stream);

/* Scratch bytes ckv_decode_attn needs for this cache shape and number of query heads.
 * Workspace contract (ckv_decode_attn and ckv_paged_decode_attn): the first 4 * batch * heads bytes
 * are arrival counters, one int32 per (batch, KV head).  They must be ZERO when a call starts and
 * every call leaves them zero, so zero-fill a workspace once when it is allocated; after that it
 * serves any number of calls (of any length it is large enough for) without being touched.  Before
 * a call with a larger batch * heads than the workspace has served since it was last zeroed, zero
 * it again (the counters of the larger call reach into what earlier calls used as scratch).  With
 * counters that are not zero the output is wrong; nothing waits on them, so no call can hang.
 * Calls that share a workspace must not overlap in time. */
int ckv_decode_attn_workspace(const ckv_layout* kv, int32_t q_heads, size_t* bytes);

/* One decode step of attention over a (compressed) cache (Eq. 3; Algorithm 1 decode line):
 *   o[b,h,:] = softmax( q[b,h,:] . K[b,kvh,t,:] * scale + ln deg[b,kvh,t] ) . V[b,kvh,t,:],
 *   t < lens[b], kvh = h / (q_heads / kv->heads).
 *   q [batch, q_heads, dim] contiguous, same dtype as the cache; lens [batch] int32 (each
 *   <= kv->seq; 0 gives a zero output) or NULL (= kv->seq); deg [batch, heads, kv->seq] int32
 *   (>= 1; row stride kv->deg_stride) or NULL (= 1: plain attention, Eq. 1); scale <= 0 selects 1/sqrt(dim);
 *   o [batch, q_heads, dim] contiguous in o_dtype.  Arithmetic is fp32.  One kernel launch: the
 *   sequence is split into slices, and the slice that finishes last for a (batch, KV head) merges
 *   the partial results of all of them in slice order (run-to-run identical bits).
 * Supported: q_heads / kv->heads in {1,2,4,8}; bf16 dim 64/128; fp32 dim 32/64/128. */
int ckv_decode_attn(const void* q, int32_t q_heads, const void* K, const void* V,
                    const ckv_layout* kv, const int32_t* lens, const int32_t* deg, float scale,
                    void* o, int32_t o_dtype, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/* ckv_decode_attn without a workspace argument, for callers that cannot allocate device memory:
 * code recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and same result bits as ckv_decode_attn; the split partials and arrival
 * counters live in a device array of CKV_NOALLOC_SCRATCH_BYTES that is part of the library (each
 * GPU the library runs on holds its own copy until the process ends; the first call on a device
 * looks its address up).  The call allocates and frees nothing and launches nothing but the
 * attention kernel: the arrival counters keep the array's first 64 KiB to themselves (zero when the
 * library is loaded, left at zero by every call), the partials use the rest.
 * CKV_EWORKSPACE when batch * kv->heads exceeds 16384 or the partials (ckv_decode_attn_workspace()
 * minus its counters) exceed CKV_NOALLOC_SCRATCH_BYTES - 64 KiB (the Llama-3-8B decode shapes,
 * batch 1 to 16 at 32 query heads, need about 1.1 MB).  All calls on
 * one GPU share that one array: calls that overlap in time on the same GPU (different streams or
 * threads) race; issue them on one stream, or otherwise order them. */
#define CKV_NOALLOC_SCRATCH_BYTES (4u << 20)
int ckv_decode_attn_noalloc(const void* q, int32_t q_heads, const void* K, const void* V,
                            const ckv_layout* kv, const int32_t* lens, const int32_t* deg, float scale,
                            void* o, int32_t o_dtype, void* hip_stream);

/* ---- block-paged caches (the layout a serving engine's block manager keeps) ------------------
 * Pool: K_pool, V_pool [n_blocks, heads, block_size, dim] contiguous (inside a block the tokens of
 * one head are contiguous: block_size*dim elements per (block, head), which keeps a head's
 * stream in long runs), deg_pool [n_blocks, heads, block_size] int32.  block_table [batch, max_blocks] int32 (device): token t of
 * sequence b lives in block block_table[b][t / block_size] at offset t % block_size.  An entry
 * outside [0, n_blocks) is never dereferenced: its tokens are masked (attention), read as zero rows
 * of degree 1 (gather) or skipped (scatter). */
typedef struct {
  int32_t batch, heads, dim, dtype; /* dtype: ckv_dtype */
  int32_t block_size;               /* tokens per block: a power of two, 1..1024 */
  int32_t max_blocks;               /* entries per row of the block table */
  int32_t n_blocks;                 /* blocks in the pool */
} ckv_paged_layout;

/* ckv_decode_attn (Eq. 3) reading the paged cache in place.  lens [batch] int32 (device, required):
 * tokens of each sequence; max_len: host upper bound on them (sizes the split of the sequence;
 * lengths are clamped to it and to max_blocks*block_size).  deg_pool NULL = all ones (Eq. 1).
 * CKV_EUNSUPPORTED for a pool of 2^31 token rows (n_blocks*heads*block_size) or more. */
int ckv_paged_decode_attn_workspace(const ckv_paged_layout* pl, int32_t q_heads, int32_t max_len, size_t* bytes);
int ckv_paged_decode_attn(const void* q, int32_t q_heads, const void* K_pool, const void* V_pool,
                          const int32_t* deg_pool, const int32_t* block_table, const int32_t* lens,
                          const ckv_paged_layout* pl, int32_t max_len, float scale, void* o, int32_t o_dtype,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* ckv_append on pages (Algorithm 1, decoding part): the new token of sequence b (k_new, v_new
 * [batch, heads, dim] contiguous) goes to position lens[b] of every head with degree 1, and lens[b]
 * is incremented on the stream afterwards.  The caller's block manager must have put a block at
 * block_table[b][lens[b] / block_size]; a sequence without one there is left untouched. */
int ckv_paged_append(const void* k_new, const void* v_new, void* K_pool, void* V_pool, int32_t* deg_pool,
                     const int32_t* block_table, int32_t* lens, const ckv_paged_layout* pl, void* hip_stream);

/* Copy the first `seq` tokens of every sequence from the pool into strided tensors K, V (layout
 * `out`, out->seq >= seq) and deg (row stride out->deg_stride; may be NULL), or back. */
int ckv_paged_gather(const void* K_pool, const void* V_pool, const int32_t* deg_pool, const int32_t* block_table,
                     const ckv_paged_layout* pl, int32_t seq, void* K, void* V, int32_t* deg,
                     const ckv_layout* out, void* hip_stream);
/* Scatter writes tokens [0, in->seq) of every sequence into its blocks and RELEASES the blocks the
 * sequence no longer needs: with old_seq the length before, table entries
 * [ceil(in->seq / bs), ceil(old_seq / bs)) are copied to freed [batch, n_freed] (may be NULL) and
 * set to -1; lens[b] := in->seq when lens != NULL.  deg NULL writes degree 1. */
int ckv_paged_scatter(const void* K, const void* V, const int32_t* deg, const ckv_layout* in, void* K_pool,
                      void* V_pool, int32_t* deg_pool, int32_t* block_table, const ckv_paged_layout* pl,
                      int32_t old_seq, int32_t* freed, int32_t* lens, void* hip_stream);

/* Host only.  Blocks per sequence that ckv_paged_scatter releases when a sequence of old_seq tokens
 * shrinks to new_seq tokens: ceil(old_seq / bs) - ceil(new_seq / bs); negative status for bad
 * arguments (new_seq > old_seq included). */
int32_t ckv_paged_freed_blocks(const ckv_paged_layout* pl, int32_t old_seq, int32_t new_seq);

/* ckv_compress on sequences that live in a paged cache (the serving-engine integration: read the
 * paged cache, compress, write the centroids back, hand the freed blocks to the block manager), with
 * the result written into the sequences' own first blocks (compaction) and the blocks behind the new
 * length released as in ckv_paged_scatter.
 *   seq_lens  HOST int32 [batch] or NULL: tokens of every sequence before the call (NULL: all `seq`).
 *             Neighbouring sequences of equal length are compressed together, so a batch sorted by
 *             length costs few launches.
 *   lens      DEVICE int32 [batch] or NULL: set to the new lengths on the stream.
 *   freed     DEVICE int32 [batch, freed_stride] or NULL: the released block ids of every sequence,
 *             padded with -1; freed_stride >= the plan's n_freed.
 * The kernels read and write the pools through the block table: the first round's similarity and
 * merge kernels read pages in place, and the last round writes every output whose pool no workgroup
 * of that round still reads straight into its pages (with two or more rounds: the keys, and unless the
 * schedule is a single deferred pair also the values and degrees); the other outputs pass through a
 * staging tensor in the workspace and one scatter.  Nothing is gathered.  Same result bits as
 * ckv_compress on the same tokens.  deg_pool is required (it receives the degrees).
 * Supported: blocks of 8 tokens or more, pools of fewer than 2^31 token rows, batch <= 4096.
 * ckv_paged_compress_plan (host only): out_seq receives the length after compression of every
 * sequence ([batch] entries when seq_lens is given, one entry otherwise; may be NULL), n_freed the
 * largest number of blocks a sequence releases, workspace_bytes the scratch the call needs. */
int ckv_paged_compress_plan(const ckv_paged_layout* pl, int32_t seq, const int32_t* seq_lens, const ckv_params* p,
                            int32_t* out_seq, int32_t* n_freed, size_t* workspace_bytes);
int ckv_paged_compress(void* K_pool, void* V_pool, int32_t* deg_pool, int32_t* block_table, int32_t* lens,
                       const ckv_paged_layout* pl, int32_t seq, const int32_t* seq_lens, const ckv_params* p,
                       int32_t* freed, int32_t freed_stride, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Per-kernel timing for benchmarks.  When enabled, every kernel launch of the calling process
 * is bracketed by HIP events on its stream (a few microseconds per launch, on the host and on the
 * GPU: 32 attention layers lose about a quarter of their speed to it).  ckv_timing_select narrows
 * that to the kernels whose timing name starts with `prefix` (NULL or "" = all again), so a
 * benchmark can time its dominant kernel inside the measured region and leave the rest alone.
 * ckv_timing_read synchronises with the recorded events, then fills up to `max` entries with the
 * accumulated time per kernel since the last reset and returns the number of kernels (or a
 * negative status).  Not thread-safe; meant for a single benchmarking thread. */
typedef struct {
  char name[48];
  double total_ms;
  int64_t launches;
} ckv_kernel_time;
int ckv_timing_enable(int on);
int ckv_timing_select(const char* prefix);
int ckv_timing_reset(void);
int ckv_timing_read(ckv_kernel_time* out, int max);

/* Measurement aid for benchmarks (not part of the method): launches, once, a kernel that does
 * nothing but bf16 MFMA 32x32x16 instructions on every CU - `waves_per_cu` (4 or 8) waves, each with
 * independent accumulator chains, `iters` rounds of 8 k-steps, operands holding pseudo-random finite
 * values - and stores in *flops the floating-point operations it performs; timed through the timing
 * hooks below (kernel name "mfma_ceiling") it gives the MFMA rate this chip sustains under its own
 * power management, the practical ceiling the similarity stage is to be read against beside the
 * nominal 2.5 PFLOP/s.  mode 0: operands in registers; 1: one operand fragment read from LDS per
 * 2 MFMAs (the similarity kernel's ratio); 2: per 4 MFMAs (waves_per_cu 4 only).
 * scratch: device, 256-byte aligned, >= 65536 + CUs * 2048 bytes (1 MiB is enough). */
int ckv_bench_mfma_ceiling(int32_t mode, int32_t waves_per_cu, int32_t iters, void* scratch, size_t scratch_bytes,
                           double* flops, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CKV_H */
