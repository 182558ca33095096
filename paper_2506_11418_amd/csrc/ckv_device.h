// Device helpers shared by the kernel translation units of libckv (bf16 pieces, LDS swizzle,
// lane-group sums, the fused tile argmax, and the single-rounding bf16 quotient).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ckv_internal.h"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;


typedef __attribute__((ext_vector_type(2))) float f32x2;

union Piece {   // 16 bytes = 8 bf16
  uint4 u;
  bf16x8 v;
  bf16x2 p[4];
};

__device__ inline float sumsq8(const Piece& x) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) s = __builtin_amdgcn_fdot2_f32_bf16(x.p[i], x.p[i], s, false);
  return s;
}

// 1/sqrt(ss) by the hardware reciprocal square root (1 ulp), 0 for a zero key.
__device__ inline float inv_norm(float ss) { return ss > 0.f ? __builtin_amdgcn_rsqf(ss) : 0.f; }

// 1/|k| of a row held as MFMA operand fragments: a lane holds the pieces of its lane half, the lane
// 32 away the other pieces of the same row.  Every kernel that scores with this row's norm uses
// this one summation order, so their scores agree bit for bit.
template <int KSTEPS>
__device__ __forceinline__ float inv_norm_of_operand_row(const bf16x8 (&frag)[KSTEPS]) {
  float ss = 0.f;
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) {
    Piece pc;
    pc.v = frag[s];
    ss += sumsq8(pc);
  }
  ss += __shfl_xor(ss, 32);
  return inv_norm(ss);
}

// Sum over the LANES lanes (8 or 16, aligned) that hold one key row, with DPP adds: xor 1 and
// xor 2 inside each quad, then the mirrored half-row and row (after the quad steps all lanes of
// a quad agree, so a mirror brings in exactly the other quad's / other half's sum).
template <int LANES>
__device__ __forceinline__ float row_sum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));
  if (LANES == 16)
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));
  return x;
}

// Block-pool rows of a workgroup's tokens.  stage_row_bases fills s_rb[i] with the pool row of the
// first token of block (first_blk + i) of sequence b for head h (-1 for a table entry outside the
// pool), for the blocks that hold tokens [u_first, u_last] of the sequence; paged_row then turns a
// token into its pool row with one LDS read.  A block outside the pool reads as row 0 (always valid
// memory, contents meaningless) and is not written.
struct RowBases {
  const int32_t* s_rb;
  int blk0, shift, mask;
  __device__ __forceinline__ int base_of(int u) const { return s_rb[(u >> shift) - blk0]; }
  __device__ __forceinline__ int row(int u) const {            // for reads
    const int rb = base_of(u);
    return rb < 0 ? 0 : rb + (u & mask);
  }
};
__device__ inline RowBases stage_row_bases(int32_t* s_rb, const PagedSide& pg, int b, int h, int heads, int u_first,
                                           int u_last, int tid, int n_threads) {
  const int blk0 = u_first >> pg.shift, n = (u_last >> pg.shift) - blk0 + 1;
  const int32_t* row = pg.table + (int64_t)b * pg.max_blocks;
  for (int i = tid; i < n; i += n_threads) {
    const int blk = (blk0 + i < pg.max_blocks) ? row[blk0 + i] : -1;
    s_rb[i] = ((unsigned)blk < (unsigned)pg.n_blocks) ? ((blk * heads + h) << pg.shift) : -1;
  }
  return RowBases{s_rb, blk0, pg.shift, (1 << pg.shift) - 1};
}

// Map dispatch order to logical work so that the 8 XCDs (which receive consecutive workgroup ids
// round-robin) each walk a contiguous range: neighbours in the range (the A blocks of one chunk,
// adjacent chunks) then share an L2.
__device__ inline int xcd_remap(int id, int per_xcd) { return (id & 7) * per_xcd + (id >> 3); }

// Fold one 32x32 tile of S^T into the running (max, argmax) of this lane's A row.  sc = acc/|k_j|
// (the row's own 1/|k_i| > 0 cannot change the argmax and is applied at the end).  Tiles arrive in
// rotated order, so an equal maximum from a tile of LOWER B indices also replaces the incumbent:
// the result is the lowest index among all maxima, whatever the visiting order.
template <bool RAGGED>
__device__ __forceinline__ void tile_argmax(const f32x16& acc, const f32x4 (&ib)[4], int jbase, int half,
                                            int valid, float& best, int& bestj) {
  float sc[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    sc[r] = acc[r] * ib[r >> 2][r & 3];
    if (RAGGED && (8 * (r >> 2) + 4 * half + (r & 3)) >= valid) sc[r] = -INFINITY;
  }
  float mt = __builtin_fmaxf(sc[0], sc[1]);
#pragma unroll
  for (int r = 2; r < 16; r += 2) mt = __builtin_fmaxf(__builtin_fmaxf(mt, sc[r]), sc[r + 1]);
  const bool upd = (mt > best) | ((mt == best) & (jbase < bestj));
  if (__any(upd)) {
    int idx = 0;
#pragma unroll
    for (int r = 15; r >= 0; --r) idx = (sc[r] == mt) ? r : idx;
    const int j = jbase + ((idx >> 2) << 3) + (half << 2) + (idx & 3);
    best = upd ? mt : best;
    bestj = upd ? j : bestj;
  }
}


// The same fold as straight-line code cut into 16 steps of at most 8 vector instructions (two
// tiles of the same 32 B rows at once), so that a caller can place one step behind each MFMA of
// the NEXT tile.  Only valid when tiles arrive in INCREASING order of B index: a strict
// comparison then keeps the lowest index among equal maxima.  jlane = first B row of the tile
// + 4 * lane half; accumulator r is B row 8*(r/4) + r%4 past it.  The scaled scores overwrite
// the accumulators' registers.
// The maximum is taken as a running maximum over the four quads of accumulators, q[k] = max of
// accumulators 0 .. 4k+3.  The lowest quad with q[k] == q[3] holds the first maximum: its four
// scores are picked with nested selects and searched, 25 instructions instead of the 31 of a
// compare + select per accumulator.  Steps 11..15 are empty.
struct FoldRegs {
  float s[2][16];      // scaled scores (held apart from the accumulator vectors: a select between two
                       // elements of ONE vector would be turned into a run-time element index)
  float q[2][4];       // running quad maxima; q[.][3] is the tile's maximum
  float x[2][4];       // the scores of the lowest quad that holds it
  int base[2];         // that quad's first B row, then the B row of the maximum
};
constexpr int kFoldSteps = 16;
template <int STEP, int T>   // the part of step STEP that belongs to tile T (accumulators v)
__device__ __forceinline__ void fold_step_tile(const f32x16& v, const f32x4 (&ib)[4], FoldRegs& f, int jlane,
                                               float& best, int& bestj) {
  float(&s)[16] = f.s[T];
  float(&q)[4] = f.q[T];
  float(&x)[4] = f.x[T];
  if constexpr (STEP < 4) {                       // scale by 1/|k_j|
#pragma unroll
    for (int i = 0; i < 4; ++i) s[4 * STEP + i] = v[4 * STEP + i] * ib[STEP][i];
  } else if constexpr (STEP == 4) {               // running quad maxima
    q[0] = __builtin_fmaxf(__builtin_fmaxf(__builtin_fmaxf(s[0], s[1]), s[2]), s[3]);
    q[1] = __builtin_fmaxf(__builtin_fmaxf(__builtin_fmaxf(q[0], s[4]), s[5]), __builtin_fmaxf(s[6], s[7]));
  } else if constexpr (STEP == 5) {
    q[2] = __builtin_fmaxf(__builtin_fmaxf(__builtin_fmaxf(q[1], s[8]), s[9]), __builtin_fmaxf(s[10], s[11]));
    q[3] = __builtin_fmaxf(__builtin_fmaxf(__builtin_fmaxf(q[2], s[12]), s[13]), __builtin_fmaxf(s[14], s[15]));
  } else if constexpr (STEP >= 6 && STEP <= 8) {  // the scores and first row of the lowest quad that
    constexpr int K = 8 - STEP;                   // has reached the maximum: quad 2 against 3, then 1, 0
    const bool in = q[K] == q[3];
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = in ? s[4 * K + i] : (K == 2 ? s[12 + i] : x[i]);
    f.base[T] = in ? 8 * K : (K == 2 ? 24 : f.base[T]);
  } else if constexpr (STEP == 9) {               // the first of its scores that is the maximum
    int i = (x[2] == q[3]) ? 2 : 3;
    i = (x[1] == q[3]) ? 1 : i;
    i = (x[0] == q[3]) ? 0 : i;
    f.base[T] += i;
  } else if constexpr (STEP == 10) {              // into the running maxima
    const bool upd = q[3] > best;
    best = upd ? q[3] : best;
    bestj = upd ? jlane + f.base[T] : bestj;
  }
}

template <int STEP>
__device__ __forceinline__ void fold_step(f32x16& c0, f32x16& c1, const f32x4 (&ib)[4], FoldRegs& f, int jlane,
                                          float (&best)[2], int (&bestj)[2]) {
  fold_step_tile<STEP, 0>(c0, ib, f, jlane, best[0], bestj[0]);
  fold_step_tile<STEP, 1>(c1, ib, f, jlane, best[1], bestj[1]);
}

template <int FIRST, int LAST>   // steps FIRST .. LAST-1
__device__ __forceinline__ void fold_steps(f32x16& c0, f32x16& c1, const f32x4 (&ib)[4], FoldRegs& f, int jlane,
                                           float (&best)[2], int (&bestj)[2]) {
  if constexpr (FIRST < LAST && FIRST < kFoldSteps) {
    fold_step<FIRST>(c0, c1, ib, f, jlane, best, bestj);
    fold_steps<FIRST + 1, LAST>(c0, c1, ib, f, jlane, best, bestj);
  }
}

// acc[0..8)/n as 8 packed bf16, ONE nearest-even rounding (n < 2^21).
// q = acc * (1/n) with a reciprocal good to an ulp lies within 3 ulp(fp32) of the true quotient
// t.  For n a power of two q = t.  Otherwise the converter's rounding of q can differ from that of
// t only if q sits within those 3 ulp of a bf16 midpoint M (low 16 bits in 0x7ffd..0x8003), and not
// even then if q*n == acc exactly (sums of bf16 values divide evenly quite often; q = t then).
// The remaining elements are decided exactly: r = acc - q*n is representable, so fma gives it
// without error; q - M is exact; and (t - M)*n = (q - M)*n + r, whose sign one more fma delivers
// (rounding keeps signs and zeros).  |t| > |M| rounds away from zero, a zero means t = M (tie to
// even).  That path is taken for the whole wave only when some element needs it.
__device__ __forceinline__ uint32_t round_bf16_near_midpoint(float S, float fn, float q) {
  const uint32_t u = __float_as_uint(q);
  const uint32_t H = u & 0xffff0000u;
  const float M = __uint_as_float(H | 0x8000u);
  const float r = fmaf(-q, fn, S);
  const float d = fmaf(q - M, fn, r);
  const bool away = (d > 0.f) == ((u >> 31) == 0u);
  const uint32_t up = (d == 0.f) ? ((H >> 16) & 1u) : (away ? 1u : 0u);
  return ((H >> 16) + up) & 0xffffu;
}

__device__ __forceinline__ uint4 round_div_pack_bf16(const float* acc, int n) {
  const float fn = (float)n;
  // 1/n: hardware reciprocal (1 ulp) + one Newton step.  Exact for powers of two; otherwise within
  // an ulp of 1/n, which keeps q within the 3 ulp the window below allows for (checked on the CPU
  // against exact rational arithmetic with the reciprocal forced one ulp off either way).
  float rcp = __builtin_amdgcn_rcpf(fn);
  rcp = fmaf(fmaf(-fn, rcp, 1.0f), rcp, rcp);
  const bool pow2 = (n & (n - 1)) == 0;          // then acc*rcp IS the quotient: no second rounding
  float qv[8];
  uint32_t nearest = 0xffffffffu;                // min over the elements of (low 16 bits - 0x7ffd) mod 2^16
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    qv[i] = acc[i] * rcp;
    nearest = min(nearest, (uint32_t)(uint16_t)(__float_as_uint(qv[i]) - 0x7ffdu));
  }
  const bool window = (nearest <= 6u) & !pow2;
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f32x2 v = {qv[2 * i], qv[2 * i + 1]};
    w[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  }
  if (__any(window)) {   // some element sits next to a midpoint: does it divide evenly (then q is exact)?
    bool risky = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool win = ((__float_as_uint(qv[i]) & 0xffffu) - 0x7ffdu) <= 6u;
      risky |= win & (fmaf(-qv[i], fn, acc[i]) != 0.f);
    }
    risky &= !pow2;
    if (__any(risky)) {  // rare (a few 1e-4 per element): decide those elements exactly
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool win = !pow2 && ((__float_as_uint(qv[i]) & 0xffffu) - 0x7ffdu) <= 6u;
        if (win) {
          const uint32_t h = round_bf16_near_midpoint(acc[i], fn, qv[i]);
          w[i >> 1] = (i & 1) ? ((w[i >> 1] & 0x0000ffffu) | (h << 16)) : ((w[i >> 1] & 0xffff0000u) | h);
        }
      }
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Streaming 16-byte accesses: rows that are read or written once and not reused by this kernel
// are marked non-temporal so they do not displace reusable lines from the caches.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ldg16_stream(const void* p) {
  const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stg16_stream(void* p, const uint4& r) {
  __builtin_nontemporal_store(u32x4{r.x, r.y, r.z, r.w}, static_cast<u32x4*>(p));
}

// 16-byte load at a 32-bit byte offset from a workgroup-uniform base (the compiler then uses the
// scalar-base + vector-offset addressing form: no 64-bit address arithmetic per lane).
__device__ __forceinline__ uint4 ldg16(const void* base, uint32_t byte_off) {
  return *reinterpret_cast<const uint4*>(static_cast<const char*>(base) + byte_off);
}
__device__ __forceinline__ void stg16(void* base, uint32_t byte_off, const uint4& v) {
  *reinterpret_cast<uint4*>(static_cast<char*>(base) + byte_off) = v;
}

// acc += w * (8 bf16 of u), element order = memory order.  Integer weights up to 256 are exact in
// bf16, so each element is ONE v_dot2 of the packed pair with (w, 0) or (0, w): the product is
// exact, the other lane of the pair contributes an exact zero, and the single fp32 rounding is
// that of fmaf (for finite data; a non-finite element also poisons its pair partner).  Larger
// weights take the unpack + fma route.
template <bool WIDE>
__device__ __forceinline__ void fma_bf16x8_t(float* acc, const uint4& u, int w) {
  const uint32_t x[4] = {u.x, u.y, u.z, u.w};
  if (WIDE) {
    const float fw = (float)w;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[2 * i] = fmaf(fw, __uint_as_float(x[i] << 16), acc[2 * i]);
      acc[2 * i + 1] = fmaf(fw, __uint_as_float(x[i] & 0xffff0000u), acc[2 * i + 1]);
    }
  } else {
    // A weight known at compile time (a literal 1) would be encoded as an inline constant, which the
    // packed instruction does not read as (w, 0): such a weight is hidden from the compiler.  (The
    // test is resolved after inlining; a run-time weight compiles as if it were not there.)
    uint32_t wb = __float_as_uint((float)w);
    if (__builtin_constant_p(wb)) asm volatile("" : "+v"(wb));
    const bf16x2 w_lo = __builtin_bit_cast(bf16x2, wb >> 16), w_hi = __builtin_bit_cast(bf16x2, wb & 0xffff0000u);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bf16x2 xi = __builtin_bit_cast(bf16x2, x[i]);
      acc[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(xi, w_lo, acc[2 * i], false);
      acc[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(xi, w_hi, acc[2 * i + 1], false);
    }
  }
}
// Both routes give the same bits, so which one runs is a matter of speed only: the caller may
// decide per call (here) or once for a whole workgroup (the merge kernel's two emit versions).
__device__ __forceinline__ void fma_bf16x8(float* acc, const uint4& u, int w) {
  if (__any(w > 256)) fma_bf16x8_t<true>(acc, u, w);
  else fma_bf16x8_t<false>(acc, u, w);
}

}  // namespace ckv
