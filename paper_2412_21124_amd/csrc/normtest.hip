// libnormtest: norm-test statistics pass fused with AdamW, hand-written for gfx950 (MI355X).
//
// One streaming kernel (k_step) reads the J gradient rows and w, m, v once, writes w, m, v once and
// leaves five fp64 values per fixed-size tile of coordinates (the sums A, B, C, the count of coordinates
// failing the coordinate-wise form of the test, and their largest ratio); k_reduce_groups / k_finalize then add
// the tile partials in double-double arithmetic and take Alg. 1's decision on the device.  The partials stay in the caller's workspace
// behind a small record of the step, from which k_layer_stats can regroup them into a per-layer table.
// k_adamw_gbar is the second phase of the gradient-clipped variant.  The
// path is bound by HBM bandwidth (about two lane-operations per byte), so there is no MFMA here: the work is
// fully coalesced 8- and 16-byte accesses, fp32 per-coordinate arithmetic, fp64 accumulation and wave64
// shuffle reductions.  Launch shapes (block size, sweeps per tile, coordinates per launch) differ per class of
// call and were chosen by measurement; see tile_cfg() and the NT_CHUNK_* constants.  Two things about the memory
// system shape the host side: blocks that start together stay in step for a while and are served faster than an
// even mix of loads and stores, so a long vector is walked by several launches; and writes sprinkled among many
// reads cost several times their volume, so with more than 16 rows (fast_tile_multi), and in long vectors from 28
// bytes of gradient per coordinate on (fast_tile_defer), a block updates the state of its whole tile only after it
// has read all the rows.
//
// Numerics.  The centred sum C = sum_j (g_j - gbar)^2 is formed directly from the J values of a
// coordinate held in registers, never as A - B/J (which cancels badly when the workers agree).  A
// rounding error e in gbar only adds J e^2 to a coordinate's centred sum because the cross term
// sums to zero.  For more than 16 rows the rows are taken 16 at a time, each chunk shifted by the
// running mean so far, and the chunks' means and centred sums are merged with the pairwise update
// M2 += M2_b + delta^2 n_a n_b / (n_a + n_b).  Row sums are carried in fp64, so the mean handed to
// AdamW is correctly rounded even when the rows cancel.
// Per-lane sums leave fp32 after one group of 4 coordinates; everything above is fp64 in a fixed
// order, so results do not depend on the grid size and are reproducible bit for bit.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "normtest.h"

// Launch shapes, chosen by measurement on MI355X (block size, block sweeps per partial-sum tile).
#define NT_BLOCK 1024            // J <= 16, fused step: one sweep of a large block per tile
#define NT_ITERS 1
#define NT_BLOCK_STATS 512       // J <= 16, statistics only: read-only and few bytes per lane, so smaller blocks
#define NT_ITERS_STATS 8         // that each walk a longer tile
#define NT_STATS_SHORT_COORDS (1ll << 21)  // ... in vectors shorter than this, the next shape (64 blocks of 512 threads
                                           // for 2^20 coordinates leave most of the chip idle: 18 -> 14 us at 8 rows)
#define NT_BLOCK_STATS_GBAR 512  // statistics that also store gbar (phase 1 of the clipped variant): one write
#define NT_ITERS_STATS_GBAR 2    // stream moves the optimum to shorter tiles
#define NT_BLOCK_ADAMW 1024      // J <= 16, AdamW only (test skipped)
#define NT_ITERS_ADAMW 1
#define NT_BLOCK_LARGE 128       // J > 16 (rows are walked inside each sweep), every mode that writes per coordinate:
#define NT_ITERS_LARGE 16        // a block walks the rows of all its sweeps first and writes for all of them afterwards,
#define NT_GENS_LARGE 1          // and a launch holds this many generations of blocks (CUs x blocks per CU)
#define NT_LDS_PAD_LARGE 1024    // LDS bytes on top of the 32 KB of means: four blocks per CU in every mode (five are slower)
#define NT_FEW_ROWS 20           // 17 .. this many rows: the same tile as 256 threads x 8 sweeps (fused step +9 % at 17 rows,
#define NT_BLOCK_FEW 256         // +7 % at 20, +3 % at 24 but AdamW only -1 % there, -1.5 % at 28): the walk is short
#define NT_ITERS_FEW 8           // there, and a block's life with it
// Up to 16 rows with at least NT_DEFER_ROW_BYTES of gradient per coordinate (14 bf16 or 7 fp32 rows; AdamW only:
// NT_DEFER_ROW_BYTES_ADAMW, 10 or 5 rows), in a vector of at least NT_DEFER_COORDS coordinates: a step that writes
// per coordinate runs like the many-row one, rows in registers but the update deferred and one generation of blocks
// per launch (+2 .. +8 % there; with fewer bytes per coordinate, or fewer than some eight generations, the
// interleaved class is as fast or faster).
#define NT_DEFER_ROW_BYTES 28
#define NT_DEFER_ROW_BYTES_ADAMW 20
#define NT_DEFER_COORDS (1ll << 26)
#define NT_BLOCK_DEFER 128
#define NT_ITERS_DEFER 16
#define NT_DEFER_UNROLL 1        // row sweeps in flight per lane in that class
#define NT_GENS_DEFER 1          // generations of blocks per launch in that class (two: -7 .. -10 %)
// J > 16, modes that write per coordinate: the shapes above from about one generation of blocks on (up to 32 rows,
// where a generation is short-lived and a half-empty one costs more, from two); shorter vectors in one launch of
// short tiles, else a few large blocks would have the chip to themselves (512 rows, d = 2^18: 607 -> 92 us).
#define NT_MANY_LONG_COORDS (3ll << 21)
#define NT_MANY_LONG_COORDS_32 (1ll << 24)
#define NT_BLOCK_MANY_SHORT 256
#define NT_ITERS_MANY_SHORT 2
#define NT_BLOCK_LARGE_STATS 256 // J > 16, statistics only (nothing written per coordinate): short tiles, so that a
#define NT_ITERS_LARGE_STATS 2   // vector of a few million coordinates still gives every CU several blocks
#define NT_BLOCKS_PER_CU 4096    // grid = min(tiles, CUs * this); blocks stride over tiles beyond that
// A long vector is walked by several launches of the step kernel, each over a run of consecutive tiles.  Blocks
// that start together move through their load and store phases together, so the memory system sees chip-wide
// bursts of reads and of writes instead of an even mix, which it serves faster; inside one long launch that
// lockstep drifts apart within some tens of block generations.  A kernel boundary restores it at the price of a
// drained machine for a few microseconds.  Coordinates per launch, by class (measured; 0: one launch):
#define NT_CHUNK_FULL (1ll << 27)        // J <= 16, fused step (+3 % at d = 1.5e9, +1 % at 16 rows)
#define NT_CHUNK_ADAMW (1ll << 25)       // J <= 16, AdamW only (+5 %)
#define NT_CHUNK_STATS_GBAR (1ll << 27)  // J <= 16, statistics + stored gbar (+2 % on the clipped step)
#define NT_CHUNK_STATS 0                 // statistics only: nothing is written, nothing to gain
#define NT_CHUNK_ADAMW_GBAR (1ll << 25)  // AdamW from a stored gbar (second phase of the clipped step)
// J > 16, modes that write per coordinate: one generation of blocks per launch, see launch_step_shape

#define NT_VEC 4              // coordinates per lane and sweep: 16-byte fp32 accesses, 8-byte bf16 row loads
#define NT_TILE_MAX 16384     // every tile size divides this: the alignment that keeps shard results bit-identical
#define NT_AUX_BLOCK 1024     // threads per block of the AdamW-from-gbar, copy and yardstick kernels

#define NT_JCHUNK 16          // up to this many rows a coordinate's values are all held in registers
#define NT_MCHUNK 16          // beyond that, rows are walked this many at a time (2 .. NT_JCHUNK + 1; 16 measured best)
#define NT_ROUND_TO_MAX (1ll << 31)  // bound on nt_hyper.round_to that keeps the rounding chain inside int64
#define NT_FIN_THREADS 1024
#define NT_FIN_SMALL 4096       // up to this many records the finalize kernel runs with 256 threads
#define NT_NSUM 4              // summed values per tile partial: A, B, C and the count of failing coordinates
#define NT_NV 5                // values per tile partial: the sums, then the largest coordinate-wise ratio
#define NT_GROUP_THREADS 256   // first-stage reduction: threads per block
#define NT_GROUP_TILES 2048    // ... and tile partials per block
#define NT_DIRECT_TILES 4096   // up to this many tiles one block reads the tile partials itself
#define NT_WS_HEADER 32        // doubles in front of the tile partials: a record of the step that wrote them
#define NT_WS_CONTROL 24       // ... of which this one starts the words the step's kernels hand to each other
#define NT_WS_MAGIC 0x4e54574f524b5350ll
#define NT_LAYER_THREADS 1024  // per-layer kernel: one block per layer

// Scratch of normtest_step_static: the per-tile partial sums and the record of the step, for callers that
// cannot hand over (or allocate) a workspace.  One copy per GPU, held until the process ends.
#define NT_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[NT_SCRATCH_BYTES];

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

enum { MODE_FULL = 0, MODE_STATS = 1, MODE_ADAMW = 2 };

template <bool NT, class T>
__device__ inline T ld_vec(const void* p) {
  if constexpr (NT)
    return __builtin_nontemporal_load((const T*)p);
  else
    return *(const T*)p;
}

struct F32 {
  static constexpr int VEC = 4;
  static constexpr int ESIZE = 4;
  typedef u32x4 raw_t;
  __device__ static inline raw_t ldraw(const void* p) { return ld_vec<true, raw_t>(p); }
  __device__ static inline float val(const raw_t& r, int e) { return __builtin_bit_cast(float, (uint32_t)r[e]); }
  __device__ static inline float ld(const void* base, int64_t i) { return ((const float*)base)[i]; }
};

struct BF16 {
  static constexpr int VEC = 4;
  static constexpr int ESIZE = 2;
  typedef u32x2 raw_t;
  __device__ static inline raw_t ldraw(const void* p) { return ld_vec<true, raw_t>(p); }
  // bfloat16 is the high half of a binary32: widening is a shift or a mask
  __device__ static inline float val(const raw_t& r, int e) {
    uint32_t u = r[e >> 1];
    return __builtin_bit_cast(float, (e & 1) ? (u & 0xffff0000u) : (u << 16));
  }
  __device__ static inline float ld(const void* base, int64_t i) {
    return __builtin_bit_cast(float, (uint32_t)((const uint16_t*)base)[i] << 16);
  }
};

struct StepParams {
  const void* grads; // row 0 of a strided matrix, or (TABLE kernels) a device array of J row pointers
  int64_t ld;       // row stride in elements
  int64_t d;
  int J;
  float* w;
  float* m;
  float* v;
  float* gbar;      // nullptr unless requested
  double* partials; // NT_NV doubles per tile
  double inv_J;
  float beta1, omb1, beta2, omb2; // omb = 1 - beta
  float decay;                    // 1 - lr * weight_decay
  float step_size;                // lr / (1 - beta1^k)
  float inv_sqrt_bc2;             // 1 / sqrt(1 - beta2^k)
  float eps;
  float coord_thr;   // eta^2 b_k (J - ddof) when the coordinate-wise count is wanted, else negative
};

// Words of the workspace record that kernels of one step hand to each other.
struct WsControl {
  unsigned int rows_aligned;  // pointer-table calls: 1 if every row pointer is 16-byte aligned
};

// Start of gradient row j: base + j*ld elements, or the j-th entry of the caller's pointer table.
template <class GT, bool TABLE>
__device__ inline const char* row_base(const StepParams& p, int j) {
  if constexpr (TABLE)
    return ((const char* const*)p.grads)[j];
  else
    return (const char*)p.grads + (int64_t)j * p.ld * GT::ESIZE;
}

__device__ inline u32x4 ld16(const void* p) { return ld_vec<true, u32x4>(p); }
__device__ inline void st16(void* p, f32x4 x) { __builtin_nontemporal_store(x, (f32x4*)p); }

// AdamW on one coordinate (Alg. 1): moments, bias corrections folded into step_size and
// inv_sqrt_bc2, decoupled decay.  sqrt and reciprocal are the 1-ulp hardware forms: the term they
// feed is scaled by lr before it meets w.  The hardware square root flushes subnormal arguments to
// zero, so a second moment below 2^-96 is scaled by 2^64 first (same bits for every normal v).
__device__ inline void adamw_coord(const StepParams& p, float g, float& w, float& m, float& v) {
  m = __builtin_fmaf(p.beta1, m, p.omb1 * g);
  v = __builtin_fmaf(p.beta2, v, (p.omb2 * g) * g);
  const bool tiny = v < 0x1p-96f;
  float root = __builtin_amdgcn_sqrtf(tiny ? v * 0x1p+64f : v);
  root = tiny ? root * 0x1p-32f : root;
  float denom = __builtin_fmaf(root, p.inv_sqrt_bc2, p.eps);
  float upd = (p.step_size * m) * __builtin_amdgcn_rcpf(denom);
  w = __builtin_fmaf(p.decay, w, -upd);
}

// fixed-order sum of a lane's VEC per-coordinate terms
template <int N>
__device__ inline float lane_tree(const float* x) {
  static_assert(N == 4, "per-coordinate terms leave fp32 in groups of four");
  return (x[0] + x[1]) + (x[2] + x[3]);
}

__device__ inline double wave_sum(double x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}
__device__ inline float wave_max(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = __builtin_fmaxf(x, __shfl_xor(x, off, 64));
  return x;
}

// What a lane gathers over the sweeps of one tile: the three sums in fp64 (each fed with fp32 sums of four
// coordinates), the number of coordinates failing the coordinate-wise test and their largest ratio.
struct LaneAcc {
  double A = 0.0, B = 0.0, C = 0.0;
  int nfail = 0;
  float rmax = 0.f;
};

// Block partial of one tile -> partials[NT_NV*tile ..].  `buf` alternates between tiles so that one
// barrier per tile is enough.
template <int BLOCK>
__device__ inline void tile_reduce(const LaneAcc& acc, double (*red)[BLOCK / 64][NT_NV], int buf, double* partials,
                                   int64_t tile) {
  const double a = wave_sum(acc.A), b = wave_sum(acc.B), c = wave_sum(acc.C), n = wave_sum((double)acc.nfail);
  const float r = wave_max(acc.rmax);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
    red[buf][wave][0] = a;
    red[buf][wave][1] = b;
    red[buf][wave][2] = c;
    red[buf][wave][3] = n;
    red[buf][wave][4] = (double)r;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double sa = red[buf][0][0], sb = red[buf][0][1], sc = red[buf][0][2], sn = red[buf][0][3], sr = red[buf][0][4];
#pragma unroll
    for (int wv = 1; wv < BLOCK / 64; ++wv) {
      sa += red[buf][wv][0];
      sb += red[buf][wv][1];
      sc += red[buf][wv][2];
      sn += red[buf][wv][3];
      sr = __builtin_fmax(sr, red[buf][wv][4]);
    }
    partials[NT_NV * tile + 0] = sa;
    partials[NT_NV * tile + 1] = sb;
    partials[NT_NV * tile + 2] = sc;
    partials[NT_NV * tile + 3] = sn;
    partials[NT_NV * tile + 4] = sr;
  }
}

// Coordinate-wise form of the test (Sec. 4, Prop. 1): with thr = eta^2 b_k (J - ddof), a coordinate with centred
// sum c and mean gb has the ratio c / (thr gb^2) and fails when that exceeds one.  A coordinate without spread
// has ratio 0 whatever its mean; spread around a zero mean gives +inf.  thr < 0 switches both off.
__device__ inline void coord_test(float thr, float c, float gb, LaneAcc& acc) {
  if (thr >= 0.f) {
    const float den = thr * (gb * gb);
    acc.nfail += (c > den) ? 1 : 0;
    const float rho = (c == 0.f) ? 0.f : c / den;
    acc.rmax = __builtin_fmaxf(acc.rmax, rho);
  }
}

// Per-chunk bookkeeping of the J > 16 walk, shared by the fast and the guarded path so that both
// perform the same operations.  For one coordinate and a chunk of nb rows with shift K (the running
// mean before the chunk, or the first row for the first chunk) two sums have been accumulated:
// sb = sum x in fp64 (exact for all practical purposes, so the mean handed to AdamW is correctly rounded
// even when the rows cancel) and q = sum (x - K)^2 in fp32.  With sr = sb - nb K, the sum of the shifted values,
//   chunk centred sum   M2_b = q - sr^2/nb
//   chunk sum of squares  a_b = q + K (2 sr + nb K)
// and the chunk is merged into the running (S, M2) with  S += sb,  M2 += M2_b + delta^2 na nb/(na + nb),
// delta = mean_b - mean_a.  Returns the shift for the next chunk.
__device__ inline float chunk_merge(bool first, int na, int nb, float K, double sb, float q, double& S, float& M2,
                                    float& a) {
  const double sr = __builtin_fma(-(double)K, (double)nb, sb);
  const float srf = (float)sr;
  const float nbf = (float)nb;
  const double inv_nb = 1.0 / (double)nb;
  const float M2b = __builtin_fmaf(-(srf * (float)inv_nb), srf, q);
  a += __builtin_fmaf(K, __builtin_fmaf(nbf, K, 2.0f * srf), q);
  if (first) {
    S = sb;
    M2 = M2b;
  } else {
    const float coef = ((float)na * nbf) / (float)(na + nb);
    const float delta = (float)(((double)K - S * (1.0 / (double)na)) + sr * inv_nb);
    M2 = M2 + __builtin_fmaf(delta * delta, coef, M2b);
    S = S + sb;
  }
  return (float)(S * (1.0 / (double)(na + nb)));
}

// ---------------------------------------------------------------------------------------------
// Guarded tile: any J, any alignment, ragged end.  Same lane-to-coordinate map and the same
// sequence of floating-point operations per coordinate as the fast tiles below (rows are re-read
// instead of held in registers), so a tile's partial sums and outputs have the same bits on either
// path.  Coordinates at or beyond d contribute exact zeros.
// ---------------------------------------------------------------------------------------------
template <class GT, bool TABLE>
__device__ inline void coord_stats_generic(const StepParams& p, int64_t i, double& S, float& M2, float& a) {
  const int J = p.J;
  a = 0.f;
  if (J <= NT_JCHUNK) {
    // all rows at once: fp64 row sum, then squares centred on the mean, exactly as in the fast tile
    double sb = (double)GT::ld(row_base<GT, TABLE>(p, 0), i);
    for (int j = 1; j < J; ++j) sb += (double)GT::ld(row_base<GT, TABLE>(p, j), i);
    const float mb = (float)(sb * p.inv_J);
    float cb = 0.f;
    for (int j = 0; j < J; ++j) {
      const float x = GT::ld(row_base<GT, TABLE>(p, j), i);
      const float r = x - mb;
      cb = __builtin_fmaf(r, r, cb);
      a = __builtin_fmaf(x, x, a);
    }
    S = sb;
    M2 = cb;
    return;
  }
  float K = GT::ld(row_base<GT, TABLE>(p, 0), i);
  int na = 0;
  for (int j0 = 0; j0 < J; j0 += NT_MCHUNK) {
    const int nb = (J - j0 < NT_MCHUNK) ? (J - j0) : NT_MCHUNK;
    double sb = 0.0;
    float q = 0.f;
    for (int j = 0; j < nb; ++j) {
      const float x = GT::ld(row_base<GT, TABLE>(p, j0 + j), i);
      const float r = x - K;
      sb += (double)x;
      q = __builtin_fmaf(r, r, q);
    }
    K = chunk_merge(na == 0, na, nb, K, sb, q, S, M2, a);
    na += nb;
  }
}

// The same for a row count known at compile time (2 .. NT_JCHUNK): the J loads of a coordinate are issued
// together and kept in registers; the arithmetic is coord_stats_generic's, operation for operation.
// J_T = 0 forwards to the generic form.
template <class GT, bool TABLE, int J_T>
__device__ inline void coord_stats(const StepParams& p, int64_t i, double& S, float& M2, float& a) {
  if constexpr (J_T > 0) {
    float x[J_T];
#pragma unroll
    for (int j = 0; j < J_T; ++j) x[j] = GT::ld(row_base<GT, TABLE>(p, j), i);
    S = (double)x[0];
#pragma unroll
    for (int j = 1; j < J_T; ++j) S += (double)x[j];
    const float mb = (float)(S * p.inv_J);
    M2 = 0.f;
    a = 0.f;
#pragma unroll
    for (int j = 0; j < J_T; ++j) {
      const float r = x[j] - mb;
      M2 = __builtin_fmaf(r, r, M2);
      a = __builtin_fmaf(x[j], x[j], a);
    }
  } else {
    coord_stats_generic<GT, TABLE>(p, i, S, M2, a);
  }
}

template <class GT, int J_T, int MODE, int BLOCK, bool TABLE, bool GBAR>
__device__ inline void guarded_tile(const StepParams& p, int64_t tile, int tile_coords, double (*red)[BLOCK / 64][NT_NV],
                                    int buf) {
  constexpr int VEC = GT::VEC;
  const int iters = tile_coords / (BLOCK * VEC);
  LaneAcc acc;
  for (int it = 0; it < iters; ++it) {
    const int64_t i0 = tile * (int64_t)tile_coords + ((int64_t)it * BLOCK + threadIdx.x) * VEC;
    float a[VEC], b[VEC], c[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const int64_t i = i0 + e;
      a[e] = b[e] = c[e] = 0.f;
      if (i < p.d) {
        double S;
        float M2, aa;
        coord_stats<GT, TABLE, J_T>(p, i, S, M2, aa);
        const float gb = (float)(S * p.inv_J);
        const float sf = (float)S;
        a[e] = aa;
        b[e] = sf * sf;
        c[e] = M2;
        if constexpr (MODE != MODE_ADAMW) coord_test(p.coord_thr, M2, gb, acc);
        if constexpr (MODE != MODE_STATS) {
          float w = p.w[i], m = p.m[i], v = p.v[i];
          adamw_coord(p, gb, w, m, v);
          p.w[i] = w;
          p.m[i] = m;
          p.v[i] = v;
        }
        if (GBAR && p.gbar) p.gbar[i] = gb;
      }
    }
    if constexpr (MODE != MODE_ADAMW) {
      acc.A += (double)lane_tree<VEC>(a);
      acc.B += (double)lane_tree<VEC>(b);
      acc.C += (double)lane_tree<VEC>(c);
    }
  }
  if constexpr (MODE != MODE_ADAMW) tile_reduce<BLOCK>(acc, red, buf, p.partials, tile);
}

// AdamW on VEC coordinates whose state was loaded as 16-byte vectors, then the 16-byte stores.
template <int VEC>
__device__ inline void adamw_store(const StepParams& p, int64_t i0, const float* gb, const u32x4* sw, const u32x4* sm,
                                   const u32x4* sv) {
  f32x4 ow[VEC / 4], om[VEC / 4], ov[VEC / 4];
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float w = __builtin_bit_cast(float, (uint32_t)sw[q][e]);
      float m = __builtin_bit_cast(float, (uint32_t)sm[q][e]);
      float v = __builtin_bit_cast(float, (uint32_t)sv[q][e]);
      adamw_coord(p, gb[4 * q + e], w, m, v);
      ow[q][e] = w;
      om[q][e] = m;
      ov[q][e] = v;
    }
  }
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q) {
    st16(p.w + i0 + 4 * q, ow[q]);
    st16(p.m + i0 + 4 * q, om[q]);
    st16(p.v + i0 + 4 * q, ov[q]);
  }
}

template <int VEC>
__device__ inline void gbar_store(const StepParams& p, int64_t i0, const float* gb) {
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q) {
    f32x4 og = {gb[4 * q], gb[4 * q + 1], gb[4 * q + 2], gb[4 * q + 3]};
    st16(p.gbar + i0 + 4 * q, og);
  }
}

// ---------------------------------------------------------------------------------------------
// Fast tiles, J <= 16 known at compile time: all J rows of a group of VEC coordinates sit in
// registers; they need 16-byte aligned rows and state and a tile that lies wholly below d.
// The row sum is carried in fp64 so that the mean is correctly rounded even when the rows cancel.
// ---------------------------------------------------------------------------------------------
// One sweep's arithmetic: the means of the lane's VEC coordinates into gb, the sweep's sums into acc.
template <class GT, int J, int MODE>
__device__ inline void sweep_rows(const StepParams& p, const typename GT::raw_t* raw, float* gb, LaneAcc& acc) {
  constexpr int VEC = GT::VEC;
  double s[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) s[e] = (double)GT::val(raw[0], e);
#pragma unroll
  for (int j = 1; j < J; ++j)
#pragma unroll
    for (int e = 0; e < VEC; ++e) s[e] += (double)GT::val(raw[j], e);
#pragma unroll
  for (int e = 0; e < VEC; ++e) gb[e] = (float)(s[e] * p.inv_J);

  if constexpr (MODE != MODE_ADAMW) {
    float a[VEC], c[VEC], b[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) a[e] = c[e] = 0.f;
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float x = GT::val(raw[j], e);
        const float r = x - gb[e];
        c[e] = __builtin_fmaf(r, r, c[e]);
        a[e] = __builtin_fmaf(x, x, a[e]);
      }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const float sf = (float)s[e];
      b[e] = sf * sf;
      coord_test(p.coord_thr, c[e], gb[e], acc);
    }
    acc.A += (double)lane_tree<VEC>(a);
    acc.B += (double)lane_tree<VEC>(b);
    acc.C += (double)lane_tree<VEC>(c);
  }
}

// State update interleaved with the rows: each sweep reads its rows and w, m, v, and writes the state back.
template <class GT, int J, int MODE, int BLOCK, int ITERS, bool TABLE, bool GBAR>
__device__ inline void fast_tile(const StepParams& p, int64_t tile, double (*red)[BLOCK / 64][NT_NV], int buf) {
  constexpr int VEC = GT::VEC;
  constexpr int TILE = BLOCK * VEC * ITERS;
  LaneAcc acc;
  // a statistics-only sweep with few rows has little in flight per lane: overlap sweeps up to about 64 bytes
  constexpr int ROW_BYTES = VEC * GT::ESIZE;
  constexpr int WANT = 64 / (J * ROW_BYTES);
  constexpr int U = (MODE == MODE_STATS && ITERS > 1) ? (WANT >= 4 ? 4 : (WANT >= 2 ? 2 : 1)) : 1;
#pragma unroll U
  for (int it = 0; it < ITERS; ++it) {
    const int64_t i0 = tile * TILE + ((int64_t)it * BLOCK + threadIdx.x) * VEC;
    typename GT::raw_t raw[J];
    u32x4 sw[VEC / 4], sm[VEC / 4], sv[VEC / 4];
#pragma unroll
    for (int j = 0; j < J; ++j) raw[j] = GT::ldraw(row_base<GT, TABLE>(p, j) + i0 * GT::ESIZE);
    if constexpr (MODE != MODE_STATS) {
#pragma unroll
      for (int q = 0; q < VEC / 4; ++q) {
        sw[q] = ld16(p.w + i0 + 4 * q);
        sm[q] = ld16(p.m + i0 + 4 * q);
        sv[q] = ld16(p.v + i0 + 4 * q);
      }
      // Every load of the sweep is issued before any arithmetic: the compiler must neither sink loads below
      // the arithmetic that precedes their use nor hoist arithmetic between them (measured: up to 5 % at 16
      // rows against schedules that issue the state loads after the rows have arrived).  Statistics-only
      // tiles are left free so that consecutive sweeps can overlap.
      __builtin_amdgcn_sched_barrier(0);
    }
    float gb[VEC];
    sweep_rows<GT, J, MODE>(p, raw, gb, acc);
    if constexpr (MODE != MODE_STATS) adamw_store<VEC>(p, i0, gb, sw, sm, sv);
    if (GBAR && p.gbar) gbar_store<VEC>(p, i0, gb);
  }
  if constexpr (MODE != MODE_ADAMW) tile_reduce<BLOCK>(acc, red, buf, p.partials, tile);
  // AdamW-only tiles end with a block barrier like the other modes: the waves of a block then finish together
  // and the next block's waves start together (measured +2 %)
  if constexpr (MODE == MODE_ADAMW) __syncthreads();
}

// The end of a tile whose state update was deferred: the means of all its sweeps wait in LDS (gbs) until every
// row has been read, then w, m, v of all sweeps are read and written in one go.  The memory system charges writes
// sprinkled among reads several times their volume; gathered at the end of a block's life, and with all blocks
// of a launch living at the same time (one generation per launch), they reach it as a dense burst.
template <int MODE, int BLOCK, int ITERS, bool GBAR>
__device__ inline void deferred_update(const StepParams& p, int64_t tile, double (*red)[BLOCK / 64][NT_NV], int buf,
                                       const LaneAcc& acc, const f32x4* gbs) {
  constexpr int VEC = 4;
  constexpr int TILE = BLOCK * VEC * ITERS;
  // the barrier inside keeps the waves of the block together on their way into the write phase
  if constexpr (MODE != MODE_ADAMW)
    tile_reduce<BLOCK>(acc, red, buf, p.partials, tile);
  else
    __syncthreads();
  if (MODE != MODE_STATS || p.gbar) {
#pragma unroll 2
    for (int it = 0; it < ITERS; ++it) {
      const int64_t i0 = tile * TILE + ((int64_t)it * BLOCK + threadIdx.x) * VEC;
      const f32x4 g4 = gbs[it * BLOCK + threadIdx.x];   // this lane's own values: no barrier needed for them
      const float gb[VEC] = {g4[0], g4[1], g4[2], g4[3]};
      if constexpr (MODE != MODE_STATS) {
        u32x4 sw[1], sm[1], sv[1];
        sw[0] = ld16(p.w + i0);
        sm[0] = ld16(p.m + i0);
        sv[0] = ld16(p.v + i0);
        adamw_store<VEC>(p, i0, gb, sw, sm, sv);
      }
      if (GBAR && p.gbar) gbar_store<VEC>(p, i0, gb);
    }
  }
}

// Deferred state update, rows in registers: the sweeps read rows only.
template <class GT, int J, int MODE, int BLOCK, int ITERS, bool TABLE, bool GBAR>
__device__ inline void fast_tile_defer(const StepParams& p, int64_t tile, double (*red)[BLOCK / 64][NT_NV], int buf,
                                       f32x4* gbs) {
  constexpr int VEC = GT::VEC;
  static_assert(VEC == 4, "one 16-byte LDS slot per lane and sweep");
  constexpr int TILE = BLOCK * VEC * ITERS;
  LaneAcc acc;
#pragma unroll NT_DEFER_UNROLL
  for (int it = 0; it < ITERS; ++it) {
    const int64_t i0 = tile * TILE + ((int64_t)it * BLOCK + threadIdx.x) * VEC;
    typename GT::raw_t raw[J];
#pragma unroll
    for (int j = 0; j < J; ++j) raw[j] = GT::ldraw(row_base<GT, TABLE>(p, j) + i0 * GT::ESIZE);
    float gb[VEC];
    sweep_rows<GT, J, MODE>(p, raw, gb, acc);
    gbs[it * BLOCK + threadIdx.x] = f32x4{gb[0], gb[1], gb[2], gb[3]};
  }
  deferred_update<MODE, BLOCK, ITERS, GBAR>(p, tile, red, buf, acc, gbs);
}

// ---------------------------------------------------------------------------------------------
// Fast tile, J > 16: rows are walked NT_MCHUNK at a time.  One pass over a chunk gives its plain sum
// (fp64) and the sum of squares of the values shifted by K, the running mean of the rows before it, hence
// its centred sum of squares without cancellation; see chunk_merge for the bookkeeping.
// ---------------------------------------------------------------------------------------------
template <class GT, bool RT>
__device__ inline void chunk_accumulate(const typename GT::raw_t* raw, int nb, const float* K, double* sb, float* q) {
  constexpr int VEC = GT::VEC;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    sb[e] = 0.0;
    q[e] = 0.f;
  }
#pragma unroll
  for (int j = 0; j < NT_MCHUNK; ++j)
    if (!RT || j < nb) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float x = GT::val(raw[j], e);
        const float r = x - K[e];
        sb[e] += (double)x;
        q[e] = __builtin_fmaf(r, r, q[e]);
      }
    }
}

// The state update (and the gbar store) of a tile is deferred (see deferred_update): with many rows the writes are
// a few per cent of the traffic.
template <class GT, int MODE, int BLOCK, int ITERS, bool TABLE, bool GBAR>
__device__ inline void fast_tile_multi(const StepParams& p, int64_t tile, double (*red)[BLOCK / 64][NT_NV], int buf,
                                       f32x4* gbs) {
  constexpr int VEC = GT::VEC;
  static_assert(VEC == 4, "one 16-byte LDS slot per lane and sweep");
  constexpr int TILE = BLOCK * VEC * ITERS;
  constexpr bool WRITES = (MODE != MODE_STATS) || GBAR;
  const int J = p.J;
  LaneAcc acc;
#pragma unroll 1
  for (int it = 0; it < ITERS; ++it) {
    const int64_t i0 = tile * TILE + ((int64_t)it * BLOCK + threadIdx.x) * VEC;
    const int64_t goff = i0 * GT::ESIZE;
    double S[VEC], sb[VEC];
    float M2[VEC], a[VEC], K[VEC], q[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) a[e] = 0.f;
    typename GT::raw_t raw[NT_MCHUNK];
    // first chunk (J > NT_JCHUNK >= NT_MCHUNK - 1 here, so it is full), shifted by the first row
#pragma unroll
    for (int j = 0; j < NT_MCHUNK; ++j) raw[j] = GT::ldraw(row_base<GT, TABLE>(p, j) + goff);
#pragma unroll
    for (int e = 0; e < VEC; ++e) K[e] = GT::val(raw[0], e);
    chunk_accumulate<GT, false>(raw, NT_MCHUNK, K, sb, q);
#pragma unroll
    for (int e = 0; e < VEC; ++e) K[e] = chunk_merge(true, 0, NT_MCHUNK, K[e], sb[e], q[e], S[e], M2[e], a[e]);
    int j0 = NT_MCHUNK;
#pragma unroll 1
    for (; j0 + NT_MCHUNK <= J; j0 += NT_MCHUNK) {
#pragma unroll
      for (int j = 0; j < NT_MCHUNK; ++j) raw[j] = GT::ldraw(row_base<GT, TABLE>(p, j0 + j) + goff);
      chunk_accumulate<GT, false>(raw, NT_MCHUNK, K, sb, q);
#pragma unroll
      for (int e = 0; e < VEC; ++e) K[e] = chunk_merge(false, j0, NT_MCHUNK, K[e], sb[e], q[e], S[e], M2[e], a[e]);
    }
    if (j0 < J) {
      const int nb = J - j0;
#pragma unroll
      for (int j = 0; j < NT_MCHUNK; ++j)
        if (j < nb) raw[j] = GT::ldraw(row_base<GT, TABLE>(p, j0 + j) + goff);
      chunk_accumulate<GT, true>(raw, nb, K, sb, q);
#pragma unroll
      for (int e = 0; e < VEC; ++e) K[e] = chunk_merge(false, j0, nb, K[e], sb[e], q[e], S[e], M2[e], a[e]);
    }
    float gb[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) gb[e] = (float)(S[e] * p.inv_J);

    if constexpr (MODE != MODE_ADAMW) {
      float b[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float sf = (float)S[e];
        b[e] = sf * sf;
        coord_test(p.coord_thr, M2[e], gb[e], acc);
      }
      acc.A += (double)lane_tree<VEC>(a);
      acc.B += (double)lane_tree<VEC>(b);
      acc.C += (double)lane_tree<VEC>(M2);
    }
    if constexpr (WRITES) gbs[it * BLOCK + threadIdx.x] = f32x4{gb[0], gb[1], gb[2], gb[3]};
  }
  if constexpr (WRITES)
    deferred_update<MODE, BLOCK, ITERS, GBAR>(p, tile, red, buf, acc, gbs);
  else
    tile_reduce<BLOCK>(acc, red, buf, p.partials, tile);
}

// ---------------------------------------------------------------------------------------------
// Kernels.  A launch covers the slots slot0 .. slot1-1 of the ntiles tile slots; block b takes slots slot0 + b,
// slot0 + b + gridDim.x, ...; tiles below nfull are whole and aligned (fast path), the others go through the
// guarded path.  When the vector ends in a ragged tile, it has slot 0, so that the slow tile overlaps with
// everything else.
// J_T = 0 selects the J > 16 row-walking variant.
// ---------------------------------------------------------------------------------------------
// GBAR = false compiles the gbar store out (statistics-only launch class, so that sweeps can overlap).
// DEFER_T: up to 16 rows with the state update deferred to the end of the tile (always so beyond 16 rows).
template <class GT, int J_T, int MODE, int BLOCK, int ITERS, bool TABLE, bool GBAR, bool DEFER_T = false>
__global__ __launch_bounds__(BLOCK) void k_step(StepParams p, int64_t nfull, int64_t ntiles, int64_t slot0, int64_t slot1,
                                                 WsControl* ctl) {
  constexpr int TILE = BLOCK * GT::VEC * ITERS;
  static_assert(NT_TILE_MAX % TILE == 0, "tile sizes must divide NT_TILE_MAX");
  __shared__ double red[2][BLOCK / 64][NT_NV];
  // the means of a tile's sweeps wait here for the deferred state update (see deferred_update)
  constexpr bool DEFER = (J_T == 0 || DEFER_T) && ((MODE != MODE_STATS) || GBAR);
  static_assert(!DEFER_T || DEFER, "a deferred update needs something to write");
  __shared__ f32x4 gbs[DEFER ? ITERS * BLOCK + NT_LDS_PAD_LARGE / 16 : 1];
  int buf = 0;
  if constexpr (TABLE) {
    // the host cannot see the row pointers: k_rows_aligned has looked at them and left its verdict here
    if (!ctl->rows_aligned) nfull = 0;
  }
  const int64_t nrest = ntiles - nfull;  // guarded tiles (0 or 1 on the aligned path)
  for (int64_t t = slot0 + blockIdx.x; t < slot1; t += gridDim.x) {
    // rotate: the first nrest slots are the guarded tiles nfull.., then the fast tiles 0..nfull-1
    const int64_t tile = (t < nrest) ? nfull + t : t - nrest;
    if (tile < nfull) {
      if constexpr (J_T > 0 && DEFER_T)
        fast_tile_defer<GT, J_T, MODE, BLOCK, ITERS, TABLE, GBAR>(p, tile, red, buf, gbs);
      else if constexpr (J_T > 0)
        fast_tile<GT, J_T, MODE, BLOCK, ITERS, TABLE, GBAR>(p, tile, red, buf);
      else
        fast_tile_multi<GT, MODE, BLOCK, ITERS, TABLE, GBAR>(p, tile, red, buf, gbs);
    } else {
      guarded_tile<GT, J_T, MODE, BLOCK, TABLE, GBAR>(p, tile, TILE, red, buf);
    }
    buf ^= 1;
  }
}

// Pointer-table calls: are all J row pointers 16-byte aligned?  One small block, once per call, so that the
// blocks of k_step need not walk the table themselves.
__global__ __launch_bounds__(256) void k_rows_aligned(const void* const* rows, int J, WsControl* ctl) {
  __shared__ unsigned int bits;
  if (threadIdx.x == 0) bits = 0u;
  __syncthreads();
  unsigned int mine = 0u;
  for (int j = threadIdx.x; j < J; j += 256) mine |= (unsigned int)((uintptr_t)rows[j] & 15u);
  if (mine) atomicOr(&bits, mine);
  __syncthreads();
  if (threadIdx.x == 0) ctl->rows_aligned = bits ? 0u : 1u;
}

// ---------------------------------------------------------------------------------------------
// Double-double helpers (error-free transformations; the file is compiled with contraction off).
// ---------------------------------------------------------------------------------------------
struct dd {
  double hi, lo;
};
__host__ __device__ inline dd dd_add(dd x, dd y) {
  double s = x.hi + y.hi;
  double bb = s - x.hi;
  double e = (x.hi - (s - bb)) + (y.hi - bb);
  e += x.lo + y.lo;
  dd r;
  r.hi = s + e;
  r.lo = e - (r.hi - s);
  return r;
}

struct DecideParams {
  int64_t J;
  double eta;
  double max_norm;  // gradient-norm bound of the clipped variant, <= 0: none
  int64_t b_k, b_max, round_to;
  int32_t ddof;
  uint32_t flags;
};

// Record of the step whose tile partials sit in a workspace, kept in its first NT_WS_HEADER doubles so that
// normtest_layer_stats can regroup them per layer and can tell when they belong to another call.
struct WsHeader {
  int64_t magic;
  int64_t tile_coords, ntiles, ngroups;  // ngroups > 0: double-double group partials follow the tile partials
  int64_t d, J;
  int32_t gdtype, has_stats;
  double coord_thr;                      // threshold factor of the coordinate-wise count, negative if off
  DecideParams q;
};
static_assert(sizeof(WsHeader) <= NT_WS_HEADER * sizeof(double), "workspace header too small");

// Global-norm clipping factor (training specifications of Sec. 5; usual convention with the 1e-6 guard).
__host__ __device__ inline double clip_coef(double gbar_sq, double max_norm) {
  if (!(max_norm > 0.0)) return 1.0;
  const double c = max_norm / (sqrt(gbar_sq) + 1e-6);
  return c < 1.0 ? c : 1.0;
}

// From the sums in r->A, r->B, r->C to ||gbar||^2, ||Var||_1, T, pass and next_b (Alg. 1: test
// statistic, strict comparison with b_k, ceiling, rounding through micro-batch, minibatch and
// global batch, which composes to the next multiple of J*M; Sec. 5: cap at the maximum batch size).
__host__ __device__ inline void decide(const DecideParams& q, nt_result* r) {
  const double Jd = (double)q.J;
  const int64_t cap = (q.b_max > q.b_k) ? q.b_max : q.b_k;
  r->pass = 1;
  r->next_b = q.b_k;
  r->gbar_sq = r->B / (Jd * Jd);
  r->var_l1 = r->C / (double)(q.J - q.ddof);
  r->clip_coef = clip_coef(r->gbar_sq, q.max_norm);
  if (!(__builtin_isfinite(r->A) && __builtin_isfinite(r->B) && __builtin_isfinite(r->C))) {
    r->status |= NT_STATUS_NONFINITE;
    r->T = __builtin_nan("");
    return;
  }
  if (r->gbar_sq == 0.0) {
    r->status |= NT_STATUS_ZERO_GRAD_NORM;
    if (r->C == 0.0) {
      r->T = __builtin_nan("");
    } else {
      r->T = __builtin_inf();
      r->pass = 0;
      r->next_b = cap;
    }
    return;
  }
  const double T = r->var_l1 / (q.eta * q.eta * r->gbar_sq);
  r->T = T;
  if (T > (double)q.b_k) {
    r->pass = 0;
    if (!(T < 4611686018427387904.0)) {
      r->status |= NT_STATUS_T_SATURATED;
      r->next_b = cap;
      return;
    }
    // t < 2^62 and round_to <= 2^31 (validated), so the next multiple fits an int64
    const int64_t t = (int64_t)ceil(T);
    int64_t nb = (t / q.round_to + (t % q.round_to != 0)) * q.round_to;
    if (q.b_max > 0 && nb > q.b_max) {
      nb = q.b_max;
      r->status |= NT_STATUS_CLAMPED;
    }
    r->next_b = nb < q.b_k ? q.b_k : nb;
  }
}

__device__ inline dd dd_wave_sum(dd x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    dd y;
    y.hi = __shfl_xor(x.hi, off, 64);
    y.lo = __shfl_xor(x.lo, off, 64);
    // both partners must form the same sum: order the operands by lane
    const bool low = (threadIdx.x & off) == 0;
    x = low ? dd_add(x, y) : dd_add(y, x);
  }
  return x;
}
__device__ inline double wave_max(double x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = __builtin_fmax(x, __shfl_xor(x, off, 64));
  return x;
}

// Running totals of partial records: the NT_NSUM sums in double-double and the largest ratio.
struct Totals {
  dd s[NT_NSUM];
  double mx;
};
__device__ inline void totals_clear(Totals& t) {
#pragma unroll
  for (int k = 0; k < NT_NSUM; ++k) t.s[k] = {0.0, 0.0};
  t.mx = 0.0;
}

// Adds this thread's share (entries threadIdx.x, threadIdx.x + THREADS, ...) of n records into acc.
// packed = false: tile partials {A, B, C, n_fail, r_max}; packed = true: group partials
// {A, A_lo, B, B_lo, C, C_lo, n, n_lo, r_max, unused}.
template <int THREADS>
__device__ inline void totals_accumulate(const double* in, int64_t n, bool packed, Totals& acc) {
  for (int64_t t = threadIdx.x; t < n; t += THREADS) {
    const double* rec = in + (packed ? 2 * NT_NV : NT_NV) * t;
#pragma unroll
    for (int k = 0; k < NT_NSUM; ++k) {
      dd x;
      if (!packed) {
        x.hi = rec[k];
        x.lo = 0.0;
      } else {
        x.hi = rec[2 * k];
        x.lo = rec[2 * k + 1];
      }
      acc.s[k] = dd_add(acc.s[k], x);
    }
    acc.mx = __builtin_fmax(acc.mx, rec[packed ? 2 * NT_NSUM : NT_NSUM]);
  }
}

// Block total of the threads' accumulators; all threads take part, thread 0 returns the totals.
template <int THREADS>
__device__ inline void block_totals_finish(Totals& acc, double (*sh)[2 * NT_NV], Totals& tot) {
#pragma unroll
  for (int k = 0; k < NT_NSUM; ++k) acc.s[k] = dd_wave_sum(acc.s[k]);
  acc.mx = wave_max(acc.mx);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < NT_NSUM; ++k) {
      sh[wave][2 * k] = acc.s[k].hi;
      sh[wave][2 * k + 1] = acc.s[k].lo;
    }
    sh[wave][2 * NT_NSUM] = acc.mx;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 0; k < NT_NSUM; ++k) {
      tot.s[k].hi = sh[0][2 * k];
      tot.s[k].lo = sh[0][2 * k + 1];
      for (int wv = 1; wv < THREADS / 64; ++wv) {
        dd x = {sh[wv][2 * k], sh[wv][2 * k + 1]};
        tot.s[k] = dd_add(tot.s[k], x);
      }
    }
    tot.mx = sh[0][2 * NT_NSUM];
    for (int wv = 1; wv < THREADS / 64; ++wv) tot.mx = __builtin_fmax(tot.mx, sh[wv][2 * NT_NSUM]);
  }
}

// Sum of n records (layouts as in totals_accumulate); thread 0 returns the totals.
template <int THREADS>
__device__ inline void block_totals(const double* in, int64_t n, bool packed, double (*sh)[2 * NT_NV], Totals& tot) {
  Totals acc;
  totals_clear(acc);
  totals_accumulate<THREADS>(in, n, packed, acc);
  block_totals_finish<THREADS>(acc, sh, tot);
}

// First stage for long vectors: block g adds tile partials [g*NT_GROUP_TILES, ...) into one double-double
// group partial.  The two stages are separate launches on purpose: the eight XCDs of this GPU do not share an
// L2, so a block that waits for the other blocks' partials inside one kernel (a ticket taken after a device-wide
// release, then a device-wide acquire) pays a write-back and an invalidation of its L2 on every block; measured,
// that made the single launch slower (26 us at 15 groups) than these two small kernels (8 + 5 us), whose
// visibility comes with the kernel boundary.
__global__ __launch_bounds__(NT_GROUP_THREADS) void k_reduce_groups(const double* tiles, int64_t ntiles, double* groups) {
  __shared__ double sh[NT_GROUP_THREADS / 64][2 * NT_NV];
  const int64_t t0 = (int64_t)blockIdx.x * NT_GROUP_TILES;
  const int64_t n = (ntiles - t0 < NT_GROUP_TILES) ? (ntiles - t0) : NT_GROUP_TILES;
  Totals tot;
  block_totals<NT_GROUP_THREADS>(tiles + NT_NV * t0, n, false, sh, tot);
  if (threadIdx.x == 0) {
    double* rec = groups + 2 * NT_NV * (int64_t)blockIdx.x;
#pragma unroll
    for (int k = 0; k < NT_NSUM; ++k) {
      rec[2 * k] = tot.s[k].hi;
      rec[2 * k + 1] = tot.s[k].lo;
    }
    rec[2 * NT_NSUM] = tot.mx;
    rec[2 * NT_NSUM + 1] = 0.0;
  }
}

// One block: partials (tile or group) -> A, B, C in double-double, then the decision.  THREADS: 1024, or 256 for
// up to NT_FIN_SMALL records (short vectors, where this kernel's latency is a large part of the step).
template <int THREADS>
__global__ __launch_bounds__(THREADS) void k_finalize(const double* in, int64_t n, bool packed, DecideParams q,
                                                      nt_result* out, WsHeader hdr, WsHeader* hdr_out) {
  __shared__ double sh[THREADS / 64][2 * NT_NV];
  const bool stats = (q.flags & NT_DO_STATS) != 0;
  Totals tot;
  totals_clear(tot);
  if (stats) block_totals<THREADS>(in, n, packed, sh, tot);
  if (threadIdx.x != 0) return;
  *hdr_out = hdr;
  nt_result r;
  r.status = 0;
  const bool coord = stats && (q.flags & NT_COORD_TEST);
  r.coord_fail = coord ? (int64_t)tot.s[3].hi : -1;
  r.coord_max_ratio = coord ? tot.mx : -1.0;
  const double nan = __builtin_nan("");
  if (!stats) {
    r.A = r.B = r.C = r.A_lo = r.B_lo = r.C_lo = nan;
    r.gbar_sq = r.var_l1 = r.T = nan;
    r.clip_coef = 1.0;
    r.pass = 1;
    r.next_b = q.b_k;
    r.status = NT_STATUS_NO_STATS;
  } else {
    r.A = tot.s[0].hi; r.A_lo = tot.s[0].lo;
    r.B = tot.s[1].hi; r.B_lo = tot.s[1].lo;
    r.C = tot.s[2].hi; r.C_lo = tot.s[2].lo;
    if (q.flags & NT_PARTIAL) {
      r.gbar_sq = r.var_l1 = r.T = nan;
      r.clip_coef = 1.0;
      r.pass = 1;
      r.next_b = q.b_k;
      r.status = NT_STATUS_PARTIAL_ONLY;
      if (!(__builtin_isfinite(r.A) && __builtin_isfinite(r.B) && __builtin_isfinite(r.C)))
        r.status |= NT_STATUS_NONFINITE;
    } else {
      decide(q, &r);
    }
  }
  *out = r;
}

// Sums over the coordinates [plo, phi) taken one by one, NT_LAYER_THREADS apart per thread.  J_T > 0: row
// count known at compile time; J_T = 0: any J.
template <class GT, bool TABLE, int J_T>
__device__ inline void piece_sums(const StepParams& p, int64_t plo, int64_t phi, LaneAcc& acc) {
#pragma unroll 2
  for (int64_t i = plo + threadIdx.x; i < phi; i += NT_LAYER_THREADS) {
    double S;
    float M2, aa;
    coord_stats<GT, TABLE, J_T>(p, i, S, M2, aa);
    const float gb = (float)(S * p.inv_J);
    const float sf = (float)S;
    acc.A += (double)aa;
    acc.B += (double)(sf * sf);
    acc.C += (double)M2;
    coord_test(p.coord_thr, M2, gb, acc);
  }
}

// Per-layer statistics from what a step left behind.  Layer l owns coordinates offsets[l] .. offsets[l+1]-1.
// Block l adds the partials of the tiles that lie wholly inside the layer (through the group partials
// where a whole group does) and recomputes, from the gradient rows, the at most two pieces at the layer's
// ends that cover only part of a tile; then the layer's own statistic (Alg. 1's T on the layer's
// coordinates) is formed.  Offsets are clamped into [0, d], so every access stays in bounds whatever
// the table holds; a clamped or descending pair is reported in the layer's status.
template <class GT, bool TABLE>
__global__ __launch_bounds__(NT_LAYER_THREADS) void k_layer_stats(StepParams p, const int64_t* offsets,
                                                                  const double* ws, nt_layer_stats* out) {
  __shared__ double sh[NT_LAYER_THREADS / 64][2 * NT_NV];
  const WsHeader h = *(const WsHeader*)ws;
  const int l = blockIdx.x;
  const double nan = __builtin_nan("");
  const bool usable = h.magic == NT_WS_MAGIC && h.has_stats && h.d == p.d && h.J == (int64_t)p.J &&
                      h.gdtype == (GT::ESIZE == 4 ? (int32_t)NT_F32 : (int32_t)NT_BF16) && h.tile_coords > 0;
  int64_t lo = offsets[l], hi = offsets[l + 1];
  uint32_t status = 0;
  if (lo < 0 || lo > p.d || hi < lo || hi > p.d) status |= NT_STATUS_BAD_RANGE;
  lo = lo < 0 ? 0 : (lo > p.d ? p.d : lo);
  hi = hi < lo ? lo : (hi > p.d ? p.d : hi);
  if (!usable) {
    if (threadIdx.x == 0) {
      nt_layer_stats r;
      r.A = r.B = r.C = r.gbar_sq = r.var_l1 = r.T = nan;
      r.coord_max_ratio = -1.0;
      r.n = hi - lo;
      r.coord_fail = -1;
      r.pass = 1;
      r.status = status | NT_STATUS_NO_STATS;
      out[l] = r;
    }
    return;
  }
  p.coord_thr = (float)h.coord_thr;
  const int64_t tc = h.tile_coords;
  const int64_t first = (lo + tc - 1) / tc;                      // first tile that starts at or after lo
  const int64_t head_end = first * tc < hi ? first * tc : hi;    // head piece [lo, head_end)
  int64_t last = first, tail_lo = hi;                            // whole tiles [first, last), tail piece [tail_lo, hi)
  if (head_end < hi) {
    last = hi / tc;
    tail_lo = last * tc;
  }
  LaneAcc piece;
  for (int part = 0; part < 2; ++part) {
    const int64_t plo = part ? tail_lo : lo, phi = part ? hi : head_end;
    if (plo >= phi) continue;
#define NT_CASE(JJ) \
  case JJ:          \
    piece_sums<GT, TABLE, JJ>(p, plo, phi, piece); \
    break;
    switch (p.J) {
      NT_CASE(2) NT_CASE(3) NT_CASE(4) NT_CASE(5) NT_CASE(6) NT_CASE(7) NT_CASE(8) NT_CASE(9)
      NT_CASE(10) NT_CASE(11) NT_CASE(12) NT_CASE(13) NT_CASE(14) NT_CASE(15) NT_CASE(16)
      default: piece_sums<GT, TABLE, 0>(p, plo, phi, piece);
    }
#undef NT_CASE
  }
  Totals acc;
  acc.s[0] = {piece.A, 0.0};
  acc.s[1] = {piece.B, 0.0};
  acc.s[2] = {piece.C, 0.0};
  acc.s[3] = {(double)piece.nfail, 0.0};
  acc.mx = (double)piece.rmax;
  const double* tiles = ws + NT_WS_HEADER;
  const double* groups = tiles + NT_NV * h.ntiles;
  const int64_t g0 = (first + NT_GROUP_TILES - 1) / NT_GROUP_TILES, g1 = last / NT_GROUP_TILES;
  if (h.ngroups > 0 && g0 < g1) {
    totals_accumulate<NT_LAYER_THREADS>(tiles + NT_NV * first, g0 * NT_GROUP_TILES - first, false, acc);
    totals_accumulate<NT_LAYER_THREADS>(groups + 2 * NT_NV * g0, g1 - g0, true, acc);
    totals_accumulate<NT_LAYER_THREADS>(tiles + NT_NV * g1 * NT_GROUP_TILES, last - g1 * NT_GROUP_TILES, false, acc);
  } else {
    totals_accumulate<NT_LAYER_THREADS>(tiles + NT_NV * first, last - first, false, acc);
  }
  Totals tot;
  block_totals_finish<NT_LAYER_THREADS>(acc, sh, tot);
  if (threadIdx.x != 0) return;
  nt_result t;
  t.A = tot.s[0].hi;
  t.B = tot.s[1].hi;
  t.C = tot.s[2].hi;
  t.status = 0;
  DecideParams q = h.q;
  q.b_max = 0;
  q.round_to = 1;
  q.max_norm = 0.0;
  decide(q, &t);
  nt_layer_stats r;
  r.A = t.A;
  r.B = t.B;
  r.C = t.C;
  r.gbar_sq = t.gbar_sq;
  r.var_l1 = t.var_l1;
  r.T = t.T;
  r.coord_max_ratio = (h.coord_thr >= 0.0) ? tot.mx : -1.0;
  r.n = hi - lo;
  r.coord_fail = (h.coord_thr >= 0.0) ? (int64_t)tot.s[3].hi : -1;
  r.pass = t.pass;
  r.status = status | (t.status & (NT_STATUS_NONFINITE | NT_STATUS_ZERO_GRAD_NORM | NT_STATUS_T_SATURATED));
  out[l] = r;
}

// Phase 2 of the clipped variant: AdamW on scale * gbar, gbar read from memory.  One sweep per block,
// 4 coordinates per lane; lanes whose 4 coordinates are not all below d, or unaligned buffers, go
// element by element.
__global__ __launch_bounds__(NT_AUX_BLOCK) void k_adamw_gbar(StepParams p, const float* gbar, float grad_scale,
                                                         const nt_result* res, int aligned, int64_t block0) {
  float scale = grad_scale;
  if (res) scale *= (float)res->clip_coef;
  const int64_t i0 = ((block0 + blockIdx.x) * NT_AUX_BLOCK + threadIdx.x) * NT_VEC;
  if (i0 >= p.d) return;
  if (aligned && i0 + NT_VEC <= p.d) {
    const u32x4 sg = ld16(gbar + i0);
    u32x4 sw = ld16(p.w + i0), sm = ld16(p.m + i0), sv = ld16(p.v + i0);
    float gb[NT_VEC];
#pragma unroll
    for (int e = 0; e < NT_VEC; ++e) gb[e] = scale * __builtin_bit_cast(float, (uint32_t)sg[e]);
    adamw_store<NT_VEC>(p, i0, gb, &sw, &sm, &sv);
  } else {
    for (int64_t i = i0; i < i0 + NT_VEC && i < p.d; ++i) {
      float w = p.w[i], m = p.m[i], v = p.v[i];
      adamw_coord(p, scale * gbar[i], w, m, v);
      p.w[i] = w;
      p.m[i] = m;
      p.v[i] = v;
    }
  }
}

__global__ __launch_bounds__(NT_AUX_BLOCK) void k_copy16(f32x4* dst, const u32x4* src, int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * NT_AUX_BLOCK + threadIdx.x; i < n16; i += (int64_t)gridDim.x * NT_AUX_BLOCK) {
    const u32x4 x = ld16(src + i);
    st16(dst + i, __builtin_bit_cast(f32x4, x));
  }
}


// ---------------------------------------------------------------------------------------------
// Yardstick: R8 row-like read streams (8 bytes per lane, like four bfloat16 values of a gradient row), R16 read
// streams and W written streams (16 bytes per lane, like four fp32 values of w, m or v; RMW: read first, as an
// in-place update does), all walked in step by one block per 4096 coordinates with the step kernel's load and
// store instructions and no arithmetic beyond an exclusive-or that keeps every load alive.  It shows what
// the memory system gives for a mix of streams, independent of the step's arithmetic.
// ---------------------------------------------------------------------------------------------
#define NT_CALIB_MAX_R8 16
#define NT_CALIB_MAX_R16 12
#define NT_CALIB_MAX_W 4
struct CalibStreams {
  const char* r8[NT_CALIB_MAX_R8];
  const char* r16[NT_CALIB_MAX_R16];
  char* w[NT_CALIB_MAX_W];
  uint32_t* sink;   // spare word behind the streams; read-only mixes store to it when a load hits one magic value
};

template <int R8, int R16, int W, bool RMW>
__global__ __launch_bounds__(NT_AUX_BLOCK) void k_calib_streams(CalibStreams s, int64_t group0, int64_t group1) {
  for (int64_t i = group0 + (int64_t)blockIdx.x * NT_AUX_BLOCK + threadIdx.x; i < group1; i += (int64_t)gridDim.x * NT_AUX_BLOCK) {
    u32x2 a[R8 > 0 ? R8 : 1];
    u32x4 b[R16 > 0 ? R16 : 1];
    u32x4 c[W > 0 ? W : 1];
#pragma unroll
    for (int k = 0; k < R8; ++k) a[k] = ld_vec<true, u32x2>(s.r8[k] + 8 * i);
#pragma unroll
    for (int k = 0; k < R16; ++k) b[k] = ld16(s.r16[k] + 16 * i);
    if constexpr (RMW) {
#pragma unroll
      for (int k = 0; k < W; ++k) c[k] = ld16(s.w[k] + 16 * i);
    }
    uint32_t acc = 0;
#pragma unroll
    for (int k = 0; k < R8; ++k) acc ^= a[k][0] ^ a[k][1];
#pragma unroll
    for (int k = 0; k < R16; ++k) acc ^= b[k][0] ^ b[k][1] ^ b[k][2] ^ b[k][3];
#pragma unroll
    for (int k = 0; k < W; ++k) {
      u32x4 o = {acc, acc + 1u, acc + 2u, acc + 3u};
      if constexpr (RMW) o ^= c[k];
      st16(s.w[k] + 16 * i, __builtin_bit_cast(f32x4, o));
    }
    if constexpr (W == 0) {
      if (acc == 0x9e3779b9u) *s.sink = acc;   // data-dependent, so the loads cannot be dropped
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
inline int hip_code(hipError_t e) { return e == hipSuccess ? NT_OK : NT_ERR_HIP_BASE - (int)e; }

int cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED);
  if (n <= 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    __atomic_store_n(&cached[dev], n, __ATOMIC_RELAXED);
  }
  return n;
}

// Launch class of a call: block size and sweeps per tile.  Every tile is block * NT_VEC * sweeps
// coordinates and divides NT_TILE_MAX.
struct TileCfg {
  int block, iters;
  int64_t coords() const { return (int64_t)block * NT_VEC * iters; }
};
constexpr int defer_row_bytes(int mode) { return mode == MODE_ADAMW ? NT_DEFER_ROW_BYTES_ADAMW : NT_DEFER_ROW_BYTES; }
// Which launch class a call takes beside its row count, dtype and mode: CLS_LONG, the classes for long vectors
// (large tiles, state update deferred, one generation of blocks per launch); CLS_SHORT_STATS, read-only statistics
// of up to 16 rows over a short vector; else CLS_BASE.  esize: bytes per gradient element; d_whole: length of the
// vector the call is a part of (its own d unless the caller said otherwise), so that the parts of a vector and the
// vector itself are cut into the same tiles.
enum { CLS_BASE = 0, CLS_LONG = 1, CLS_SHORT_STATS = 2 };
inline int launch_class(int64_t J, int esize, int mode, bool gbar, int64_t d_whole) {
  if (mode == MODE_STATS && !gbar) return (J <= NT_JCHUNK && d_whole < NT_STATS_SHORT_COORDS) ? CLS_SHORT_STATS : CLS_BASE;
  if (J > NT_JCHUNK) return d_whole >= (J <= 32 ? NT_MANY_LONG_COORDS_32 : NT_MANY_LONG_COORDS) ? CLS_LONG : CLS_BASE;
  return (J * esize >= defer_row_bytes(mode) && d_whole >= NT_DEFER_COORDS) ? CLS_LONG : CLS_BASE;
}
inline TileCfg tile_cfg(int64_t J, int esize, int mode, bool gbar, int64_t d_whole) {
  const int cls = launch_class(J, esize, mode, gbar, d_whole);
  if (J > NT_JCHUNK) {
    if (mode == MODE_STATS && !gbar) return {NT_BLOCK_LARGE_STATS, NT_ITERS_LARGE_STATS};
    return cls == CLS_LONG ? TileCfg{NT_BLOCK_LARGE, NT_ITERS_LARGE} : TileCfg{NT_BLOCK_MANY_SHORT, NT_ITERS_MANY_SHORT};
  }
  if (cls == CLS_LONG) return {NT_BLOCK_DEFER, NT_ITERS_DEFER};
  if (mode == MODE_STATS && (gbar || cls == CLS_SHORT_STATS)) return {NT_BLOCK_STATS_GBAR, NT_ITERS_STATS_GBAR};
  if (mode == MODE_STATS) return {NT_BLOCK_STATS, NT_ITERS_STATS};
  if (mode == MODE_ADAMW) return {NT_BLOCK_ADAMW, NT_ITERS_ADAMW};
  return {NT_BLOCK, NT_ITERS};
}
static_assert(NT_BLOCK_FEW * NT_ITERS_FEW == NT_BLOCK_LARGE * NT_ITERS_LARGE, "both many-row shapes own the same tile");
static_assert(NT_BLOCK_DEFER * NT_ITERS_DEFER >= NT_BLOCK * NT_ITERS &&
                  NT_BLOCK_DEFER * NT_ITERS_DEFER >= NT_BLOCK_ADAMW * NT_ITERS_ADAMW &&
                  NT_BLOCK_DEFER * NT_ITERS_DEFER >= NT_BLOCK_STATS_GBAR * NT_ITERS_STATS_GBAR,
              "the deferred class never has more tiles than the class it replaces: the workspace is sized by the latter");
// tile slots per launch of the step kernel for the same classes (at least one, at most all)
inline int64_t launch_tiles(int64_t J, int esize, int mode, bool gbar, int cls, int64_t ntiles) {
  int64_t coords;
  if (J > NT_JCHUNK || cls != CLS_BASE)
    return ntiles;   // one launch, or generations of blocks: launch_step_shape knows the kernel's occupancy
  else if (mode == MODE_STATS)
    coords = gbar ? NT_CHUNK_STATS_GBAR : NT_CHUNK_STATS;
  else
    coords = (mode == MODE_ADAMW) ? NT_CHUNK_ADAMW : NT_CHUNK_FULL;
  const int64_t n = coords / tile_cfg(J, esize, mode, gbar, 0).coords();
  return (n < 1 || n > ntiles) ? ntiles : n;
}
// smallest tile any mode and gradient type uses for this J: sizes the workspace
inline int64_t min_tile_coords(int64_t J) {
  int64_t best = tile_cfg(J, 2, MODE_FULL, false, 0).coords();
  const int modes[3] = {MODE_FULL, MODE_STATS, MODE_ADAMW};
  for (int m : modes)
    for (int g = 0; g < 2; ++g)
      for (int esize = 2; esize <= 4; esize += 2) {
        for (int64_t d_whole = 0; d_whole <= NT_DEFER_COORDS; d_whole += NT_DEFER_COORDS) {   // shortest and longest
          const int64_t c = tile_cfg(J, esize, m, g != 0, d_whole).coords();
          if (c < best) best = c;
        }
      }
  return best;
}

bool hyper_ok(const nt_hyper* h, int64_t J) {
  if (!h) return false;
  const uint32_t known = NT_DO_STATS | NT_DO_ADAMW | NT_PARTIAL | NT_WRITE_GBAR | NT_COORD_TEST | NT_ONE_PASS;
  if (h->flags & ~known) return false;
  if (!(h->flags & (NT_DO_STATS | NT_DO_ADAMW))) return false;
  if ((h->flags & (NT_PARTIAL | NT_COORD_TEST)) && !(h->flags & NT_DO_STATS)) return false;
  if (!(h->eta > 0.0) || !std::isfinite(h->eta)) return false;
  if (h->b_k < 1 || h->b_max < 0 || h->round_to < 1 || h->round_to > NT_ROUND_TO_MAX) return false;
  if (h->ddof != 0 && h->ddof != 1) return false;
  if (J - h->ddof < 1) return false;
  if (h->flags & NT_DO_ADAMW) {
    if (h->step < 1) return false;
    if (!(h->lr >= 0.0) || !std::isfinite(h->lr)) return false;
    if (!(h->beta1 >= 0.0 && h->beta1 < 1.0) || !(h->beta2 >= 0.0 && h->beta2 < 1.0)) return false;
    if (!(h->eps >= 0.0) || !std::isfinite(h->eps)) return false;
    if (!(h->weight_decay >= 0.0) || !std::isfinite(h->weight_decay)) return false;
  }
  return true;
}

// How many blocks of a kernel with a deferred update a CU holds at a time (the runtime's occupancy query, asked
// once per device and kernel; 4 if it cannot be had).
template <auto KERNEL, int BS>
int blocks_per_cu() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 4;
  int n = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED);
  if (n <= 0) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, KERNEL, BS, 0) != hipSuccess || n < 1) {
      (void)hipGetLastError();
      n = 4;
    }
    __atomic_store_n(&cached[dev], n, __ATOMIC_RELAXED);
  }
  return n;
}

template <class GT, int MODE, bool TABLE, int BS, int IS, bool GBAR>
hipError_t launch_step_shape(const StepParams& p, int cls, int64_t nfull, int64_t ntiles, WsControl* ctl,
                             int max_grid, hipStream_t st) {
  const bool long_class = cls == CLS_LONG;
  constexpr bool WRITES = (MODE != MODE_STATS) || GBAR;
  const bool gbar = MODE == MODE_STATS && p.gbar != nullptr;
  int64_t per_launch = launch_tiles(p.J, GT::ESIZE, MODE, gbar, cls, ntiles);
  if (WRITES && long_class) {
    // blocks that write per coordinate do so at the end of their lives: a launch holds whole generations of blocks
    // (as many as the chip runs at a time), so that all of them read together and write together
    int per_cu = 4;
    if constexpr (WRITES) {
#define NT_OCC(JJ)                                                                                          \
  case JJ:                                                                                                  \
    if constexpr (JJ * GT::ESIZE >= defer_row_bytes(MODE))                                                  \
      per_cu = blocks_per_cu<k_step<GT, JJ, MODE, NT_BLOCK_DEFER, NT_ITERS_DEFER, TABLE, true, true>,       \
                             NT_BLOCK_DEFER>();                                                             \
    break;
      switch (p.J) {
        NT_OCC(2) NT_OCC(3) NT_OCC(4) NT_OCC(5) NT_OCC(6) NT_OCC(7) NT_OCC(8) NT_OCC(9)
        NT_OCC(10) NT_OCC(11) NT_OCC(12) NT_OCC(13) NT_OCC(14) NT_OCC(15) NT_OCC(16)
        default:
          per_cu = (p.J <= NT_FEW_ROWS)
                       ? blocks_per_cu<k_step<GT, 0, MODE, NT_BLOCK_FEW, NT_ITERS_FEW, TABLE, true>, NT_BLOCK_FEW>()
                       : blocks_per_cu<k_step<GT, 0, MODE, NT_BLOCK_LARGE, NT_ITERS_LARGE, TABLE, true>, NT_BLOCK_LARGE>();
      }
#undef NT_OCC
    }
    per_launch = (int64_t)cu_count() * per_cu * (p.J <= NT_JCHUNK ? NT_GENS_DEFER : NT_GENS_LARGE);
    if (per_launch > ntiles) per_launch = ntiles;
  }
  for (int64_t slot0 = 0; slot0 < ntiles; slot0 += per_launch) {
    const int64_t slot1 = (ntiles - slot0 < per_launch) ? ntiles : slot0 + per_launch;
    const unsigned grid = (unsigned)((slot1 - slot0 < max_grid) ? slot1 - slot0 : max_grid);
#define NT_CASE(JJ)                                                                                             \
  case JJ:                                                                                                      \
    if constexpr (WRITES && JJ * GT::ESIZE >= defer_row_bytes(MODE)) {                                          \
      if (long_class) {                                                                                         \
        hipLaunchKernelGGL((k_step<GT, JJ, MODE, NT_BLOCK_DEFER, NT_ITERS_DEFER, TABLE, true, true>), dim3(grid), \
                           dim3(NT_BLOCK_DEFER), 0, st, p, nfull, ntiles, slot0, slot1, ctl);                   \
        break;                                                                                                  \
      }                                                                                                         \
    }                                                                                                           \
    hipLaunchKernelGGL((k_step<GT, JJ, MODE, BS, IS, TABLE, GBAR>), dim3(grid), dim3(BS), 0, st, p, nfull,      \
                       ntiles, slot0, slot1, ctl);                                                              \
    break;
    switch (p.J) {
      NT_CASE(2) NT_CASE(3) NT_CASE(4) NT_CASE(5) NT_CASE(6) NT_CASE(7) NT_CASE(8) NT_CASE(9)
      NT_CASE(10) NT_CASE(11) NT_CASE(12) NT_CASE(13) NT_CASE(14) NT_CASE(15) NT_CASE(16)
      default:
        if (MODE == MODE_STATS && p.gbar == nullptr)
          hipLaunchKernelGGL((k_step<GT, 0, MODE, NT_BLOCK_LARGE_STATS, NT_ITERS_LARGE_STATS, TABLE, false>), dim3(grid),
                             dim3(NT_BLOCK_LARGE_STATS), 0, st, p, nfull, ntiles, slot0, slot1, ctl);
        else if (!long_class)
          hipLaunchKernelGGL((k_step<GT, 0, MODE, NT_BLOCK_MANY_SHORT, NT_ITERS_MANY_SHORT, TABLE, true>), dim3(grid),
                             dim3(NT_BLOCK_MANY_SHORT), 0, st, p, nfull, ntiles, slot0, slot1, ctl);
        else if (p.J <= NT_FEW_ROWS)
          hipLaunchKernelGGL((k_step<GT, 0, MODE, NT_BLOCK_FEW, NT_ITERS_FEW, TABLE, true>), dim3(grid),
                             dim3(NT_BLOCK_FEW), 0, st, p, nfull, ntiles, slot0, slot1, ctl);
        else
          hipLaunchKernelGGL((k_step<GT, 0, MODE, NT_BLOCK_LARGE, NT_ITERS_LARGE, TABLE, true>), dim3(grid),
                             dim3(NT_BLOCK_LARGE), 0, st, p, nfull, ntiles, slot0, slot1, ctl);
    }
#undef NT_CASE
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// picks the launch class (block size, sweeps per tile) that tile_cfg() describes
template <class GT, int MODE, bool TABLE>
hipError_t launch_step(const StepParams& p, int cls, int64_t nfull, int64_t ntiles, WsControl* ctl, int grid,
                       hipStream_t st) {
  if constexpr (MODE == MODE_STATS) {
    // read-only statistics over a short vector borrow the kernels that can also store gbar (there is none to store)
    if (p.gbar || (cls == CLS_SHORT_STATS && p.J <= NT_JCHUNK))
      return launch_step_shape<GT, MODE, TABLE, NT_BLOCK_STATS_GBAR, NT_ITERS_STATS_GBAR, true>(p, cls, nfull, ntiles,
                                                                                                 ctl, grid, st);
    return launch_step_shape<GT, MODE, TABLE, NT_BLOCK_STATS, NT_ITERS_STATS, false>(p, cls, nfull, ntiles, ctl, grid,
                                                                                      st);
  } else if constexpr (MODE == MODE_ADAMW) {
    return launch_step_shape<GT, MODE, TABLE, NT_BLOCK_ADAMW, NT_ITERS_ADAMW, true>(p, cls, nfull, ntiles, ctl, grid,
                                                                                     st);
  } else {
    return launch_step_shape<GT, MODE, TABLE, NT_BLOCK, NT_ITERS, true>(p, cls, nfull, ntiles, ctl, grid, st);
  }
}

template <class GT, bool TABLE>
hipError_t launch_step_mode(int mode, const StepParams& p, int cls, int64_t nfull, int64_t ntiles, WsControl* ctl,
                            int grid, hipStream_t st) {
  switch (mode) {
    case MODE_FULL: return launch_step<GT, MODE_FULL, TABLE>(p, cls, nfull, ntiles, ctl, grid, st);
    case MODE_STATS: return launch_step<GT, MODE_STATS, TABLE>(p, cls, nfull, ntiles, ctl, grid, st);
    default: return launch_step<GT, MODE_ADAMW, TABLE>(p, cls, nfull, ntiles, ctl, grid, st);
  }
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

inline void launch_finalize(const double* in, int64_t n, bool packed, const DecideParams& q, nt_result* out,
                            const WsHeader& hdr, WsHeader* hdr_out, hipStream_t st) {
  if (n <= NT_FIN_SMALL)
    hipLaunchKernelGGL(k_finalize<256>, dim3(1), dim3(256), 0, st, in, n, packed, q, out, hdr, hdr_out);
  else
    hipLaunchKernelGGL(k_finalize<NT_FIN_THREADS>, dim3(1), dim3(NT_FIN_THREADS), 0, st, in, n, packed, q, out, hdr,
                       hdr_out);
}

}  // namespace

extern "C" {

int64_t normtest_tile_coords(int64_t J) { return J >= 2 ? NT_TILE_MAX : 0; }

// Bytes of the record, the tile partials and the group partials: what every call needs.
static size_t partials_bytes(int64_t J, int64_t d) {
  const int64_t tc = min_tile_coords(J);
  const int64_t ntiles = (d + tc - 1) / tc;
  const int64_t n = ntiles > 0 ? ntiles : 1;
  const int64_t ngroups = ntiles > NT_DIRECT_TILES ? (ntiles + NT_GROUP_TILES - 1) / NT_GROUP_TILES : 0;
  return (size_t)(NT_WS_HEADER + n * NT_NV + ngroups * 2 * NT_NV) * sizeof(double);
}

size_t normtest_workspace_bytes(int64_t J, int64_t d) {
  if (J < 2 || d < 0) return 0;
  return partials_bytes(J, d);
}

// dtype and flags do not change the size (they did while many-row steps kept gbar in the workspace)
size_t normtest_workspace_bytes_for(nt_dtype gdtype, int64_t J, int64_t d, uint32_t flags) {
  (void)flags;
  if (J < 2 || d < 0 || (gdtype != NT_F32 && gdtype != NT_BF16)) return 0;
  return partials_bytes(J, d);
}

// AdamW constants in fp64 on the host, rounded once to fp32.
static void fill_adamw_params(StepParams& p, const nt_hyper* hyper) {
  const double bc1 = 1.0 - std::pow(hyper->beta1, (double)hyper->step);
  const double bc2 = 1.0 - std::pow(hyper->beta2, (double)hyper->step);
  p.beta1 = (float)hyper->beta1;
  p.omb1 = (float)(1.0 - hyper->beta1);
  p.beta2 = (float)hyper->beta2;
  p.omb2 = (float)(1.0 - hyper->beta2);
  p.decay = (float)(1.0 - hyper->lr * hyper->weight_decay);
  p.step_size = (float)(hyper->lr / bc1);
  p.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
  p.eps = (float)hyper->eps;
}

// Validation shared by normtest_step and normtest_step_clipped; `flags` are the flags the kernels
// will run with.  Nothing is enqueued here.
static int check_step_args(const void* grads, nt_dtype gdtype, int64_t J, int64_t d, int64_t ld, const float* w,
                           const float* m, const float* v, const float* gbar_out, uint32_t flags,
                           const nt_hyper* hyper, const nt_shard_info* shard, const void* workspace,
                           size_t workspace_bytes, const nt_result* result_dev) {
  if (gdtype != NT_F32 && gdtype != NT_BF16) return NT_ERR_UNSUPPORTED;
  if (J < 2 || J > (1 << 20) || d < 0 || ld < d) return NT_ERR_BAD_ARG;
  if (!hyper_ok(hyper, J) || !result_dev || !workspace) return NT_ERR_BAD_ARG;
  if (((uintptr_t)result_dev & 7u) || ((uintptr_t)workspace & 7u)) return NT_ERR_BAD_ARG;
  if (d > 0 && !grads) return NT_ERR_BAD_ARG;
  if (d > 0 && (flags & NT_DO_ADAMW) && (!w || !m || !v)) return NT_ERR_BAD_ARG;
  if (d > 0 && (flags & NT_WRITE_GBAR) && !gbar_out) return NT_ERR_BAD_ARG;
  const int esize = gdtype == NT_F32 ? 4 : 2;
  if (((uintptr_t)grads & (uintptr_t)(esize - 1)) || ((uintptr_t)w & 3u) || ((uintptr_t)m & 3u) ||
      ((uintptr_t)v & 3u) || ((flags & NT_WRITE_GBAR) && ((uintptr_t)gbar_out & 3u)))
    return NT_ERR_BAD_ARG;
  if (shard) {
    if (shard->num_shards < 1 || shard->shard_id < 0 || shard->shard_id >= shard->num_shards ||
        shard->shard_offset < 0 || shard->d_global < 0 || shard->shard_offset + d > shard->d_global)
      return NT_ERR_BAD_ARG;
  }
  if (workspace_bytes < normtest_workspace_bytes_for(gdtype, J, d, flags)) return NT_ERR_WORKSPACE_TOO_SMALL;
  return NT_OK;
}

// Enqueue the streaming kernel and the reduction/decision kernels.  Arguments are already validated.
// `table`: grads is a device array of J row pointers instead of the first row of a strided matrix.
// `d_whole`: length of the vector these d coordinates are a part of (d itself for a call that stands alone).
static int enqueue_step(const void* grads, bool table, nt_dtype gdtype, int64_t J, int64_t d, int64_t d_whole,
                        int64_t ld, float* w, float* m, float* v, float* gbar_out, uint32_t flags, const nt_hyper* hyper,
                        double max_norm, void* workspace, nt_result* result_dev, hipStream_t st) {
  const int esize = gdtype == NT_F32 ? 4 : 2;
  const int mode = (flags & NT_DO_STATS) ? ((flags & NT_DO_ADAMW) ? MODE_FULL : MODE_STATS) : MODE_ADAMW;
  const int cls = launch_class(J, esize, mode, (flags & NT_WRITE_GBAR) != 0, d_whole);
  const int64_t tc = tile_cfg(J, esize, mode, (flags & NT_WRITE_GBAR) != 0, d_whole).coords();
  const int64_t ntiles = (d + tc - 1) / tc;

  StepParams p;
  std::memset(&p, 0, sizeof(p));
  p.grads = grads;
  p.ld = ld;
  p.d = d;
  p.J = (int)J;
  p.w = w;
  p.m = m;
  p.v = v;
  p.gbar = (flags & NT_WRITE_GBAR) ? gbar_out : nullptr;
  p.partials = (double*)workspace + NT_WS_HEADER;
  p.inv_J = 1.0 / (double)J;
  if (flags & NT_DO_ADAMW) fill_adamw_params(p, hyper);
  p.coord_thr = (flags & NT_COORD_TEST)
                    ? (float)(hyper->eta * hyper->eta * (double)hyper->b_k * (double)(J - hyper->ddof))
                    : -1.0f;

  WsControl* ctl = (WsControl*)((double*)workspace + NT_WS_CONTROL);
  if (ntiles > 0) {
    // row alignment: checked here for a strided matrix, by a small kernel for a pointer table
    if (table) {
      hipLaunchKernelGGL(k_rows_aligned, dim3(1), dim3(256), 0, st, (const void* const*)grads, (int)J, ctl);
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return hip_code(e);
    }
    bool al = table || (aligned16(grads) && ((ld * esize) % 16 == 0));
    if (mode != MODE_STATS) al = al && aligned16(w) && aligned16(m) && aligned16(v);
    if (p.gbar) al = al && aligned16(p.gbar);
    const int64_t nfull = al ? d / tc : 0;
    const int64_t max_grid = (int64_t)cu_count() * NT_BLOCKS_PER_CU;
    const int grid = (int)(ntiles < max_grid ? ntiles : max_grid);
    hipError_t e;
    if (table)
      e = (gdtype == NT_F32) ? launch_step_mode<F32, true>(mode, p, cls, nfull, ntiles, ctl, grid, st)
                             : launch_step_mode<BF16, true>(mode, p, cls, nfull, ntiles, ctl, grid, st);
    else
      e = (gdtype == NT_F32) ? launch_step_mode<F32, false>(mode, p, cls, nfull, ntiles, ctl, grid, st)
                             : launch_step_mode<BF16, false>(mode, p, cls, nfull, ntiles, ctl, grid, st);
    if (e != hipSuccess) return hip_code(e);
  }

  DecideParams q;
  q.J = J;
  q.eta = hyper->eta;
  q.max_norm = max_norm;
  q.b_k = hyper->b_k;
  q.b_max = hyper->b_max;
  q.round_to = hyper->round_to;
  q.ddof = hyper->ddof;
  q.flags = flags;
  const double* partials = (const double*)workspace + NT_WS_HEADER;
  const bool two_level = (flags & NT_DO_STATS) && ntiles > NT_DIRECT_TILES;
  const int64_t ngroups = two_level ? (ntiles + NT_GROUP_TILES - 1) / NT_GROUP_TILES : 0;
  WsHeader hdr;
  std::memset(&hdr, 0, sizeof(hdr));
  hdr.magic = NT_WS_MAGIC;
  hdr.tile_coords = tc;
  hdr.ntiles = ntiles;
  hdr.ngroups = ngroups;
  hdr.d = d;
  hdr.J = J;
  hdr.gdtype = (int32_t)gdtype;
  hdr.has_stats = (flags & NT_DO_STATS) ? 1 : 0;
  hdr.coord_thr = (double)p.coord_thr;
  hdr.q = q;
  WsHeader* hdr_out = (WsHeader*)workspace;
  if (two_level) {
    double* groups = (double*)workspace + NT_WS_HEADER + NT_NV * ntiles;
    hipLaunchKernelGGL(k_reduce_groups, dim3((unsigned)ngroups), dim3(NT_GROUP_THREADS), 0, st, partials, ntiles, groups);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_code(e);
    launch_finalize(groups, ngroups, true, q, result_dev, hdr, hdr_out, st);
  } else {
    launch_finalize(partials, ntiles, false, q, result_dev, hdr, hdr_out, st);
  }
  return hip_code(hipGetLastError());
}

// Enqueue AdamW on scale * gbar (phase 2 of the clipped variant).  Arguments are already validated.
static int enqueue_adamw_gbar(const float* gbar, int64_t d, float* w, float* m, float* v, const nt_hyper* hyper,
                              double grad_scale, const nt_result* result_dev, hipStream_t st) {
  if (d == 0) return NT_OK;
  StepParams p;
  std::memset(&p, 0, sizeof(p));
  p.d = d;
  p.w = w;
  p.m = m;
  p.v = v;
  fill_adamw_params(p, hyper);
  const int aligned = aligned16(gbar) && aligned16(w) && aligned16(m) && aligned16(v);
  const int64_t per_block = (int64_t)NT_AUX_BLOCK * NT_VEC;
  const int64_t nblocks = (d + per_block - 1) / per_block;
  // in runs of blocks, like the step kernel (see NT_CHUNK_FULL)
  const int64_t per_launch = NT_CHUNK_ADAMW_GBAR / per_block;
  for (int64_t b0 = 0; b0 < nblocks; b0 += per_launch) {
    const int64_t grid = (nblocks - b0 < per_launch) ? nblocks - b0 : per_launch;
    hipLaunchKernelGGL(k_adamw_gbar, dim3((unsigned)grid), dim3(NT_AUX_BLOCK), 0, st, p, gbar, (float)grad_scale,
                       result_dev, aligned, b0);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_code(e);
  }
  return NT_OK;
}

// Length of the vector a call's d coordinates belong to: what the caller's shard record says, else d.
inline int64_t whole_length(int64_t d, const nt_shard_info* shard) {
  return (shard && shard->d_global > d) ? shard->d_global : d;
}

// The step as the caller's flags describe it, always one pass (NT_ONE_PASS, which once kept many-row steps from
// being split into two passes, is accepted and changes nothing).
static int enqueue_step_routed(const void* grads, bool table, nt_dtype gdtype, int64_t J, int64_t d,
                               const nt_shard_info* shard, int64_t ld, float* w, float* m, float* v, float* gbar_out,
                               const nt_hyper* hyper, void* workspace, nt_result* result_dev, hipStream_t st) {
  return enqueue_step(grads, table, gdtype, J, d, whole_length(d, shard), ld, w, m, v, gbar_out, hyper->flags, hyper, 0.0,
                      workspace, result_dev, st);
}

int normtest_step(const void* grads, nt_dtype gdtype, int64_t J, int64_t d, int64_t ld, float* w, float* m,
                  float* v, float* gbar_out, const nt_hyper* hyper, const nt_shard_info* shard, void* workspace,
                  size_t workspace_bytes, nt_result* result_dev, void* hip_stream) {
  if (!hyper) return NT_ERR_BAD_ARG;
  const int rc = check_step_args(grads, gdtype, J, d, ld, w, m, v, gbar_out, hyper->flags, hyper, shard, workspace,
                                 workspace_bytes, result_dev);
  if (rc != NT_OK) return rc;
  return enqueue_step_routed(grads, false, gdtype, J, d, shard, ld, w, m, v, gbar_out, hyper, workspace, result_dev,
                             (hipStream_t)hip_stream);
}

int normtest_step_rows(const void* const* grad_rows_dev, nt_dtype gdtype, int64_t J, int64_t d, float* w, float* m,
                       float* v, float* gbar_out, const nt_hyper* hyper, const nt_shard_info* shard, void* workspace,
                       size_t workspace_bytes, nt_result* result_dev, void* hip_stream) {
  if (!hyper || ((uintptr_t)grad_rows_dev & 7u)) return NT_ERR_BAD_ARG;
  // the table stands in for the matrix; its entries cannot be inspected from the host
  const int rc = check_step_args(grad_rows_dev, gdtype, J, d, d, w, m, v, gbar_out, hyper->flags, hyper, shard,
                                 workspace, workspace_bytes, result_dev);
  if (rc != NT_OK) return rc;
  return enqueue_step_routed(grad_rows_dev, true, gdtype, J, d, shard, d, w, m, v, gbar_out, hyper, workspace, result_dev,
                             (hipStream_t)hip_stream);
}

// Address of this device's copy of `scratch`, looked up once per device (the array's name is only a host-side
// handle of the symbol; kernels, copies and fills take this pointer).
static int scratch_address(void** out) {
  static void* cached[64] = {nullptr};
  int dev = 0;
  const hipError_t e0 = hipGetDevice(&dev);
  if (e0 != hipSuccess) return hip_code(e0);
  if (dev < 0 || dev >= 64) return NT_ERR_UNSUPPORTED;
  void* ptr = __atomic_load_n(&cached[dev], __ATOMIC_ACQUIRE);
  if (!ptr) {
    const hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_code(e);
    if (!ptr) return NT_ERR_UNSUPPORTED;
    __atomic_store_n(&cached[dev], ptr, __ATOMIC_RELEASE);
  }
  *out = ptr;
  return NT_OK;
}

int64_t normtest_static_max_coords(int64_t J) {
  if (J < 2 || J > (1 << 20)) return 0;
  // largest d whose record, tile partials and group partials fit: partials_bytes is monotone in d
  int64_t lo = 0, hi = (int64_t)1 << 40;
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo + 1) / 2;
    if (partials_bytes(J, mid) <= NT_SCRATCH_BYTES) lo = mid; else hi = mid - 1;
  }
  return lo;
}

int normtest_step_static(const void* grads, nt_dtype gdtype, int64_t J, int64_t d, int64_t ld, float* w, float* m,
                         float* v, float* gbar_out, const nt_hyper* hyper, const nt_shard_info* shard,
                         nt_result* result_dev, void* hip_stream) {
  if (!hyper) return NT_ERR_BAD_ARG;
  if (J >= 2 && J <= (1 << 20) && d > normtest_static_max_coords(J)) return NT_ERR_TOO_LARGE;
  nt_hyper hy = *hyper;
  // validate with a stand-in for the workspace (any non-null, aligned address: nothing is enqueued here)
  const int rc = check_step_args(grads, gdtype, J, d, ld, w, m, v, gbar_out, hy.flags, &hy, shard, (const void*)256,
                                 (size_t)-1, result_dev);
  if (rc != NT_OK) return rc;
  void* ws = nullptr;
  const int rs = scratch_address(&ws);
  if (rs != NT_OK) return rs;
  return enqueue_step_routed(grads, false, gdtype, J, d, shard, ld, w, m, v, gbar_out, &hy, ws, result_dev,
                             (hipStream_t)hip_stream);
}

int normtest_step_clipped(const void* grads, nt_dtype gdtype, int64_t J, int64_t d, int64_t ld, float* w, float* m,
                          float* v, float* gbar_buf, double max_norm, const nt_hyper* hyper,
                          const nt_shard_info* shard, void* workspace, size_t workspace_bytes, nt_result* result_dev,
                          void* hip_stream) {
  if (!hyper || std::isnan(max_norm)) return NT_ERR_BAD_ARG;
  const uint32_t need = NT_DO_STATS | NT_DO_ADAMW;
  if ((hyper->flags & need) != need || (hyper->flags & NT_PARTIAL)) return NT_ERR_BAD_ARG;
  // validate as the fused step with the mean written out (this also checks w, m, v and the AdamW scalars)
  const int rc = check_step_args(grads, gdtype, J, d, ld, w, m, v, gbar_buf, hyper->flags | NT_WRITE_GBAR, hyper,
                                 shard, workspace, workspace_bytes, result_dev);
  if (rc != NT_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  const int rc1 = enqueue_step(grads, false, gdtype, J, d, whole_length(d, shard), ld, nullptr, nullptr, nullptr, gbar_buf,
                               NT_DO_STATS | NT_WRITE_GBAR | (hyper->flags & NT_COORD_TEST), hyper, max_norm, workspace,
                               result_dev, st);
  if (rc1 != NT_OK) return rc1;
  return enqueue_adamw_gbar(gbar_buf, d, w, m, v, hyper, 1.0, result_dev, st);
}

int normtest_layer_stats(const void* grads, int rows_are_table, nt_dtype gdtype, int64_t J, int64_t d, int64_t ld,
                         const int64_t* layer_offsets_dev, int32_t L, const void* workspace,
                         nt_layer_stats* layers_dev, void* hip_stream) {
  if (gdtype != NT_F32 && gdtype != NT_BF16) return NT_ERR_UNSUPPORTED;
  if (J < 2 || J > (1 << 20) || d < 0 || (!rows_are_table && ld < d)) return NT_ERR_BAD_ARG;
  if (L < 1 || L > (1 << 24) || !layer_offsets_dev || !workspace || !layers_dev) return NT_ERR_BAD_ARG;
  if (((uintptr_t)layer_offsets_dev & 7u) || ((uintptr_t)workspace & 7u) || ((uintptr_t)layers_dev & 7u))
    return NT_ERR_BAD_ARG;
  if (d > 0 && !grads) return NT_ERR_BAD_ARG;
  const int esize = gdtype == NT_F32 ? 4 : 2;
  if ((uintptr_t)grads & (uintptr_t)(rows_are_table ? 7 : esize - 1)) return NT_ERR_BAD_ARG;
  StepParams p;
  std::memset(&p, 0, sizeof(p));
  p.grads = grads;
  p.ld = rows_are_table ? d : ld;
  p.d = d;
  p.J = (int)J;
  p.inv_J = 1.0 / (double)J;
  p.coord_thr = -1.0f;  // the kernel takes the threshold of the recorded step
  hipStream_t st = (hipStream_t)hip_stream;
  const double* ws = (const double*)workspace;
  if (rows_are_table) {
    if (gdtype == NT_F32)
      hipLaunchKernelGGL((k_layer_stats<F32, true>), dim3(L), dim3(NT_LAYER_THREADS), 0, st, p, layer_offsets_dev, ws, layers_dev);
    else
      hipLaunchKernelGGL((k_layer_stats<BF16, true>), dim3(L), dim3(NT_LAYER_THREADS), 0, st, p, layer_offsets_dev, ws, layers_dev);
  } else {
    if (gdtype == NT_F32)
      hipLaunchKernelGGL((k_layer_stats<F32, false>), dim3(L), dim3(NT_LAYER_THREADS), 0, st, p, layer_offsets_dev, ws, layers_dev);
    else
      hipLaunchKernelGGL((k_layer_stats<BF16, false>), dim3(L), dim3(NT_LAYER_THREADS), 0, st, p, layer_offsets_dev, ws, layers_dev);
  }
  return hip_code(hipGetLastError());
}

int normtest_adamw_gbar(const float* gbar, int64_t d, float* w, float* m, float* v, const nt_hyper* hyper,
                        double grad_scale, const nt_result* result_dev, void* hip_stream) {
  if (!hyper || d < 0 || !std::isfinite(grad_scale)) return NT_ERR_BAD_ARG;
  if (hyper->step < 1 || !(hyper->lr >= 0.0) || !std::isfinite(hyper->lr) ||
      !(hyper->beta1 >= 0.0 && hyper->beta1 < 1.0) || !(hyper->beta2 >= 0.0 && hyper->beta2 < 1.0) ||
      !(hyper->eps >= 0.0) || !std::isfinite(hyper->eps) || !(hyper->weight_decay >= 0.0) ||
      !std::isfinite(hyper->weight_decay))
    return NT_ERR_BAD_ARG;
  if (d > 0 && (!gbar || !w || !m || !v)) return NT_ERR_BAD_ARG;
  if (((uintptr_t)gbar & 3u) || ((uintptr_t)w & 3u) || ((uintptr_t)m & 3u) || ((uintptr_t)v & 3u) ||
      ((uintptr_t)result_dev & 7u))
    return NT_ERR_BAD_ARG;
  return enqueue_adamw_gbar(gbar, d, w, m, v, hyper, grad_scale, result_dev, (hipStream_t)hip_stream);
}

double normtest_clip_coef(double gbar_sq, double max_norm) { return clip_coef(gbar_sq, max_norm); }

int normtest_resplit(int64_t b, int64_t J, int64_t accum_base, int64_t micro_max, int64_t* micro, int64_t* accum,
                     int64_t* global_batch) {
  if (b < 1 || J < 1 || accum_base < 1 || micro_max < 1 || !micro || !accum || !global_batch) return NT_ERR_BAD_ARG;
  // samples each worker must see, accumulation steps needed at the largest micro-batch, never below the base
  const int64_t per_worker = (b + J - 1) / J;
  int64_t steps = (per_worker + micro_max - 1) / micro_max;
  if (steps < accum_base) steps = accum_base;
  const int64_t chunk = J * steps;
  *micro = (b + chunk - 1) / chunk;
  *accum = steps;
  *global_batch = chunk * *micro;
  return NT_OK;
}

uint32_t normtest_schedule_flags(int64_t step, int64_t test_interval, int64_t b_k, int64_t b_max, uint32_t flags) {
  if (step < 1 || test_interval < 1 || b_k < 1 || b_max < 0) return flags;
  const bool at_maximum = b_max > 0 && b_k >= b_max;
  const bool on_interval = (step - 1) % test_interval == 0;
  if (on_interval && !at_maximum) return flags;
  return flags & ~(uint32_t)(NT_DO_STATS | NT_PARTIAL | NT_COORD_TEST);
}

int normtest_combine(const nt_result* partials, int32_t n, int64_t J, const nt_hyper* hyper, nt_result* out) {
  if (!partials || !out || n < 1 || J < 2 || !hyper) return NT_ERR_BAD_ARG;
  if (!(hyper->eta > 0.0) || !std::isfinite(hyper->eta) || hyper->b_k < 1 || hyper->b_max < 0 ||
      hyper->round_to < 1 || hyper->round_to > NT_ROUND_TO_MAX || (hyper->ddof != 0 && hyper->ddof != 1) || J - hyper->ddof < 1)
    return NT_ERR_BAD_ARG;
  dd tot[3] = {{0.0, 0.0}, {0.0, 0.0}, {0.0, 0.0}};
  uint32_t status = 0;
  int64_t coord_fail = 0;  // the count is additive over shards; missing in one shard = missing in the total
  double coord_max = 0.0;  // the largest ratio over shards is the largest of the shards' values
  for (int32_t s = 0; s < n; ++s) {
    if (partials[s].status & NT_STATUS_NO_STATS) return NT_ERR_BAD_ARG;
    coord_fail = (coord_fail < 0 || partials[s].coord_fail < 0) ? -1 : coord_fail + partials[s].coord_fail;
    if (partials[s].coord_fail >= 0 && partials[s].coord_max_ratio > coord_max) coord_max = partials[s].coord_max_ratio;
    const dd a = {partials[s].A, partials[s].A_lo}, b = {partials[s].B, partials[s].B_lo},
             c = {partials[s].C, partials[s].C_lo};
    tot[0] = dd_add(tot[0], a);
    tot[1] = dd_add(tot[1], b);
    tot[2] = dd_add(tot[2], c);
    status |= partials[s].status & NT_STATUS_NONFINITE;
  }
  nt_result r;
  std::memset(&r, 0, sizeof(r));
  r.A = tot[0].hi; r.A_lo = tot[0].lo;
  r.B = tot[1].hi; r.B_lo = tot[1].lo;
  r.C = tot[2].hi; r.C_lo = tot[2].lo;
  if (status & NT_STATUS_NONFINITE) {
    // a non-finite low part would otherwise poison finite high parts; report the plain sums
    r.A = r.B = r.C = 0.0;
    for (int32_t s = 0; s < n; ++s) {
      r.A += partials[s].A;
      r.B += partials[s].B;
      r.C += partials[s].C;
    }
    r.A_lo = r.B_lo = r.C_lo = 0.0;
  }
  r.status = 0;
  DecideParams q;
  q.J = J;
  q.eta = hyper->eta;
  q.b_k = hyper->b_k;
  q.b_max = hyper->b_max;
  q.round_to = hyper->round_to;
  q.max_norm = 0.0;
  q.ddof = hyper->ddof;
  q.flags = NT_DO_STATS;
  decide(q, &r);
  r.coord_fail = coord_fail;
  r.coord_max_ratio = coord_fail < 0 ? -1.0 : coord_max;
  *out = r;
  return NT_OK;
}

int normtest_calib_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src || !aligned16(dst) || !aligned16(src) || (bytes & 15u)) return NT_ERR_BAD_ARG;
  if (bytes == 0) return NT_OK;
  const int64_t n16 = (int64_t)(bytes / 16);
  const int64_t want = (n16 + NT_AUX_BLOCK - 1) / NT_AUX_BLOCK;
  const int64_t max_grid = (int64_t)cu_count() * NT_BLOCKS_PER_CU;
  const int grid = (int)(want < max_grid ? want : max_grid);
  hipLaunchKernelGGL(k_copy16, dim3(grid), dim3(NT_AUX_BLOCK), 0, (hipStream_t)hip_stream, (f32x4*)dst,
                     (const u32x4*)src, n16);
  return hip_code(hipGetLastError());
}

int normtest_calib_streams(void* buf, size_t buf_bytes, int64_t coords, int row_reads, int reads, int writes, int rmw,
                           int64_t launch_coords, void* hip_stream) {
  if (!buf || !aligned16(buf) || coords < 0 || (coords & 3) || row_reads < 0 || reads < 0 || writes < 0 ||
      launch_coords < 0 || (launch_coords & 3))
    return NT_ERR_BAD_ARG;
  if (row_reads > NT_CALIB_MAX_R8 || reads > NT_CALIB_MAX_R16 || writes > NT_CALIB_MAX_W || row_reads + reads + writes == 0)
    return NT_ERR_UNSUPPORTED;
  // streams sit one after the other: row-like ones of 2 bytes per coordinate first, then those of 4
  const size_t row_bytes = (((size_t)coords * 2 + 255u) & ~(size_t)255u), vec_bytes = (((size_t)coords * 4 + 255u) & ~(size_t)255u);
  const size_t need = row_bytes * (size_t)row_reads + vec_bytes * (size_t)(reads + writes) + 16;
  if (buf_bytes < need) return NT_ERR_WORKSPACE_TOO_SMALL;
  if (coords == 0) return NT_OK;
  CalibStreams s;
  std::memset(&s, 0, sizeof(s));
  char* at = (char*)buf;
  for (int k = 0; k < row_reads; ++k, at += row_bytes) s.r8[k] = at;
  for (int k = 0; k < reads; ++k, at += vec_bytes) s.r16[k] = at;
  for (int k = 0; k < writes; ++k, at += vec_bytes) s.w[k] = at;
  s.sink = (uint32_t*)at;
  const int64_t ngroups = coords / 4;
  // like the step kernel, in launches over runs of consecutive coordinates (whole blocks) if the caller says so
  const int64_t per_block = NT_AUX_BLOCK;
  int64_t per_launch = launch_coords > 0 ? launch_coords / 4 / per_block * per_block : ngroups;
  if (per_launch < per_block) per_launch = per_block;
  const int64_t max_grid = (int64_t)cu_count() * NT_BLOCKS_PER_CU;
  hipStream_t st = (hipStream_t)hip_stream;
  bool found = false;
#define NT_CALIB(R8, R16, W, RMW)                                                                                  \
  if (!found && row_reads == R8 && reads == R16 && writes == W && (rmw != 0) == RMW) {                              \
    for (int64_t g0 = 0; g0 < ngroups; g0 += per_launch) {                                                         \
      const int64_t g1 = (ngroups - g0 < per_launch) ? ngroups : g0 + per_launch;                                  \
      const int64_t want = (g1 - g0 + per_block - 1) / per_block;                                                  \
      const int grid = (int)(want < max_grid ? want : max_grid);                                                   \
      hipLaunchKernelGGL((k_calib_streams<R8, R16, W, RMW>), dim3(grid), dim3(NT_AUX_BLOCK), 0, st, s, g0, g1);    \
    }                                                                                                              \
    found = true;                                                                                                  \
  }
#define NT_CALIB_ROW(R16) NT_CALIB(0, R16, 0, false) NT_CALIB(0, R16, 1, false) NT_CALIB(0, R16, 2, false) NT_CALIB(0, R16, 3, false)
  // the matrix of read streams x written streams ...
  NT_CALIB(0, 0, 1, false) NT_CALIB(0, 0, 2, false) NT_CALIB(0, 0, 3, false)
  NT_CALIB_ROW(1) NT_CALIB_ROW(2) NT_CALIB_ROW(4) NT_CALIB_ROW(8) NT_CALIB_ROW(11)
  // ... in-place updates alone ...
  NT_CALIB(0, 0, 1, true) NT_CALIB(0, 0, 3, true)
  // ... and the traffic of the step itself: J row reads with three in-place fp32 arrays, rows alone, and the same
  // bytes with the results going to separate arrays
  NT_CALIB(4, 0, 3, true) NT_CALIB(8, 0, 3, true) NT_CALIB(16, 0, 3, true)
  NT_CALIB(4, 0, 0, false) NT_CALIB(8, 0, 0, false) NT_CALIB(16, 0, 0, false)
  NT_CALIB(8, 0, 1, false) NT_CALIB(8, 3, 3, false)
#undef NT_CALIB_ROW
#undef NT_CALIB
  if (!found) return NT_ERR_UNSUPPORTED;
  return hip_code(hipGetLastError());
}

const char* normtest_strerror(int code) {
  switch (code) {
    case NT_OK: return "success";
    case NT_ERR_BAD_ARG: return "bad argument (null or misaligned pointer, J < 2, d < 0, ld < d, or invalid hyper-parameters)";
    case NT_ERR_UNSUPPORTED: return "unsupported gradient dtype";
    case NT_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than normtest_workspace_bytes(J, d)";
    case NT_ERR_TOO_LARGE: return "d beyond normtest_static_max_coords(J): the built-in scratch cannot hold the partial sums";
    default: break;
  }
  if (code <= NT_ERR_HIP_BASE) return hipGetErrorString((hipError_t)(NT_ERR_HIP_BASE - code));
  return "unknown error code";
}

}  // extern "C"
