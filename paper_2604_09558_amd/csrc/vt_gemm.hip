// GEMM consumer on the matrix cores: C[g] = A[g] . B[g], A and B read through virtual-tensor
// descriptors (Sec. 2.3: the three stages of a tiled matmul; only stage 1 changes, Sec. 4.2).
// gfx950, wave64, v_mfma_f32_32x32x16 (bf16 / f16 operands, fp32 accumulation).
//
// Tiling: one workgroup of 4 waves computes a 256 x 256 tile of C over K in steps of 64; each
// wave owns a 128 x 128 quadrant (4 x 4 MFMA blocks, 256 accumulator registers per lane).
// A is staged in LDS with the contraction index contiguous ([row][k], 16-byte units,
// XOR-swizzled: a fragment is one conflict-free ds_read_b128 in the matrix-core operand layout),
// B as [k][n] with padded rows; LDS is double buffered, one barrier per step.
//
// Stage 1 through the map (block-wise virtual tensor I/O): the map of a 2-D operand separates
// into row_offset(m) + col_offset(k).  A thread keeps the offsets of its 8 rows for the whole
// K loop (mixed-radix digits and, for index_select, a table lookup: evaluated once) and
// evaluates the column offset of its 8-element chunk once per step.  Global loads stay
// 16 bytes per lane and cover whole 128-byte lines whenever the map keeps runs of 64 elements.
//   A ([M,K], K contiguous in runs of >= 8): chunk -> LDS directly.
//   B ([K,N], N contiguous, the usual row-major weight): rows go to LDS as they are loaded
//     ([k][n], 16 bytes per lane); the transposition into the operand layout (8 consecutive k
//     per lane) is done by the LDS itself on the way out (ds_read_b64_tr_b16, two per fragment).
//   B ([K,N] with K contiguous: an [N,K] weight seen through a Permute, the B_KMAJOR
//     instantiation): treated like A, chunks of 8 k of one column n -> LDS [n][k], swizzled.
// Workgroup ids are remapped so that each XCD (own L2) works on a contiguous band of tiles,
// walked in groups of 8 tile rows, which keeps the A and B panels of neighbouring tiles in
// that L2.  A launch covers up to 8 groups (grouped GEMM: one tile list over all groups).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <type_traits>
#include <vector>

#include "vt_gemm_common.h"
#include "vt_profile.h"

using namespace vt;
using namespace vt::gemm;

// profile marks: 0 start, 1 first tiles in LDS (K loop starts), 2 K loop done, 3 tile stored, 4 and 5 the
// shader cycle counter at marks 1 and 2, 7 compute die
VT_PROF_DECLARE(gemm)

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kMaxGroups = 8;
constexpr int kGroupRows = 8;      // tile rows walked together (L2 reuse of the B panel)
constexpr int kBPitch = BN * 2 + 64;   // bytes between k-rows of the B tile in LDS
constexpr int kMaxSteps = 1024;        // K steps whose offsets are tabulated in LDS (K <= 65536)

struct GemmGroup {
  const char* a;
  const char* b;
  char* c;
  AxisMap<5> a_row;
  AxisMap<3> a_col, b_row, b_col;
  int32_t M, tile_begin, tiles_m;
  int32_t k64;   // a K step of 64 never leaves the innermost K digit of A or of B: the step's offset is uniform
  int32_t b_kmajor;   // B's contiguous axis is K (all groups of a launch agree)
};

struct GemmParams {
  GemmGroup g[kMaxGroups];
  int32_t n_groups, N, K, tiles_n, total_tiles, chunk, c_f32, pad;
};

// Output written through a map (producer-side store, Sec. 4.2): columns [col_lo, col_hi) of C
// live in one physical tensor, element (m, n) at base + 2 * (row(m) + col(n - col_lo)).
struct OutPiece {
  char* base;
  int32_t col_lo, col_hi;
  AxisMap<3> row, col;
};
struct OutMap {
  OutPiece p[4];
  int32_t n, pad;
};

template <typename T, bool C_F32, bool K_TAIL, bool MAPPED, bool B_KMAJOR = false>
__global__ void __launch_bounds__(256) k_gemm(const GemmParams P, const OutMap O) {
  typedef Mma<T> M_;
  typedef typename M_::vec opvec;
  __shared__ uint4 ldsA[2][BM * 8];     // [row][8 chunks of 8 k], chunk c of row r at r*8 + (c ^ (r & 7))
  // B stays as loaded, [k][n] with n contiguous; rows are kBPitch bytes apart (64 bytes more than
  // a row, so that the 4 rows one transposing read touches fall into different banks)
  __shared__ __attribute__((aligned(16))) char ldsB[2][BK * kBPitch];
  // byte offsets of every K step along A's columns and B's rows (the part of the map that depends
  // on the step only), evaluated once per workgroup: nothing in the K loop reads kernel arguments
  __shared__ uint32_t step_a[kMaxSteps];
  __shared__ int64_t step_b[kMaxSteps];

  VT_PROF_BEGIN();
  VT_PROF(0);
  // ---- which tile: XCD-contiguous bands, groups of kGroupRows tile rows
  const int wg = blockIdx.x;
  const int slot = wg >> 3;
  const int idx = (wg & 7) * P.chunk + slot;
  if (slot >= P.chunk || idx >= P.total_tiles) return;
  int gi = 0;
#pragma unroll
  for (int i = 1; i < kMaxGroups; ++i)
    if (i < P.n_groups && idx >= P.g[i].tile_begin) gi = i;
  const GemmGroup& G = P.g[gi];
  const int local = idx - G.tile_begin;
  const int width = kGroupRows * P.tiles_n;
  const int first_m = (local / width) * kGroupRows;
  const int gsz = min(G.tiles_m - first_m, kGroupRows);
  const int tm = first_m + (local % width) % gsz;
  const int tn = (local % width) / gsz;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const int Mg = G.M, N = P.N, K = P.K;

  // ---- stage-1 bookkeeping: A rows of this thread (fixed over the K loop); pointers include the row offset
  const int a_c = t & 7, a_r0 = t >> 3;                 // chunk (8 k) and first row; rows a_r0 + 32 i
  uint32_t a_rowoff[8];                                 // byte offsets (the host checks that A spans < 4 GiB)
  if (G.a_row.tdig >= 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      a_rowoff[i] = (uint32_t)(axis_off_table(G.a_row, (uint32_t)min(tm * BM + a_r0 + 32 * i, Mg - 1)) * 2);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      a_rowoff[i] = (uint32_t)(axis_off(G.a_row, (uint32_t)min(tm * BM + a_r0 + 32 * i, Mg - 1)) * 2);
  }
  // B: an 8 (k) x 8 (n) block per thread; column chunk fixed over the K loop; the 8 rows are
  // consecutive k inside one innermost digit (its radix is a multiple of 8), stride b_kstride
  const int b_cn = t & 31, b_kb = t >> 5;
  const int b_n = tn * BN + b_cn * 8;
  const char* b_colptr = G.b + axis_off(G.b_col, (uint32_t)min(b_n, N - 8)) * 2;
  const int64_t b_kstride = G.b_row.stride[2] * 2;
  // B_KMAJOR: the thread's 8 columns n = a_r0 + 32 i (as for A's rows), chunk a_c of 8 k
  int64_t bk_coloff[8];
  if (B_KMAJOR) {
#pragma unroll
    for (int i = 0; i < 8; ++i) bk_coloff[i] = axis_off(G.b_col, (uint32_t)min(tn * BN + a_r0 + 32 * i, N - 1)) * 2;
  }

  // ---- the pieces of one K step, each small enough to be placed between two MFMAs ----------
  uint4 ra[8], rb[8];
  uint32_t g_aco = 0;            // column offset of this thread's A chunk for the tile being fetched
  const char* g_bp = nullptr;    // first of this thread's 8 B rows for the tile being fetched
  // Chunks past K (only when K is not a multiple of 64: the K_TAIL instantiation) read a
  // clamped, valid address and are zeroed when they are written to LDS.  Columns past N need no
  // masking: they only feed C columns that are never stored.
  const int nk = (K + BK - 1) / BK;
  const bool tabulated = !K_TAIL && G.k64 && nk <= kMaxSteps;
  if (tabulated) {
    for (int st = t; st < nk; st += 256) {
      step_a[st] = (uint32_t)(axis_off(G.a_col, (uint32_t)(st * BK)) * 2);
      step_b[st] = axis_off(G.b_row, (uint32_t)(st * BK)) * 2;
    }
    __syncthreads();
  }
  const uint32_t a_lane = (uint32_t)(a_c * 16);
  const char* b_lane = B_KMAJOR ? G.b + a_c * 16 : b_colptr + (int64_t)(b_kb * 8) * b_kstride;
  uint32_t t_a = 0;              // table entries of the step about to be fetched, read well ahead of their use
  int64_t t_b = 0;
  auto gload_lookup = [&](int k0) {
    if (tabulated) {
      t_a = step_a[k0 / BK];
      t_b = step_b[k0 / BK];
    }
  };
  auto gload_prepare = [&](int k0) {
    if (tabulated) {
      // a K step of 64 stays inside the innermost K digit of both operands: step offset + lane constant
      g_aco = t_a + a_lane;
      g_bp = b_lane + t_b;
    } else {
      const int ka = k0 + a_c * 8, kb = B_KMAJOR ? ka : k0 + b_kb * 8;
      g_aco = (uint32_t)(axis_off(G.a_col, (uint32_t)(K_TAIL ? min(ka, K - 8) : ka)) * 2);
      g_bp = (B_KMAJOR ? G.b : b_colptr) + axis_off(G.b_row, (uint32_t)(K_TAIL ? min(kb, K - 8) : kb)) * 2;
    }
  };
  auto gload_a = [&](int i) { ra[i] = *reinterpret_cast<const uint4*>(G.a + (a_rowoff[i] + g_aco)); };
  auto gload_b = [&](int j) {
    if (B_KMAJOR) rb[j] = *reinterpret_cast<const uint4*>(g_bp + bk_coloff[j]);
    else rb[j] = *reinterpret_cast<const uint4*>(g_bp + j * b_kstride);
  };
  auto store_a = [&](int buf, int i, int k0) {
    const int r = a_r0 + 32 * i;
    uint4 v = ra[i];
    if (K_TAIL && k0 + a_c * 8 >= K) v = make_uint4(0, 0, 0, 0);
    ldsA[buf][r * 8 + (a_c ^ (r & 7))] = v;
  };
  // row j of the thread's 8 (k) x 8 (n) block of B goes to LDS as it is (16 bytes, n contiguous);
  // the transposition the matrix core needs happens in the LDS read (ds_read_b64_tr_b16)
  auto store_b = [&](int buf, int j, int k0) {
    uint4 v = rb[j];
    if (B_KMAJOR) {
      // [n][8 chunks of 8 k], swizzled like A's tile
      const int r = a_r0 + 32 * j;
      if (K_TAIL && k0 + a_c * 8 >= K) v = make_uint4(0, 0, 0, 0);
      reinterpret_cast<uint4*>(&ldsB[buf][0])[r * 8 + (a_c ^ (r & 7))] = v;
      return;
    }
    if (K_TAIL && k0 + b_kb * 8 >= K) v = make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(&ldsB[buf][(b_kb * 8 + j) * kBPitch + b_cn * 16]) = v;
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // fragment addresses (16-byte units) for k-chunk 0; chunk c is reached by XOR with c
  int a_unit[4], a_key[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
    const int r = wm * 128 + mb * 32 + l32;
    a_unit[mb] = r * 8;
    a_key[mb] = r & 7;
  }
  // B fragments: a transposing LDS read hands lane i of a 16-lane group the 4 consecutive k of
  // column n0 + i when lane L of the group points at row k0 + (L >> 2), columns n0 + 4 (L & 3) .. + 3.
  // Lane group q = lane / 16: columns 16 (q & 1) .. + 15 of the 32-column block, k-half q >> 1.
  const int lq = lane >> 4, ll = lane & 15;
  const int b_lane_off = (8 * (lq >> 1) + (ll >> 2)) * kBPitch + (wn * 128 + 16 * (lq & 1) + 4 * (ll & 3)) * 2;
  opvec af[2][4], bf[2][4];
  // fragment f of k16 step ks (f = 0: A0, 1..4: B0..B3, 5..7: A1..A3: the order the MFMAs need them)
  auto read_frag = [&](int buf, int ks, int p, int f) {
    const int chunk = ks * 2 + lh;
    if (f == 0 || f >= 5) {
      const int mb = f == 0 ? 0 : f - 4;
      af[p][mb] = __builtin_bit_cast(opvec, ldsA[buf][a_unit[mb] + (chunk ^ a_key[mb])]);
    } else if (B_KMAJOR) {
      const int nb = f - 1;
      const int r = wn * 128 + nb * 32 + l32;
      bf[p][nb] = __builtin_bit_cast(opvec, reinterpret_cast<const uint4*>(&ldsB[buf][0])[r * 8 + (chunk ^ (r & 7))]);
    } else {
      const int nb = f - 1;
      typedef short s16x4 __attribute__((ext_vector_type(4)));
      typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
      const char* base = &ldsB[buf][b_lane_off + ks * 16 * kBPitch + nb * 64];
      struct { s16x4 lo, hi; } v;
      v.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(base));                  // k = 8 lh + 0..3
      v.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(base + 4 * kBPitch));    // k = 8 lh + 4..7
      bf[p][nb] = __builtin_bit_cast(opvec, v);
    }
  };
  auto mma = [&](int p, int m) { acc[m >> 2][m & 3] = M_::run(af[p][m >> 2], bf[p][m & 3], acc[m >> 2][m & 3]); };
#define VT_SB() __builtin_amdgcn_sched_barrier(0)

  // ---- one K step (64 MFMAs per wave).  Source order IS the issue order: each group between
  // two scheduling barriers holds two MFMAs and a little memory work that issues in the shadow
  // of the matrix pipe.  Global loads run two K steps ahead and are issued as soon as their
  // registers are free (A under k16 step 2, B under k16 step 3), three quarters of a K step
  // before the LDS stores that consume them (k16 steps 1 and 2 of the next K step); fragments are
  // read one k16 step ahead, and the only barrier comes before k16 step 3 so that the next
  // tile's first fragments are in flight under its MFMAs.
  auto k_step = [&](int it, auto do_store, auto do_load) {
    const int cur = it & 1, nxt = cur ^ 1;
    const int k_next = (it + 1) * BK;
    if (do_load.value) gload_lookup((it + 2) * BK);
#pragma unroll
    for (int i = 0; i < 8; ++i) {            // k16 step 0 | read fragments of step 1
      mma(0, 2 * i);
      read_frag(cur, 1, 1, i);
      mma(0, 2 * i + 1);
      VT_SB();
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {            // k16 step 1 | fragments of step 2, A tile of the next K step -> LDS
      mma(1, 2 * i);
      read_frag(cur, 2, 0, i);
      mma(1, 2 * i + 1);
      if (do_store.value) store_a(nxt, i, k_next);
      VT_SB();
    }
    if (do_load.value) gload_prepare((it + 2) * BK);
#pragma unroll
    for (int i = 0; i < 8; ++i) {            // k16 step 2 | fragments of step 3, B tile -> LDS, A rows two K steps ahead
      mma(0, 2 * i);
      read_frag(cur, 3, 1, i);
      if (do_load.value) gload_a(i);         // the A registers are free again: their tile went to LDS in k16 step 1
      mma(0, 2 * i + 1);
      if (do_store.value) store_b(nxt, i, k_next);
      VT_SB();
    }
    __syncthreads();
    VT_SB();
#pragma unroll
    for (int i = 0; i < 8; ++i) {            // k16 step 3 | first fragments of the next tile, B rows two K steps ahead
      mma(1, 2 * i);
      if (do_store.value) read_frag(nxt, 0, 0, i);
      mma(1, 2 * i + 1);
      if (do_load.value) gload_b(i);
      VT_SB();
    }
  };

  gload_lookup(0);
  gload_prepare(0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    gload_a(i);
    gload_b(i);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    store_a(0, i, 0);
    store_b(0, i, 0);
  }
  if (nk > 1) {
    gload_lookup(BK);
    gload_prepare(BK);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      gload_a(i);
      gload_b(i);
    }
  }
  __syncthreads();
  VT_PROF(1);
  VT_PROF_CYCLES(4);
#pragma unroll
  for (int f = 0; f < 8; ++f) read_frag(0, 0, 0, f);
  int it = 0;
  for (; it + 2 < nk; ++it) k_step(it, std::true_type{}, std::true_type{});
  if (it + 1 < nk) {
    k_step(it, std::true_type{}, std::false_type{});
    ++it;
  }
  k_step(it, std::false_type{}, std::false_type{});
#undef VT_SB
  VT_PROF(2);
  VT_PROF_CYCLES(5);

  if (MAPPED) {
    // ---- stage 3 through the output map.  The row part of the map is evaluated once per row of
    // the tile (one thread each, per piece) and parked in LDS, which the K loop no longer needs;
    // the column part once per lane and column block.
    __syncthreads();
    int64_t* rowoff = reinterpret_cast<int64_t*>(&ldsA[0][0]);       // [pieces][BM]
    for (int pc = 0; pc < O.n; ++pc) rowoff[pc * BM + t] = axis_off(O.p[pc].row, (uint32_t)min(tm * BM + t, Mg - 1));
    __syncthreads();
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int col = tn * BN + wn * 128 + nb * 32 + l32;
      if (col >= N) continue;
      int pc = 0;
#pragma unroll
      for (int i = 1; i < 4; ++i)
        if (i < O.n && col >= O.p[i].col_lo) pc = i;
      T* base = reinterpret_cast<T*>(O.p[pc].base) + axis_off(O.p[pc].col, (uint32_t)(col - O.p[pc].col_lo));
      const int64_t* ro = rowoff + pc * BM;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        const int r0 = wm * 128 + mb * 32 + lh * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (tm * BM + r0 + 8 * j + i < Mg) base[ro[r0 + 8 * j + i]] = from_float<T>(acc[mb][nb][4 * j + i]);
      }
    }
    return;
  }
  // ---- stage 3: plain contiguous store of the tile (lanes 0..31 write 32 consecutive columns)
  typedef typename std::conditional<C_F32, float, T>::type CT;
  CT* cbase = reinterpret_cast<CT*>(G.c);
  const bool full = (tm + 1) * BM <= Mg && (tn + 1) * BN <= N;
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int col = tn * BN + wn * 128 + nb * 32 + l32;
      const int row0 = tm * BM + wm * 128 + mb * 32 + lh * 4;
      CT* cp = cbase + (size_t)row0 * N + col;
      if (full) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i) cp[(size_t)(8 * j + i) * N] = from_float<CT>(acc[mb][nb][4 * j + i]);
      } else if (col < N) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (row0 + 8 * j + i < Mg) cp[(size_t)(8 * j + i) * N] = from_float<CT>(acc[mb][nb][4 * j + i]);
      }
    }
#ifdef VT_PROFILE
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  VT_PROF(3);
  VT_PROF_FLUSH(gemm, blockIdx.x);
#endif
}

// ------------------------------------------------------------------------------------------
// The same product for ANY pair of maps the descriptor can hold (pieces along K, stacked index
// stages, tables anywhere, no contiguity at all): every element of A and B is found through the
// generic evaluator, staged in LDS with the contraction index contiguous, and multiplied on the
// matrix cores.  Correct for every representable chain, and slow (one evaluation per element):
// the tiled kernel above takes over whenever the maps have its separable form.
// 64 x 64 tile per workgroup, one 32 x 32 block per wave, K in steps of 16.
// ------------------------------------------------------------------------------------------
// LN: per-row LayerNorm over K (gamma 1, beta 0, biased variance, fp32, two passes) applied to A,
// rounded to the operand type, before the product.
template <typename T, bool C_F32, bool LN>
__global__ void __launch_bounds__(256) k_gemm_generic(const DevDesc A_, const DevDesc B_, void* __restrict__ Cout, int M, int N, int K, float eps) {
  typedef Mma<T> M_;
  typedef typename M_::vec opvec;
  __shared__ __attribute__((aligned(16))) T la[64][24];      // [row][k], 16 k used, pitch 48 bytes
  __shared__ __attribute__((aligned(16))) T lb[64][24];      // [col][k]
  __shared__ DevDesc maps[2];                                // the evaluator reads the maps from LDS
  {
    const DevDesc* const from[2] = {&A_, &B_};
    stage_maps(maps, from);
  }
  const DevDesc& A = maps[0];
  const DevDesc& B = maps[1];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  float mean = 0.f, rstd = 1.f;                      // of row t / 4 (the four threads of a row agree)
  if (LN) {
    const int m = min(m0 + (t >> 2), M - 1);
    auto a_at = [&](int k) {
      int64_t off;
      const void* ptr;
      vtd_eval(A, 0, (uint32_t)m * (uint32_t)K + (uint32_t)k, &off, &ptr);
      return to_float(static_cast<const T*>(ptr)[off]);
    };
    float s1 = 0.f;
    for (int k = t & 3; k < K; k += 4) s1 += a_at(k);
    s1 += __shfl_xor(s1, 1, 64);
    s1 += __shfl_xor(s1, 2, 64);
    mean = s1 / (float)K;
    float s2 = 0.f;
    for (int k = t & 3; k < K; k += 4) {
      const float dlt = a_at(k) - mean;
      s2 += dlt * dlt;
    }
    s2 += __shfl_xor(s2, 1, 64);
    s2 += __shfl_xor(s2, 2, 64);
    rstd = 1.0f / sqrtf(s2 / (float)K + eps);
  }
  for (int k0 = 0; k0 < K; k0 += 16) {
    {  // A: thread -> row t / 4, k = (t % 4) * 4 .. + 3
      const int r = t >> 2, m = min(m0 + r, M - 1);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int k = k0 + (t & 3) * 4 + i;
        T v = from_float<T>(0.f);
        if (k < K) {
          int64_t off;
          const void* ptr;
          vtd_eval(A, 0, (uint32_t)m * (uint32_t)K + (uint32_t)k, &off, &ptr);
          v = static_cast<const T*>(ptr)[off];
          if (LN) v = from_float<T>((to_float(v) - mean) * rstd);
        }
        la[r][(t & 3) * 4 + i] = v;
      }
    }
    {  // B: thread -> k = t / 16, n = (t % 16) * 4 .. + 3, written transposed
      const int kk = t >> 4, k = k0 + kk;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = (t & 15) * 4 + i, n = min(n0 + c, N - 1);
        T v = from_float<T>(0.f);
        if (k < K) {
          int64_t off;
          const void* ptr;
          vtd_eval(B, 0, (uint32_t)k * (uint32_t)N + (uint32_t)n, &off, &ptr);
          v = static_cast<const T*>(ptr)[off];
        }
        lb[c][kk] = v;
      }
    }
    __syncthreads();
    const opvec af = *reinterpret_cast<const opvec*>(&la[wm * 32 + l32][lh * 8]);
    const opvec bf = *reinterpret_cast<const opvec*>(&lb[wn * 32 + l32][lh * 8]);
    acc = M_::run(af, bf, acc);
    __syncthreads();
  }
  typedef typename std::conditional<C_F32, float, T>::type CT;
  CT* c = static_cast<CT*>(Cout);
  const int col = n0 + wn * 32 + l32;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = m0 + wm * 32 + lh * 4 + 8 * j + i;
      if (row < M && col < N) c[(size_t)row * N + col] = from_float<CT>(acc[4 * j + i]);
    }
}

}  // namespace

namespace vt {
int launch_generic(const vt_desc& a, const vt_desc& b, void* c, int c_dtype, bool layernorm, float eps, hipStream_t st) {
  const int n = (int)a.shape.size();
  if (n < 2 || b.shape.size() != 2) return fail(VT_ERR_SHAPE, "vt_gemm: A must be [.., K] and B [K, N]");
  int64_t M = 1;
  for (int i = 0; i < n - 1; ++i) M *= a.shape[i];
  const int64_t K = a.shape[n - 1], N = b.shape[1];
  if (b.shape[0] != K) return fail(VT_ERR_SHAPE, "vt_gemm: inner dims of A and B differ");
  DevDesc DA, DB;
  int64_t oa, ia, ob, ib;
  int rc = to_device(a, &DA, &oa, &ia);
  if (rc != VT_OK) return rc;
  rc = to_device(b, &DB, &ob, &ib);
  if (rc != VT_OK) return rc;
  if (oa != 1 || ob != 1 || M > 65535ll * 64 || N > 65535ll * 64) return fail(VT_ERR_UNSUPPORTED, "vt_gemm: operand too large for the generic path");
  dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
#define VT_GENERIC(TT, CF)                                                                                          \
  do {                                                                                                              \
    if (layernorm) hipLaunchKernelGGL((k_gemm_generic<TT, CF, true>), grid, dim3(256), 0, st, DA, DB, c, (int)M, (int)N, (int)K, eps); \
    else hipLaunchKernelGGL((k_gemm_generic<TT, CF, false>), grid, dim3(256), 0, st, DA, DB, c, (int)M, (int)N, (int)K, eps);          \
  } while (0)
  if (a.dtype == VT_BF16) {
    if (c_dtype == VT_F32) VT_GENERIC(bf16_t, true);
    else VT_GENERIC(bf16_t, false);
  } else {
    if (c_dtype == VT_F32) VT_GENERIC(f16_t, true);
    else VT_GENERIC(f16_t, false);
  }
#undef VT_GENERIC
  return check_launch("vt_gemm (generic maps)");
}
}  // namespace vt

namespace {

// Piece `pi` of A as one operand of its own: a Concat along the rows makes A a stack of pieces,
// each of which is a range of rows [*row_begin, *row_begin + *M) of the product.
int plan_a(const vt_desc& d, GemmGroup* g, int64_t* M, int64_t* K, size_t pi = 0, int64_t* row_begin = nullptr) {
  int n = (int)d.shape.size();
  if (n < 2) return fail(VT_ERR_SHAPE, "vt_gemm: A must have at least 2 dims");
  if (pi >= d.pieces.size() || !d.pieces[pi].v.lower.empty())
    return fail(VT_ERR_UNSUPPORTED, "vt_gemm: A must have one index stage");
  const Piece& p = d.pieces[pi];
  *K = d.shape[n - 1];
  *M = 1;
  int64_t inner_rows = 1;
  for (int i = n - 2; i >= 0; --i) {
    *M *= p.hi[i] - p.lo[i];
    if (i > 0) {
      if (p.lo[i] != 0 || p.hi[i] != d.shape[i]) return fail(VT_ERR_UNSUPPORTED, "vt_gemm: the pieces of A must be ranges of rows (a Concat along the outermost dim)");
      inner_rows *= d.shape[i];
    }
  }
  if (p.lo[n - 1] != 0 || p.hi[n - 1] != d.shape[n - 1]) return fail(VT_ERR_UNSUPPORTED, "vt_gemm: A is cut into pieces along K");
  if (row_begin) *row_begin = p.lo[0] * inner_rows;
  else if (d.pieces.size() != 1) return fail(VT_ERR_UNSUPPORTED, "vt_gemm: A must be a single piece here");
  int rc = make_axis(d, p, 0, n - 1, &g->a_row, "vt_gemm: A rows", true);
  if (rc != VT_OK) return rc;
  rc = make_axis(d, p, n - 1, n, &g->a_col, "vt_gemm: A columns");
  if (rc != VT_OK) return rc;
  const vt_source& src = d.sources[p.src];
  if (!src.ptr) return fail(VT_ERR_INVALID_ARG, "vt_gemm: A source without a device pointer");
  g->a = static_cast<const char*>(src.ptr) + p.v.base * 2;
  {
    int64_t span = 0;
    for (int i = 0; i < 5; ++i) span += (int64_t)(g->a_row.radix[i].d - 1) * g->a_row.stride[i];
    for (int i = 0; i < 3; ++i) span += (int64_t)(g->a_col.radix[i].d - 1) * g->a_col.stride[i];
    if (g->a_row.table) {
      // a table digit can reach any row of the source dim it indexes: bound by the source size
      span = 1;
      for (int i = 0; i < src.ndim; ++i) span *= src.shape[i];
    }
    if (span * 2 >= (1ll << 32)) return fail(VT_ERR_UNSUPPORTED, "vt_gemm: A spans 4 GiB or more");
  }
  const AxisMap<3>& c = g->a_col;
  bool ok = *K % 8 == 0 && (uintptr_t)g->a % 16 == 0 && strides_multiple_of(g->a_row, 8, 0);
  ok = ok && c.nd >= 1 && c.stride[2] == 1 && c.radix[2].d % 8 == 0 && strides_multiple_of(c, 8, 1);
  if (!ok) return fail(VT_ERR_UNSUPPORTED, "vt_gemm: A needs runs of 8 contiguous, 16-byte aligned elements along K");
  return VT_OK;
}

int plan_b(const vt_desc& d, GemmGroup* g, int64_t* K, int64_t* N) {
  if (d.shape.size() != 2) return fail(VT_ERR_SHAPE, "vt_gemm: B must be [K,N]");
  if (d.pieces.size() != 1 || !d.pieces[0].v.lower.empty())
    return fail(VT_ERR_UNSUPPORTED, "vt_gemm: B must be a single piece with one index stage");
  const Piece& p = d.pieces[0];
  *K = d.shape[0];
  *N = d.shape[1];
  int rc = make_axis(d, p, 0, 1, &g->b_row, "vt_gemm: B rows");
  if (rc != VT_OK) return rc;
  rc = make_axis(d, p, 1, 2, &g->b_col, "vt_gemm: B columns");
  if (rc != VT_OK) return rc;
  const vt_source& src = d.sources[p.src];
  if (!src.ptr) return fail(VT_ERR_INVALID_ARG, "vt_gemm: B source without a device pointer");
  g->b = static_cast<const char*>(src.ptr) + p.v.base * 2;
  const AxisMap<3>& c = g->b_col;
  const AxisMap<3>& r = g->b_row;
  g->b_kmajor = 0;
  bool ok = *N % 8 == 0 && *K % 8 == 0 && r.radix[2].d % 8 == 0 && (uintptr_t)g->b % 16 == 0 &&
            strides_multiple_of(r, 8, 0) && c.nd >= 1 &&
            c.stride[2] == 1 && c.radix[2].d % 8 == 0 && strides_multiple_of(c, 8, 1);
  if (ok) return VT_OK;
  // K contiguous instead (an [N,K] weight through a Permute): runs of 8 along K, everything else 16-byte aligned
  ok = *K % 8 == 0 && (uintptr_t)g->b % 16 == 0 && r.nd >= 1 && r.stride[2] == 1 && r.radix[2].d % 8 == 0 &&
       strides_multiple_of(r, 8, 1) && strides_multiple_of(c, 8, 0);
  if (ok) {
    g->b_kmajor = 1;
    return VT_OK;
  }
  return fail(VT_ERR_UNSUPPORTED, "vt_gemm: B needs runs of 8 contiguous, 16-byte aligned elements along N or along K");
}

}  // namespace

namespace vt {
int ln_gemm_launch(const vt_desc& A, const vt_desc& B, void* C, int c_dtype, float eps, hipStream_t st);
}

namespace vt {

// C = A . B with the result written through the output descriptor Cd (pieces split the columns;
// the caller has checked that the map is one to one).  One group, operands' dtype for the output.
int gemm_store_launch(const vt_desc& A, const vt_desc& B, const vt_desc& Cd, hipStream_t st) {
  const int dt = A.dtype;
  GemmParams P;
  memset(&P, 0, sizeof(P));
  int64_t M, Ka, Kb, N;
  int rc = plan_a(A, &P.g[0], &M, &Ka);
  if (rc != VT_OK) return rc;
  rc = plan_b(B, &P.g[0], &Kb, &N);
  if (rc != VT_OK) return rc;
  if (Ka != Kb) return fail(VT_ERR_SHAPE, "vt_gemm_store: inner dims of A and B differ");
  if (P.g[0].b_kmajor) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: B must be row-major [K,N]");
  if (M >= (1ll << 31) || N >= (1ll << 31) || Ka >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: extents too large");
  OutMap O;
  memset(&O, 0, sizeof(O));
  if (Cd.pieces.size() > 4) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: more than 4 output pieces");
  std::vector<const Piece*> ps;
  for (const Piece& p : Cd.pieces) ps.push_back(&p);
  std::sort(ps.begin(), ps.end(), [](const Piece* x, const Piece* y) { return x->lo[1] < y->lo[1]; });
  int64_t expect = 0;
  for (size_t i = 0; i < ps.size(); ++i) {
    const Piece& p = *ps[i];
    if (p.lo[0] != 0 || p.hi[0] != M || p.lo[1] != expect) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: output pieces must split the columns only");
    expect = p.hi[1];
    rc = make_axis(Cd, p, 0, 1, &O.p[i].row, "vt_gemm_store: output rows");
    if (rc != VT_OK) return rc;
    rc = make_axis(Cd, p, 1, 2, &O.p[i].col, "vt_gemm_store: output columns");
    if (rc != VT_OK) return rc;
    const vt_source& s = Cd.sources[p.src];
    if (!s.ptr) return fail(VT_ERR_INVALID_ARG, "vt_gemm_store: output tensor without a device pointer");
    O.p[i].base = static_cast<char*>(s.ptr) + p.v.base * 2;
    O.p[i].col_lo = (int32_t)p.lo[1];
    O.p[i].col_hi = (int32_t)p.hi[1];
  }
  if (expect != N) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: output pieces do not cover the columns");
  O.n = (int32_t)ps.size();
  P.g[0].c = nullptr;
  P.g[0].M = (int32_t)M;
  P.g[0].tiles_m = (int32_t)((M + BM - 1) / BM);
  P.g[0].tile_begin = 0;
  P.g[0].k64 = P.g[0].a_col.radix[2].d % 64 == 0 && P.g[0].b_row.radix[2].d % 64 == 0;
  P.n_groups = 1;
  P.N = (int32_t)N;
  P.K = (int32_t)Ka;
  P.tiles_n = (int32_t)((N + BN - 1) / BN);
  P.total_tiles = P.g[0].tiles_m * P.tiles_n;
  P.chunk = (P.total_tiles + 7) / 8;
  dim3 grid(P.chunk * 8);
  const bool kt = Ka % BK != 0;
  if (dt == VT_BF16) {
    if (kt) hipLaunchKernelGGL((k_gemm<bf16_t, false, true, true>), grid, dim3(256), 0, st, P, O);
    else hipLaunchKernelGGL((k_gemm<bf16_t, false, false, true>), grid, dim3(256), 0, st, P, O);
  } else {
    if (kt) hipLaunchKernelGGL((k_gemm<f16_t, false, true, true>), grid, dim3(256), 0, st, P, O);
    else hipLaunchKernelGGL((k_gemm<f16_t, false, false, true>), grid, dim3(256), 0, st, P, O);
  }
  return check_launch("vt_gemm_store");
}

}  // namespace vt

extern "C" int vt_gemm(const vt_desc* const* A, const vt_desc* const* B, void* const* C, int n_groups, int c_dtype,
                       int prologue, float eps, void* stream) {
  if (!A || !B || !C || n_groups < 1) return fail(VT_ERR_INVALID_ARG, "vt_gemm: NULL argument");
  if (prologue != VT_GEMM_PLAIN && prologue != VT_GEMM_LAYERNORM) return fail(VT_ERR_INVALID_ARG, "vt_gemm: unknown prologue");
  const int dt = A[0] ? A[0]->dtype : -1;
  if (dt != VT_BF16 && dt != VT_F16) return fail(VT_ERR_INVALID_ARG, "vt_gemm: operands must be f16 or bf16");
  if (c_dtype != dt && c_dtype != VT_F32) return fail(VT_ERR_INVALID_ARG, "vt_gemm: C must have the operand dtype or f32");
  hipStream_t st = (hipStream_t)stream;
  if (prologue == VT_GEMM_LAYERNORM) {
    for (int i = 0; i < n_groups; ++i) {
      if (!A[i] || !B[i] || !C[i]) return fail(VT_ERR_INVALID_ARG, "vt_gemm: NULL descriptor or output");
      if (A[i]->dtype != dt || B[i]->dtype != dt) return fail(VT_ERR_INVALID_ARG, "vt_gemm: mixed operand dtypes");
      int rc = ln_gemm_launch(*A[i], *B[i], C[i], c_dtype, eps, st);
      // shapes or maps the fused kernel is not built for: the generic kernel with the same prologue
      if (rc == VT_ERR_UNSUPPORTED) rc = launch_generic(*A[i], *B[i], C[i], c_dtype, true, eps, st);
      if (rc != VT_OK) return rc;
    }
    return VT_OK;
  }
  // Can the tiled kernel take every operand?  If a map lacks the separable form it needs (and only
  // then: wrong arguments are still errors), the whole call runs on the generic kernel, group by group.
  {
    bool generic = false;
    for (int i = 0; i < n_groups && !generic; ++i) {
      if (!A[i] || !B[i] || !C[i]) return fail(VT_ERR_INVALID_ARG, "vt_gemm: NULL descriptor or output");
      if (A[i]->dtype != dt || B[i]->dtype != dt) return fail(VT_ERR_INVALID_ARG, "vt_gemm: mixed operand dtypes");
      GemmGroup probe;
      int64_t m_, k_, n_, rb_;
      for (size_t pi = 0; pi < A[i]->pieces.size() && !generic; ++pi) generic = plan_a(*A[i], &probe, &m_, &k_, pi, &rb_) == VT_ERR_UNSUPPORTED;
      generic = generic || plan_b(*B[i], &probe, &k_, &n_) == VT_ERR_UNSUPPORTED;
    }
    if (generic) {
      for (int i = 0; i < n_groups; ++i) {
        int rc = launch_generic(*A[i], *B[i], C[i], c_dtype, false, 0.f, st);
        if (rc != VT_OK) return rc;
      }
      return VT_OK;
    }
  }
  int64_t N = -1, K = -1;
  // one unit of the launch per (group, piece of its A): a Concat along the rows of A is executed as
  // a grouped launch, every piece writing its own range of rows of C
  struct Unit {
    int group;
    size_t piece;
  };
  std::vector<Unit> units;
  for (int i = 0; i < n_groups; ++i) {
    if (!A[i] || !B[i] || !C[i]) return fail(VT_ERR_INVALID_ARG, "vt_gemm: NULL descriptor or output");
    for (size_t pi = 0; pi < A[i]->pieces.size(); ++pi) units.push_back({i, pi});
  }
  for (size_t u0 = 0; u0 < units.size(); u0 += kMaxGroups) {
    GemmParams P;
    memset(&P, 0, sizeof(P));
    const int ng = (int)std::min<size_t>(kMaxGroups, units.size() - u0);
    int tiles = 0;
    for (int i = 0; i < ng; ++i) {
      const vt_desc* a = A[units[u0 + i].group];
      const vt_desc* b = B[units[u0 + i].group];
      void* c = C[units[u0 + i].group];
      if (a->dtype != dt || b->dtype != dt) return fail(VT_ERR_INVALID_ARG, "vt_gemm: mixed operand dtypes");
      int64_t M, Ka, Kb, Nb, row_begin = 0;
      int rc = plan_a(*a, &P.g[i], &M, &Ka, units[u0 + i].piece, &row_begin);
      if (rc != VT_OK) return rc;
      rc = plan_b(*b, &P.g[i], &Kb, &Nb);
      if (rc != VT_OK) return rc;
      if (Ka != Kb) return fail(VT_ERR_SHAPE, "vt_gemm: inner dims of A and B differ");
      if (N < 0) {
        N = Nb;
        K = Ka;
      }
      if (Nb != N || Ka != K) return fail(VT_ERR_SHAPE, "vt_gemm: all groups must share K and N");
      if (M >= (1ll << 31) || N >= (1ll << 31) || K >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, "vt_gemm: extents too large");
      if ((uintptr_t)c % 4) return fail(VT_ERR_INVALID_ARG, "vt_gemm: misaligned C");
      P.g[i].c = static_cast<char*>(c) + (size_t)row_begin * (size_t)N * (c_dtype == VT_F32 ? 4 : 2);
      P.g[i].M = (int32_t)M;
      P.g[i].tiles_m = (int32_t)((M + BM - 1) / BM);
      P.g[i].tile_begin = tiles;
      P.g[i].k64 = P.g[i].a_col.radix[2].d % 64 == 0 && P.g[i].b_row.radix[2].d % 64 == 0;
      if (P.g[i].b_kmajor != P.g[0].b_kmajor) return fail(VT_ERR_UNSUPPORTED, "vt_gemm: the groups of one call must store B the same way (all [K,N] or all [N,K])");
      tiles += P.g[i].tiles_m * (int32_t)((N + BN - 1) / BN);
    }
    P.n_groups = ng;
    P.N = (int32_t)N;
    P.K = (int32_t)K;
    P.tiles_n = (int32_t)((N + BN - 1) / BN);
    P.total_tiles = tiles;
    P.chunk = (tiles + 7) / 8;
    P.c_f32 = c_dtype == VT_F32;
    dim3 grid(P.chunk * 8);
    const bool kt = K % BK != 0;
    OutMap no_map;
    memset(&no_map, 0, sizeof(no_map));
#define VT_GEMM_LAUNCH(TT, CF, KT)                                                                              \
  do {                                                                                                          \
    if (P.g[0].b_kmajor) hipLaunchKernelGGL((k_gemm<TT, CF, KT, false, true>), grid, dim3(256), 0, st, P, no_map); \
    else hipLaunchKernelGGL((k_gemm<TT, CF, KT, false, false>), grid, dim3(256), 0, st, P, no_map);             \
  } while (0)
    if (dt == VT_BF16) {
      if (P.c_f32) { if (kt) VT_GEMM_LAUNCH(bf16_t, true, true); else VT_GEMM_LAUNCH(bf16_t, true, false); }
      else { if (kt) VT_GEMM_LAUNCH(bf16_t, false, true); else VT_GEMM_LAUNCH(bf16_t, false, false); }
    } else {
      if (P.c_f32) { if (kt) VT_GEMM_LAUNCH(f16_t, true, true); else VT_GEMM_LAUNCH(f16_t, true, false); }
      else { if (kt) VT_GEMM_LAUNCH(f16_t, false, true); else VT_GEMM_LAUNCH(f16_t, false, false); }
    }
#undef VT_GEMM_LAUNCH
    int rc = check_launch("vt_gemm");
    if (rc != VT_OK) return rc;
  }
  return VT_OK;
}
