// LayerNorm fused into the load stage of a skinny GEMM: C = LN(A) . W with A virtual [.., K],
// K = 64 or 128, W virtual [K, N], N <= 384 (the window-partition -> LayerNorm -> linear chain).
// The whole path is bound by HBM (the output is 3x the input), so the design goal is to touch
// every byte once and to keep enough waves resident to hide latency: the normalised tokens never
// exist in global memory, and W never leaves registers.
//
// A persistent workgroup of 8 waves (two per SIMD) walks over blocks of 64 rows.  Each wave owns
// N/8 output columns (up to 48) and keeps its slice of W in registers for the whole kernel as
// v_mfma_f32_16x16x32 operands.  Stage 1 through the map: 16 (K=128) or 8 (K=64) lanes fetch one
// row with 16-byte loads at row_offset(m) (mixed-radix digits / index table; one lane evaluates a
// row and hands the offset to the lanes that load it); the same lanes reduce mean and variance
// with DPP row operations, normalise in fp32, round to the operand type and write the row into
// an XOR-swizzled LDS tile; rows of the next two blocks are in flight while the current block is
// multiplied.  The product is formed transposed (W^T as the first operand), so a lane ends up
// with 4 consecutive output columns; stage 3 packs them, bounces the wave's 64 x N/8 sub-tile
// through LDS and leaves with 16-byte stores (the output is three quarters of all traffic).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <type_traits>

#include "vt_gemm_common.h"
#include "vt_profile.h"

using namespace vt;
using namespace vt::gemm;

// profile marks (LDS writes: they are not among the vector memory operations the waits below count):
// 0 start, 1 first two blocks requested, 2 W in registers, 3 first block multiplied, 4 last block
// multiplied, 5 last stores issued, 6 all memory operations complete, 7 compute die
VT_PROF_DECLARE(ln_gemm)

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T>
struct Mma16;
template <>
struct Mma16<bf16_t> {
  typedef bf16x8 vec;
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};
template <>
struct Mma16<f16_t> {
  typedef f16x8 vec;
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int LBM = 64;           // rows per block
constexpr int LWAVES = 8;
constexpr int LTHREADS = LWAVES * 64;

struct LnGemmParams {
  const char* a;
  const char* b;
  char* c;
  AxisMap<5> a_row;
  AxisMap<3> b_row, b_col;
  int32_t M, N, K;
  int32_t n_full;        // rounds of full blocks: in round i workgroup w takes block i * gridDim.x + w
  int32_t tail_rows;     // then rows [tail0 + w * tail_rows, + tail_rows) of what is left, tail0 = n_full * gridDim.x * LBM
  float eps;
  int32_t w_rows_of_8;   // W has runs of 8 contiguous, 16-byte aligned elements along N: coalesced prologue
  int32_t w_k_runs_of_8; // rows 8i .. 8i+7 of W are equally spaced (innermost K digit has a radix that 8 divides)
  FastDiv n8, nblk;      // N / 8 and (N / 8) * (K / 8): divisors of the W prologue
};

// LPR = lanes per row = K / 8; NB = 16-column blocks per wave
template <typename T, bool C_F32, int LPR, int NB>
__global__ void __launch_bounds__(LTHREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_ln_gemm(const LnGemmParams P) {
  typedef Mma16<T> M_;
  typedef typename M_::vec opvec;
  constexpr int K = LPR * 8;
  constexpr int KS = K / 32;                 // k32 steps
  constexpr int RPP = LTHREADS / LPR;        // rows staged per pass of the workgroup
  constexpr int PASSES = LBM / RPP;
  constexpr int CW = NB * 16;                // output columns per wave
  constexpr int kTileUnits = LBM * LPR;      // 16-byte units of one A tile
  constexpr int CPW = LWAVES * CW * 2 + 16;  // bytes per row of the staged C tile (16 more than a row: de-phased banks)
  constexpr int kTilesBytes = 3 * kTileUnits * 16, kCBytes = C_F32 ? 0 : 2 * LBM * CPW, kWBytes = LWAVES * CW * K * 2;
  constexpr int kRegion0 = kCBytes > kWBytes ? kCBytes : kWBytes;   // W^T during the prologue, then the C tiles
  constexpr int kLdsBytes = kRegion0 + kTilesBytes;
  __shared__ __attribute__((aligned(16))) char lds_raw[kLdsBytes];
  // Steady state: two C tiles [row][N] (16-bit outputs only; during the prologue their memory holds
  // W^T) and three A tiles [row][LPR chunks of 8 k] (chunk c of row r at r*LPR + (c ^ (r & 7))), which
  // W^T never overlaps: the first rows are already arriving while W is transposed.
  // A tile goes through three states in place: rows arriving from global memory (requested two
  // blocks ahead, global -> LDS without touching registers, already in the swizzled order: the lane
  // that lands at position p of row r asks for chunk p ^ (r & 7)); normalised (each lane reads
  // back exactly the 16 bytes its own request delivered, so this needs no barrier, and writes the
  // result to the same place); multiplied.
  uint4* tiles = reinterpret_cast<uint4*>(lds_raw + kRegion0);
  char* cstage = lds_raw;
  VT_PROF_BEGIN();
  VT_PROF(0);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int M = P.M, N = P.N;

  // ---- stage 1 bookkeeping.  LPR lanes share a row.  A wave stages 8 rows of every block; their
  // offsets are evaluated through the map for 8 blocks at a time (lane: block lane/8 of the batch,
  // row lane%8) and handed to the lanes that load them.
  const int a_c = t % LPR, a_r0 = t / LPR;             // chunk and first row; rows a_r0 + RPP * i
  constexpr int RW = 64 / LPR;                          // rows per wave and pass
  static_assert(RW * PASSES == 8, "a wave stages 8 rows per block");
  // This workgroup's blocks.  Rounds of full blocks are interleaved over the workgroups, so that at
  // any moment the chip reads and writes one compact window of memory (contiguous ranges per
  // workgroup, 256 separate streams, measured 10% slower); the rows left after the last full round
  // are dealt out in shares of tail_rows.
  const int n_full = P.n_full, wg = blockIdx.x;
  const int64_t tail0 = (int64_t)n_full * gridDim.x * LBM + (int64_t)wg * P.tail_rows;
  const int n_it = n_full + (tail0 < M ? 1 : 0);
  if (n_it == 0) return;
  auto block_rows = [&](int i, int64_t* first, int64_t* end) {   // rows [first, end) of this workgroup's block i
    if (i < n_full) {
      *first = ((int64_t)i * gridDim.x + wg) * LBM;
      *end = *first + LBM;
    } else {
      *first = tail0;
      *end = min((int64_t)M, tail0 + P.tail_rows);
    }
  };
  const int ev_row = wave * RW + (lane & 7) % RW + RPP * ((lane & 7) / RW);
  uint32_t ro32 = 0;                                    // byte offset of this lane's row (the host checks that A spans < 4 GiB)
  auto eval_rows = [&](int it0) {                       // blocks it0 .. it0+7 of this workgroup
    int64_t first, end;
    block_rows(min(it0 + (lane >> 3), n_it - 1), &first, &end);   // past the last block: it again, not used
    const int m = (int)min(first + ev_row, end - 1);
    const int64_t ro = P.a_row.tdig >= 0 ? axis_off_table(P.a_row, (uint32_t)m) : axis_off(P.a_row, (uint32_t)m);
    ro32 = (uint32_t)(ro * 2);
  };
  typedef __attribute__((address_space(3))) void* lptr_t;
  auto load_rows = [&](int j, int slot) {               // block j of the evaluated batch -> tile `slot`
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      const uint32_t o = (uint32_t)__shfl((int)ro32, j * 8 + i * RW + lane / LPR, 64);
      const int r = a_r0 + RPP * i;                     // row of the block this lane serves
      // lane l of the wave lands at (wave base) + 16 l.  Written as assembly so that the request
      // stays unknown to the compiler, which would otherwise order every later LDS access of the
      // kernel behind it; the waits for these requests are the explicit ones below.
      const uint32_t dst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lptr_t)&tiles[slot * kTileUnits + (wave * RW + RPP * i) * LPR]);
      // (M0 holds the LDS destination; it is saved and put back, so nothing is clobbered)
      uint32_t m0_saved;
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_nop 0\n\ts_mov_b32 m0, %0"
                   : "=&s"(m0_saved) : "v"(o + ((a_c ^ (r & 7)) * 16)), "s"(P.a), "s"(dst) : "memory");
    }
  };
  // the first two blocks' rows are requested before anything else: their latency hides behind the W prologue
  eval_rows(0);
  load_rows(0, 0);
  load_rows(1, 1);
  VT_PROF(1);

  // Memory operations a step issues after its row requests; together with the next step's requests
  // they are what may still be in flight when the rows requested one step earlier are needed
  // (vector memory operations complete in the order they were issued).
  constexpr int kStores = C_F32 ? (LBM / 16) * NB : LBM * (CW / 8) / 64;
  constexpr int kInFlight = 2 * kStores + PASSES;
  constexpr int kWaitRows = (kInFlight & 15) | ((kInFlight >> 4) << 14) | 0x0F70;   // s_waitcnt vmcnt(kInFlight)
  static_assert(kInFlight < 64, "vmcnt has 6 bits");
  // LayerNorm in place of the rows that landed in tile `slot` (each row spread over LPR
  // consecutive lanes; a lane reads the 16 bytes of its own request and writes them back normalised)
  auto norm_tile = [&](int slot) {
    u32x4 raw[PASSES];
    uint4* mine = &tiles[slot * kTileUnits + wave * RW * LPR + lane];
    {
      const uint32_t addr = (uint32_t)(uintptr_t)(lptr_t)mine;
      if constexpr (PASSES == 1)
        asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(raw[0]) : "v"(addr) : "memory");
      else
        asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:%3\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(raw[0]), "=&v"(raw[PASSES - 1]) : "v"(addr), "i"(RPP * LPR * 16) : "memory");
    }
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      float x[8];
      {
        const Vec<T, 8> v = __builtin_bit_cast(Vec<T, 8>, raw[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = to_float(v.v[j]);
      }
      float s = ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
      s = group_sum<LPR>(s);
      const float mean = s * (1.0f / K);
      float q = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        x[j] -= mean;
        q += x[j] * x[j];
      }
      q = group_sum<LPR>(q);
      const float rstd = __builtin_amdgcn_rsqf(q * (1.0f / K) + P.eps);
      Vec<T, 8> o;
#pragma unroll
      for (int j = 0; j < 8; ++j) o.v[j] = from_float<T>(x[j] * rstd);
      mine[i * RPP * LPR] = __builtin_bit_cast(uint4, o);
    }
  };
  static_assert(PASSES <= 2, "the read-back above handles one or two passes");

  bool normed0 = false;

  // ---- this wave's slice of W as MFMA operands (lane: column n = wave*CW + nb*16 + l16, the 8
  // consecutive k of its quarter), kept in registers for the whole kernel
  opvec wf[KS][NB];
  if (P.w_rows_of_8) {
    // coalesced: 8x8 blocks of W are loaded row-wise (16 bytes per lane), transposed in registers
    // and parked in LDS as W^T [n][k]; every wave then picks its operands with ds_read_b128
    uint4* ldsW = reinterpret_cast<uint4*>(lds_raw);   // unit (n, kc) at n*LPR + (kc ^ ((n ^ (n >> 3)) & 7))
    const int nblk = (N / 8) * LPR;                    // 8x8 blocks: N/8 across, K/8 down; at most 2 per thread
    static_assert(48 * LPR <= 2 * LTHREADS, "two rounds cover W");
    uint4 rb[2][8];
    // Every workgroup reads all of W at the same moment; each starts at a different block so
    // that they do not all queue on the same L2 channel.
    const uint32_t rot61 = blockIdx.x * 61u;
    const int rot = (int)(rot61 - fdiv(rot61, P.nblk) * P.nblk.d);
    int kbs[2], cns[2];
    const bool wave_r1 = LTHREADS + wave * 64 < nblk;  // this wave has blocks in the second round
#pragma unroll
    for (int r = 0; r < 2; ++r) {                      // all loads of both rounds are in flight together
      const int idx = t + r * LTHREADS;
      if (r == 0 || wave_r1) {
        // a wave issues a round for all its lanes or not at all (a lane without a block of its own
        // reads the last one again and drops it): the number of loads in flight is then uniform
        // in the wave, and the wait for the rows requested before them can be an exact count
        int bidx = min(idx, nblk - 1) + rot;
        bidx = bidx >= nblk ? bidx - nblk : bidx;
        const int kb = (int)fdiv((uint32_t)bidx, P.n8), cn = bidx - kb * (N / 8);
        kbs[r] = kb, cns[r] = cn;
        const char* bp = P.b + axis_off(P.b_col, (uint32_t)(cn * 8)) * 2;
        if (P.w_k_runs_of_8) {                         // the 8 rows of a block are one stride apart
          bp += axis_off(P.b_row, (uint32_t)(kb * 8)) * 2;
          const int64_t rs = P.b_row.stride[2] * 2;
#pragma unroll
          for (int j = 0; j < 8; ++j) rb[r][j] = *reinterpret_cast<const uint4*>(bp + j * rs);
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j) rb[r][j] = *reinterpret_cast<const uint4*>(bp + axis_off(P.b_row, (uint32_t)(kb * 8 + j)) * 2);
        }
      }
    }
    // block 0's rows were requested before W and have landed by now: normalise them while W is
    // still on its way (8 or 16 loads are in flight behind them)
    if (wave_r1) __builtin_amdgcn_s_waitcnt(0x4F70);   // vmcnt(16)
    else __builtin_amdgcn_s_waitcnt(0x0F78);           // vmcnt(8)
    norm_tile(0);
    normed0 = true;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      if (t + r * LTHREADS < nblk) {
        const int kb = kbs[r], cn = cns[r];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
          uint32_t w[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) w[u] = __builtin_amdgcn_perm(word(rb[r][2 * u + 1], e >> 1), word(rb[r][2 * u], e >> 1), sel);
          const int n = cn * 8 + e;
          ldsW[n * LPR + (kb ^ ((n ^ (n >> 3)) & 7))] = make_uint4(w[0], w[1], w[2], w[3]);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int n = wave * CW + nb * 16 + l16;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (n < N) v = ldsW[n * LPR + ((ks * 4 + lg) ^ ((n ^ (n >> 3)) & 7))];
        wf[ks][nb] = __builtin_bit_cast(opvec, v);
      }
    }
    __syncthreads();                                   // W^T is no longer needed: the memory becomes tiles
  } else {
    const T* bp = reinterpret_cast<const T*>(P.b);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int n = wave * CW + nb * 16 + l16;
      const int64_t co = axis_off(P.b_col, (uint32_t)min(n, N - 1));
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Vec<T, 8> e;
#pragma unroll
        for (int j = 0; j < 8; ++j) e.v[j] = bp[axis_off(P.b_row, (uint32_t)(ks * 32 + lg * 8 + j)) + co];
        wf[ks][nb] = __builtin_bit_cast(opvec, e);
      }
    }
  }

  // 16-bit outputs leave through the staged C tile one step after they were computed: a wave
  // writes 8 complete rows (6 x 1 KB, whole cache lines) with streaming stores.  The buffer
  // descriptor ends with the block, so rows past it are dropped by the hardware; lanes whose
  // columns are past N get an offset outside it.  No store is conditional: every step issues the
  // same number of memory operations, which the explicit wait for the rows relies on (for the
  // step that has no finished block yet the descriptor is empty).
  auto store_block = [&](int cs, int64_t row0, int64_t r_end) {
    const uint64_t c_skip = (uint64_t)row0 * (uint64_t)N * 2u;
    const uint64_t c_left = (uint64_t)(r_end - row0) * (uint64_t)N * 2u;
    const __amdgpu_buffer_rsrc_t c_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        P.c + c_skip, 0, (int)min(c_left, (uint64_t)0x7fffffffu), 0x00020000);
    const char* sc = cstage + cs * (LBM * CPW);
#pragma unroll
    for (int q = 0; q < kStores; ++q) {
      const int id = q * 64 + lane;
      const int rl = id / CW, ch = id - rl * CW;          // CW 16-byte chunks per row of 8 waves x CW columns
      const int r = wave * (LBM / LWAVES) + rl, col = ch * 8;
      const u32x4 v = *reinterpret_cast<const u32x4*>(sc + r * CPW + ch * 16);
      const uint32_t off = col < N ? (uint32_t)(r * N + col) * 2u : 0x80000000u;
      __builtin_amdgcn_raw_buffer_store_b128(v, c_rsrc, (int)off, 0, 2);   // streaming: no dirty lines left in L2
    }
  };

  VT_PROF(2);
  int it = 0, slot = 0;                               // block `it` is multiplied from tile `slot` = it % 3
  int64_t prev_row0 = 0, prev_end = 0;                // the block whose outputs wait in the staged C tile
  __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): the first two blocks' rows are in LDS
  if (!normed0) norm_tile(0);
  for (;;) {
    int64_t row0, r_end;
    block_rows(it, &row0, &r_end);
    __syncthreads();                                  // tile `slot` is normalised; the staged C tile of the previous step is complete
    {
      // request the rows two blocks ahead, unconditionally (past the end they are not used): the
      // explicit wait below counts on the same number of operations in every step.  Their tile held
      // block it - 1, which every wave finished multiplying before it arrived at the barrier.
      const int j = (it + 2) & 7;
      if (j == 0) eval_rows(it + 2);
      load_rows(j, slot == 0 ? 2 : slot - 1);
    }
    if (!C_F32) store_block((it & 1) ^ 1, prev_row0, prev_end);
    f32x4 acc[LBM / 16][NB];
    const uint4* tile = tiles + slot * kTileUnits;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      opvec af[LBM / 16];
      const int chunk = ks * 4 + lg;
#pragma unroll
      for (int mb = 0; mb < LBM / 16; ++mb) {
        const int r = mb * 16 + l16;
        af[mb] = __builtin_bit_cast(opvec, tile[r * LPR + (chunk ^ (r & 7))]);
      }
#pragma unroll
      for (int mb = 0; mb < LBM / 16; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const f32x4 c0 = ks == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[mb][nb];
          acc[mb][nb] = M_::run(wf[ks][nb], af[mb], c0);   // C^T block: rows = n, cols = m
        }
    }
    // ---- stage 3: lane holds row m = mb*16 + l16 and columns nb*16 + lg*4 + (0..3)
    if (C_F32) {
      // fp32 outputs go straight from the accumulators (16 bytes per lane), through a buffer
      // descriptor that ends with the block
      const uint64_t c_skip = (uint64_t)row0 * (uint64_t)N * 4u;
      const uint64_t c_left = (uint64_t)(r_end - row0) * (uint64_t)N * 4u;
      const __amdgpu_buffer_rsrc_t c_rsrc = __builtin_amdgcn_make_buffer_rsrc(
          P.c + c_skip, 0, (int)min(c_left, (uint64_t)0x7fffffffu), 0x00020000);
#pragma unroll
      for (int mb = 0; mb < LBM / 16; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const int col = wave * CW + nb * 16 + lg * 4;   // N is a multiple of 8, so the 4 columns are valid together
          const uint32_t off = col < N ? (uint32_t)((mb * 16 + l16) * N + col) * 4u : 0x80000000u;
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[mb][nb]), c_rsrc, (int)off, 0, 0);
        }
    } else {
      char* sc = cstage + (it & 1) * (LBM * CPW);
#pragma unroll
      for (int mb = 0; mb < LBM / 16; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          Vec<T, 4> o;
#pragma unroll
          for (int i = 0; i < 4; ++i) o.v[i] = from_float<T>(acc[mb][nb][i]);
          *reinterpret_cast<Vec<T, 4>*>(sc + (mb * 16 + l16) * CPW + (wave * CW + nb * 16 + lg * 4) * 2) = o;
        }
      prev_row0 = row0;
      prev_end = r_end;
    }
    VT_PROF_ONCE(3);
    const int nslot = slot == 2 ? 0 : slot + 1;
    if (it + 1 < n_it) {
      __builtin_amdgcn_s_waitcnt(kWaitRows);          // the rows requested one step ago have landed
      norm_tile(nslot);
    }
    slot = nslot;
    if (++it >= n_it) break;
  }
  VT_PROF(4);
  if (!C_F32) {
    __syncthreads();                                  // the last staged C tile is complete
    store_block((it & 1) ^ 1, prev_row0, prev_end);
  }
  VT_PROF(5);
  __builtin_amdgcn_s_waitcnt(0x0F70);                 // requests past the last block still target this workgroup's LDS
  VT_PROF(6);
  VT_PROF_FLUSH(ln_gemm, blockIdx.x);
}

template <typename T, bool C_F32>
int launch_t(const LnGemmParams& P, int lpr, int nb, hipStream_t st) {
  static const int n_cu = [] {
    int dev = 0, n = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 256;
    return n > 0 ? n : 256;
  }();
  // One workgroup per compute unit: full rounds of blocks, then one more block for as many
  // workgroups as the rest needs.  (Dealing the rest out in 16-row shares to all workgroups was
  // measured and is slower: every workgroup then pays the fixed cost of one more step.)
  LnGemmParams Q = P;
  Q.n_full = P.M / (n_cu * LBM);
  const int rest = P.M - Q.n_full * n_cu * LBM;
  Q.tail_rows = LBM;
  dim3 grid((unsigned)(Q.n_full > 0 ? n_cu : (rest + Q.tail_rows - 1) / Q.tail_rows));
#define VT_LN_CASE(L, B)                                                                     \
  if (lpr == L && nb == B) {                                                                 \
    hipLaunchKernelGGL((k_ln_gemm<T, C_F32, L, B>), grid, dim3(LTHREADS), 0, st, Q);              \
    return check_launch("vt_gemm(layernorm)");                                               \
  }
  VT_LN_CASE(16, 1) VT_LN_CASE(16, 2) VT_LN_CASE(16, 3) VT_LN_CASE(8, 1) VT_LN_CASE(8, 2) VT_LN_CASE(8, 3)
#undef VT_LN_CASE
  return fail(VT_ERR_UNSUPPORTED, "vt_gemm(layernorm): shape outside the fused kernel");
}

}  // namespace

namespace vt {

// One group of vt_gemm with prologue = VT_GEMM_LAYERNORM.
int ln_gemm_launch(const vt_desc& A, const vt_desc& B, void* C, int c_dtype, float eps, hipStream_t st) {
  const int dt = A.dtype;
  int n = (int)A.shape.size();
  if (n < 2) return fail(VT_ERR_SHAPE, "vt_gemm(layernorm): A must have at least 2 dims");
  if (B.shape.size() != 2) return fail(VT_ERR_SHAPE, "vt_gemm(layernorm): B must be [K,N]");
  const int64_t K = A.shape[n - 1], N = B.shape[1];
  if (B.shape[0] != K) return fail(VT_ERR_SHAPE, "vt_gemm(layernorm): inner dims of A and B differ");
  if (K != 64 && K != 128) return fail(VT_ERR_UNSUPPORTED, "vt_gemm(layernorm): the fused kernel takes K = 64 or 128 (run vt_elementwise + vt_gemm otherwise)");
  if (N > 384 || N % 8) return fail(VT_ERR_UNSUPPORTED, "vt_gemm(layernorm): the fused kernel takes N <= 384, a multiple of 8");
  if (A.pieces.size() != 1 || !A.pieces[0].v.lower.empty() || B.pieces.size() != 1 || !B.pieces[0].v.lower.empty())
    return fail(VT_ERR_UNSUPPORTED, "vt_gemm(layernorm): operands must be single pieces with one index stage");
  int64_t M = 1;
  for (int i = 0; i < n - 1; ++i) M *= A.shape[i];
  if (M >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, "vt_gemm(layernorm): too many rows");
  LnGemmParams P;
  memset(&P, 0, sizeof(P));
  const Piece& pa = A.pieces[0];
  const Piece& pb = B.pieces[0];
  int rc = make_axis(A, pa, 0, n - 1, &P.a_row, "vt_gemm(layernorm): A rows", true);
  if (rc != VT_OK) return rc;
  AxisMap<3> a_col;
  rc = make_axis(A, pa, n - 1, n, &a_col, "vt_gemm(layernorm): A columns");
  if (rc != VT_OK) return rc;
  if (!(a_col.nd == 1 && a_col.stride[2] == 1)) return fail(VT_ERR_UNSUPPORTED, "vt_gemm(layernorm): rows of A must be contiguous");
  rc = make_axis(B, pb, 0, 1, &P.b_row, "vt_gemm(layernorm): B rows");
  if (rc != VT_OK) return rc;
  rc = make_axis(B, pb, 1, 2, &P.b_col, "vt_gemm(layernorm): B columns");
  if (rc != VT_OK) return rc;
  const vt_source& sa = A.sources[pa.src];
  const vt_source& sb = B.sources[pb.src];
  if (!sa.ptr || !sb.ptr) return fail(VT_ERR_INVALID_ARG, "vt_gemm(layernorm): source without a device pointer");
  P.a = static_cast<const char*>(sa.ptr) + pa.v.base * 2;
  P.b = static_cast<const char*>(sb.ptr) + pb.v.base * 2;
  if ((uintptr_t)P.a % 16 || !strides_multiple_of(P.a_row, 8, 0))
    return fail(VT_ERR_UNSUPPORTED, "vt_gemm(layernorm): rows of A must be 16-byte aligned");
  if ((uintptr_t)C % 16) return fail(VT_ERR_INVALID_ARG, "vt_gemm(layernorm): C must be 16-byte aligned");
  {
    int64_t span = 0;
    for (int i = 0; i < 5; ++i) span += (int64_t)(P.a_row.radix[i].d - 1) * P.a_row.stride[i];
    if (P.a_row.table) {
      span = 1;
      for (int i = 0; i < sa.ndim; ++i) span *= sa.shape[i];
    }
    if ((span + K) * 2 >= (1ll << 32)) return fail(VT_ERR_UNSUPPORTED, "vt_gemm(layernorm): A spans 4 GiB or more");
  }
  P.w_rows_of_8 = (uintptr_t)P.b % 16 == 0 && P.b_col.stride[2] == 1 && P.b_col.radix[2].d % 8 == 0 &&
                  strides_multiple_of(P.b_col, 8, 1) && strides_multiple_of(P.b_row, 8, 0);
  P.w_k_runs_of_8 = P.b_row.radix[2].d % 8 == 0;
  P.n8 = make_fastdiv((uint32_t)(N / 8));
  P.nblk = make_fastdiv((uint32_t)((N / 8) * (K / 8)));
  P.c = static_cast<char*>(C);
  P.M = (int32_t)M;
  P.N = (int32_t)N;
  P.K = (int32_t)K;
  P.eps = eps;
  if (M == 0) return VT_OK;                            // nothing to compute
  const int lpr = (int)(K / 8);
  const int nb = (int)((N + 127) / 128);               // 16-column blocks per wave: 8 waves x nb x 16 >= N
  const bool c32 = c_dtype == VT_F32;
  if (dt == VT_BF16) return c32 ? launch_t<bf16_t, true>(P, lpr, nb, st) : launch_t<bf16_t, false>(P, lpr, nb, st);
  return c32 ? launch_t<f16_t, true>(P, lpr, nb, st) : launch_t<f16_t, false>(P, lpr, nb, st);
}

}  // namespace vt
