// LayerNorm fused into the load stage of a skinny GEMM: C = LN(A) . W with A virtual [.., K],
// K = 64 or 128, W virtual [K, N], N <= 384 (the window-partition -> LayerNorm -> linear chain).
// The whole path is bound by HBM (the output is 3x the input), so the design goal is to touch
// every byte once: the normalised tokens never exist in global memory, and W never leaves
// registers.
//
// A persistent workgroup of 4 waves walks over blocks of 64 rows.  Each wave owns N/4 output
// columns and keeps its slice of W in registers for the whole kernel (K/16 x NB MFMA operands).
// Stage 1 through the map: 16 (K=128) or 8 (K=64) lanes fetch one row with 16-byte loads at
// row_offset(m) (mixed-radix digits / index table, evaluated per row); the same lanes reduce
// mean and variance with xor-shuffles, normalise in fp32, round to the operand type and write
// the row into an XOR-swizzled LDS tile; the rows of the next block are in flight while the
// current block is multiplied (v_mfma_f32_32x32x16).  The product is formed transposed (W^T as the
// first operand), so a lane ends up with 4 consecutive output columns; stage 3 packs them,
// bounces the wave's 64 x N/4 sub-tile through LDS and leaves with 16-byte stores that cover
// whole row segments (the output is three quarters of all traffic).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <type_traits>

#include "vt_gemm_common.h"

using namespace vt;
using namespace vt::gemm;

namespace {

// Sum over the LPR (8 or 16) consecutive lanes that share a row, on the VALU's data-parallel
// primitives (mirror within 16 / 8 lanes, then the two quad permutes): every lane gets the total.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
  if (LPR == 16) v += dpp_move<0x140>(v);   // row_mirror: lane i <-> 15 - i
  v += dpp_move<0x141>(v);                  // row_half_mirror: i <-> 7 - i
  v += dpp_move<0xB1>(v);                   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);                   // quad_perm [2,3,0,1]
  return v;
}

constexpr int LBM = 64;           // rows per block
constexpr int LMB = LBM / 32;     // 32-row MFMA blocks per block

struct LnGemmParams {
  const char* a;
  const char* b;
  char* c;
  AxisMap<5> a_row;
  AxisMap<3> b_row, b_col;
  int32_t M, N, K, n_blocks;
  float eps;
  int32_t w_rows_of_8;   // W has runs of 8 contiguous, 16-byte aligned elements along N: coalesced prologue
};

// LPR = lanes per row = K / 8; NB = 32-column blocks per wave
template <typename T, bool C_F32, int LPR, int NB>
__global__ void __launch_bounds__(256) k_ln_gemm(const LnGemmParams P) {
  typedef Mma<T> M_;
  typedef typename M_::vec opvec;
  constexpr int K = LPR * 8;
  constexpr int KS = K / 16;                 // k16 steps
  constexpr int RPP = 256 / LPR;             // rows staged per pass of the workgroup
  constexpr int PASSES = LBM / RPP;
  constexpr int CW = NB * 32;                // output columns per wave
  constexpr int CPITCH = CW * 2 + 16;        // bytes per staged row (16-byte aligned, de-phased banks)
  constexpr int kABytes = 2 * LBM * LPR * 16, kCBytes = 4 * LBM * CPITCH, kWBytes = 4 * CW * K * 2;
  constexpr int kLdsBytes = kABytes + kCBytes > kWBytes ? kABytes + kCBytes : kWBytes;
  __shared__ __attribute__((aligned(16))) char lds_raw[kLdsBytes];
  // steady state: two A tiles [row][LPR chunks of 8 k] (chunk c of row r at r*LPR + (c ^ (r & 7))) and
  // one staging area per wave for its C sub-tile; during the prologue the same memory holds W^T
  uint4 (*ldsA)[LBM * LPR] = reinterpret_cast<uint4 (*)[LBM * LPR]>(lds_raw);
  char (*ldsC)[LBM * CPITCH] = reinterpret_cast<char (*)[LBM * CPITCH]>(lds_raw + kABytes);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int M = P.M, N = P.N;

  // ---- this wave's slice of W as MFMA operands (lane: column n = wave*CW + nb*32 + l32, the 8
  // consecutive k of its half), kept in registers for the whole kernel
  opvec wf[KS][NB];
  if (P.w_rows_of_8) {
    // coalesced: 8x8 blocks of W are loaded row-wise (16 bytes per lane), transposed in registers
    // and parked in LDS as W^T [n][k]; every wave then picks its operands with ds_read_b128
    uint4* ldsW = reinterpret_cast<uint4*>(lds_raw);   // unit (n, kc) at n*LPR + (kc ^ ((n ^ (n >> 3)) & 7))
    const int nblk = (N / 8) * LPR;                    // 8x8 blocks: N/8 across, K/8 down
    for (int bidx = t; bidx < nblk; bidx += 256) {
      const int kb = bidx / (N / 8), cn = bidx - kb * (N / 8);
      const char* bp = P.b + axis_off(P.b_col, (uint32_t)(cn * 8)) * 2;
      uint4 rb[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) rb[j] = *reinterpret_cast<const uint4*>(bp + axis_off(P.b_row, (uint32_t)(kb * 8 + j)) * 2);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        uint32_t w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w[u] = __builtin_amdgcn_perm(word(rb[2 * u + 1], e >> 1), word(rb[2 * u], e >> 1), sel);
        const int n = cn * 8 + e;
        ldsW[n * LPR + (kb ^ ((n ^ (n >> 3)) & 7))] = make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
    __syncthreads();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int n = wave * CW + nb * 32 + l32;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (n < N) v = ldsW[n * LPR + ((ks * 2 + lh) ^ ((n ^ (n >> 3)) & 7))];
        wf[ks][nb] = __builtin_bit_cast(opvec, v);
      }
    }
    __syncthreads();                                   // W^T is no longer needed: the memory becomes tiles
  } else {
    const T* bp = reinterpret_cast<const T*>(P.b);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int n = wave * CW + nb * 32 + l32;
      const int64_t co = axis_off(P.b_col, (uint32_t)min(n, N - 1));
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Vec<T, 8> e;
#pragma unroll
        for (int j = 0; j < 8; ++j) e.v[j] = bp[axis_off(P.b_row, (uint32_t)(ks * 16 + lh * 8 + j)) + co];
        wf[ks][nb] = __builtin_bit_cast(opvec, e);
      }
    }
  }

  // ---- stage 1 bookkeeping.  LPR lanes share a row; the 16 rows a wave stages per block are
  // evaluated through the map by 16 lanes (one row each) and handed to the lanes that load them.
  const int a_c = t % LPR, a_r0 = t / LPR;             // chunk and first row; rows a_r0 + RPP * i
  uint4 ra[2][PASSES];                                  // rows of the next two blocks (prefetch distance 2)
  constexpr int RW = 64 / LPR;                          // rows per wave and pass
  const int my_i = (lane & 15) / RW, my_g = (lane & 15) % RW;   // the row this lane evaluates: pass my_i, group my_g
  auto load_rows = [&](int blk, int slot) {
    const int m = min(blk * LBM + wave * RW + my_g + RPP * my_i, M - 1);
    const int64_t ro = P.a_row.tdig >= 0 ? axis_off_table(P.a_row, (uint32_t)m) : axis_off(P.a_row, (uint32_t)m);
    const uint32_t ro32 = (uint32_t)(ro * 2);           // byte offset (the host checks that A spans < 4 GiB)
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      const uint32_t o = (uint32_t)__shfl((int)ro32, i * RW + lane / LPR, 64);
      ra[slot][i] = *reinterpret_cast<const uint4*>(P.a + (o + a_c * 16));
    }
  };
  // LayerNorm of the rows held in ra (each row spread over LPR consecutive lanes), then -> LDS
  auto norm_store = [&](int buf) {   // rows come from register slot `buf`, go to LDS tile `buf`
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      float x[8];
      {
        const Vec<T, 8> v = __builtin_bit_cast(Vec<T, 8>, ra[buf][i]);
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
      const float rstd = 1.0f / sqrtf(q * (1.0f / K) + P.eps);
      Vec<T, 8> o;
#pragma unroll
      for (int j = 0; j < 8; ++j) o.v[j] = from_float<T>(x[j] * rstd);
      const int r = a_r0 + RPP * i;
      ldsA[buf][r * LPR + (a_c ^ (r & 7 & (LPR - 1)))] = __builtin_bit_cast(uint4, o);
    }
  };

  int blk = blockIdx.x;
  if (blk >= P.n_blocks) return;
  const int stride = gridDim.x;
  load_rows(blk, 0);
  if (blk + stride < P.n_blocks) load_rows(blk + stride, 1);
  norm_store(0);
  auto step = [&](int blk, auto parity) {
    constexpr int buf = decltype(parity)::value;
    const int nxt = blk + stride;
    __syncthreads();                                  // tile `buf` is complete; tile buf^1 is free again
    if (nxt + stride < P.n_blocks) load_rows(nxt + stride, buf);   // two blocks ahead: lands while this and the next block are multiplied
    f32x16 acc[LMB][NB];
#pragma unroll
    for (int mb = 0; mb < LMB; ++mb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mb][nb][e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      opvec af[LMB];
      const int chunk = ks * 2 + lh;
#pragma unroll
      for (int mb = 0; mb < LMB; ++mb) {
        const int r = mb * 32 + l32;
        af[mb] = __builtin_bit_cast(opvec, ldsA[buf][r * LPR + (chunk ^ (r & 7 & (LPR - 1)))]);
      }
#pragma unroll
      for (int mb = 0; mb < LMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = M_::run(wf[ks][nb], af[mb], acc[mb][nb]);   // C^T block: rows = n, cols = m
    }
    // ---- stage 3: lane holds row m = mb*32 + l32 and columns nb*32 + lh*4 + 8j + (0..3)
    if (C_F32) {
#pragma unroll
      for (int mb = 0; mb < LMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const int row = blk * LBM + mb * 32 + l32;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int col = wave * CW + nb * 32 + lh * 4 + 8 * j;
            if (row < M && col < N) {       // N is a multiple of 8, so the 4 columns are valid together
              float4 v = make_float4(acc[mb][nb][4 * j], acc[mb][nb][4 * j + 1], acc[mb][nb][4 * j + 2], acc[mb][nb][4 * j + 3]);
              *reinterpret_cast<float4*>(reinterpret_cast<float*>(P.c) + (size_t)row * N + col) = v;
            }
          }
        }
    } else {
      char* sc = ldsC[wave];
#pragma unroll
      for (int mb = 0; mb < LMB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            Vec<T, 4> o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o.v[i] = from_float<T>(acc[mb][nb][4 * j + i]);
            *reinterpret_cast<Vec<T, 4>*>(sc + (mb * 32 + l32) * CPITCH + (nb * 32 + lh * 4 + 8 * j) * 2) = o;
          }
      // wave-local: the same wave reads back what it wrote (LDS operations of a wave stay in order)
      constexpr int CH = CW / 8;             // 16-byte chunks per staged row
#pragma unroll
      for (int q = 0; q < LBM * CH / 64; ++q) {
        const int id = q * 64 + lane;
        const int r = id / CH, ch = id - r * CH;
        const int row = blk * LBM + r, col = wave * CW + ch * 8;
        const uint4 v = *reinterpret_cast<const uint4*>(sc + r * CPITCH + ch * 16);
        if (row < M && col < N) *reinterpret_cast<uint4*>(reinterpret_cast<T*>(P.c) + (size_t)row * N + col) = v;
      }
    }
    if (nxt < P.n_blocks) norm_store(buf ^ 1);
  };
  for (;;) {
    step(blk, std::integral_constant<int, 0>{});
    blk += stride;
    if (blk >= P.n_blocks) break;
    step(blk, std::integral_constant<int, 1>{});
    blk += stride;
    if (blk >= P.n_blocks) break;
  }
}

template <typename T, bool C_F32>
int launch_t(const LnGemmParams& P, int lpr, int nb, hipStream_t st) {
  static const int n_cu = [] {
    int dev = 0, n = 256;
    if (hipGetDevice(&dev) == hipSuccess) hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    return n > 0 ? n : 256;
  }();
  dim3 grid((unsigned)std::min(P.n_blocks, n_cu));     // persistent: one workgroup per compute unit
#define VT_LN_CASE(L, B)                                                                     \
  if (lpr == L && nb == B) {                                                                 \
    hipLaunchKernelGGL((k_ln_gemm<T, C_F32, L, B>), grid, dim3(256), 0, st, P);              \
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
  P.c = static_cast<char*>(C);
  P.M = (int32_t)M;
  P.N = (int32_t)N;
  P.K = (int32_t)K;
  P.n_blocks = (int32_t)((M + LBM - 1) / LBM);
  P.eps = eps;
  const int lpr = (int)(K / 8);
  const int nb = (int)((N + 127) / 128);
  const bool c32 = c_dtype == VT_F32;
  if (dt == VT_BF16) return c32 ? launch_t<bf16_t, true>(P, lpr, nb, st) : launch_t<bf16_t, false>(P, lpr, nb, st);
  return c32 ? launch_t<f16_t, true>(P, lpr, nb, st) : launch_t<f16_t, false>(P, lpr, nb, st);
}

}  // namespace vt
