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
// current block is multiplied (v_mfma_f32_32x32x16).  Stage 3 is a plain store of C.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <type_traits>

#include "vt_gemm_common.h"

using namespace vt;
using namespace vt::gemm;

namespace {

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
  int32_t pad;
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
  __shared__ uint4 ldsA[2][LBM * LPR];       // [row][LPR chunks of 8 k], chunk c of row r at r*LPR + (c ^ (r & (LPR-1) & 7))

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int M = P.M, N = P.N;

  // ---- this wave's slice of W, as MFMA B operands: lane holds column n = col0 + nb*32 + l32 and
  // the 8 consecutive k of its half; read once through the map
  opvec wf[KS][NB];
  {
    const T* bp = reinterpret_cast<const T*>(P.b);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int n = wave * (NB * 32) + nb * 32 + l32;
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

  const int a_c = t % LPR, a_r0 = t / LPR;             // chunk and first row; rows a_r0 + RPP * i
  uint4 ra[PASSES];
  auto load_rows = [&](int blk) {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      const int m = min(blk * LBM + a_r0 + RPP * i, M - 1);
      const int64_t ro = P.a_row.tdig >= 0 ? axis_off_table(P.a_row, (uint32_t)m) : axis_off(P.a_row, (uint32_t)m);
      ra[i] = *reinterpret_cast<const uint4*>(P.a + (ro + a_c * 8) * 2);
    }
  };
  // LayerNorm of the rows held in ra (each row spread over LPR consecutive lanes), then -> LDS
  auto norm_store = [&](int buf) {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      float x[8];
      {
        const Vec<T, 8> v = __builtin_bit_cast(Vec<T, 8>, ra[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = to_float(v.v[j]);
      }
      float s = ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
#pragma unroll
      for (int d = 1; d < LPR; d <<= 1) s += __shfl_xor(s, d, 64);
      const float mean = s * (1.0f / K);
      float q = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        x[j] -= mean;
        q += x[j] * x[j];
      }
#pragma unroll
      for (int d = 1; d < LPR; d <<= 1) q += __shfl_xor(q, d, 64);
      const float rstd = 1.0f / sqrtf(q * (1.0f / K) + P.eps);
      Vec<T, 8> o;
#pragma unroll
      for (int j = 0; j < 8; ++j) o.v[j] = from_float<T>(x[j] * rstd);
      const int r = a_r0 + RPP * i;
      ldsA[buf][r * LPR + (a_c ^ (r & 7 & (LPR - 1)))] = __builtin_bit_cast(uint4, o);
    }
  };

  typedef typename std::conditional<C_F32, float, T>::type CT;
  CT* cbase = reinterpret_cast<CT*>(P.c);

  int blk = blockIdx.x;
  if (blk >= P.n_blocks) return;
  load_rows(blk);
  norm_store(0);
  int buf = 0;
  for (; blk < P.n_blocks; blk += gridDim.x, buf ^= 1) {
    const int nxt = blk + gridDim.x;
    __syncthreads();                                  // tile `buf` is complete; tile buf^1 is free again
    if (nxt < P.n_blocks) load_rows(nxt);             // in flight during the MFMAs below
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
        for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = M_::run(af[mb], wf[ks][nb], acc[mb][nb]);
    }
    // ---- stage 3
#pragma unroll
    for (int mb = 0; mb < LMB; ++mb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int col = wave * (NB * 32) + nb * 32 + l32;
        const int row0 = blk * LBM + mb * 32 + lh * 4;
        if (col < N) {
          CT* cp = cbase + (size_t)row0 * N + col;
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (row0 + 8 * j + i < M) cp[(size_t)(8 * j + i) * N] = from_float<CT>(acc[mb][nb][4 * j + i]);
        }
      }
    if (nxt < P.n_blocks) norm_store(buf ^ 1);
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
