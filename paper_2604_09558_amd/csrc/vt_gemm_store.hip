// Skinny GEMM with a producer-side virtual store: C = A . B for a handful of rows (a decode
// step's merged QKV projection: M = batch), each result element written straight to the
// physical tensor and place that the OUTPUT descriptor names (Sec. 3.1, Fig. 4: stage 3 of the
// MatMul writes Q to its buffer and K, V into the cache slot of the current position, so the
// Split, Reshape and ScatterND between projection and attention are never executed; Sec. 4.2:
// only the store stage of the kernel changes).  gfx950, wave64, v_mfma_f32_16x16x32.
//
// The kernel is bound by reading B (the weight) once from HBM.  Work split: one workgroup per
// (128-column block, slice of K, block of 16 rows); its 4 waves take tiles of 32 k-rows.  Per
// tile a lane loads 8 rows of its own 8-column chunk of B (whole 256-byte row segments per 16
// lanes), transposes the 8x8 block inside its registers (v_perm_b32) and feeds it as the MFMA's
// first operand, C^T += B^T . A^T; the contraction index is permuted identically for A, whose
// fragment is two 8-byte loads per lane.  B never touches LDS.  The waves of a workgroup are
// summed through LDS, the K slices through a workspace: the workgroup that finishes last for a
// (column block, row block) adds the partial sums in slice order (a ticket counter; no second
// launch, no spinning, bitwise reproducible) and performs the mapped store.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <type_traits>

#include "vt_coherent.h"
#include "vt_gemm_common.h"
#include "vt_profile.h"

using namespace vt;
using namespace vt::gemm;

// profile marks: 0 start, 1 first tile multiplied, 2 tile loop done, 3 partial sums stored, 4 ticket taken,
// 5 mapped store done, 7 compute die
VT_PROF_DECLARE(gemm_store)
#define STORE_WG (blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z))

namespace vt {
int gemm_store_launch(const vt_desc& A, const vt_desc& B, const vt_desc& Cd, hipStream_t st);   // vt_gemm.hip
}

namespace {

constexpr int kBN = 128;          // columns per workgroup
constexpr int kBM = 16;           // rows per workgroup (one MFMA block)
constexpr int kTileK = 32;        // k-rows per wave step
constexpr int kWaves = 4;
constexpr int kMaxOutPieces = 4;
constexpr int kTiledFrom = 128;   // more rows than this go to the 256 x 256 tiled kernel

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T>
struct Mma16;
template <>
struct Mma16<bf16_t> {
  typedef bf16x8 vec;
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
};
template <>
struct Mma16<f16_t> {
  typedef f16x8 vec;
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
};

// Columns [col_lo, col_hi) of the virtual output live in one physical tensor:
// element (m, n) at base + 2 * (row(m) + col(n - col_lo)).
struct OutPiece {
  char* base;
  int32_t col_lo, col_hi;
  AxisMap<3> row, col;
};

struct StoreParams {
  const char* a;           // A element (0, 0)
  const char* b;           // B element (0, 0)
  AxisMap<3> a_row;        // row m of A -> element offset; K is contiguous
  int64_t ldb;             // elements between consecutive rows of B
  OutPiece out[kMaxOutPieces];
  int32_t n_out;
  int32_t M, N, K;
  int32_t n_splits, k_per_split;   // k_per_split is a multiple of kTileK
  uint32_t* tickets;       // [row blocks][column blocks], zero between launches
  float* partial;          // [row blocks][column blocks][n_splits][kBM][kBN]
};

struct Regs16 {
  uint32_t w[4];
};

// B is read exactly once per launch: streaming (nontemporal) loads
__device__ __forceinline__ Regs16 load16(const char* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  Regs16 r;
  r.w[0] = t[0]; r.w[1] = t[1]; r.w[2] = t[2]; r.w[3] = t[3];
  return r;
}

template <typename T>
__global__ void __launch_bounds__(kWaves * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) k_gemm_store(const StoreParams P) {
  typedef Mma16<T> M_;
  typedef typename M_::vec opvec;
  __shared__ __attribute__((aligned(16))) float red[kWaves][kBM * kBN];     // 32 KB
  __shared__ uint32_t ticket_sh;
  // The output pieces' maps, copied from the arguments while the tiles stream: the store stage
  // picks a piece per lane and evaluates its row and column maps, and read from the argument
  // segment every step of that would be a dependent read of memory at the very end of the kernel.
  __shared__ OutPiece out_sh[kMaxOutPieces];
  {
    const uint32_t* from = reinterpret_cast<const uint32_t*>(&P.out[0]);
    uint32_t* to = reinterpret_cast<uint32_t*>(&out_sh[0]);
    for (uint32_t i = threadIdx.x; i < sizeof(out_sh) / 4; i += kWaves * 64) to[i] = from[i];
  }

  VT_PROF_BEGIN();
  VT_PROF(0);
  const int split = blockIdx.x, cb = blockIdx.y, rb = blockIdx.z;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int l16 = lane & 15, lg = lane >> 4;
  const int M = P.M, N = P.N, K = P.K;
  const int k_begin = split * P.k_per_split, k_end = min(K, k_begin + P.k_per_split);
  const int n_tiles = (k_end - k_begin + kTileK - 1) / kTileK;

  // this lane's 8 columns of B (the last column block of a ragged N reads clamped columns,
  // whose results are never stored) and its row of A
  const int col = min(cb * kBN + l16 * 8, N - 8);
  const char* bp = P.b + (size_t)col * 2;
  const size_t row_bytes = (size_t)P.ldb * 2;
  const uint32_t lane_off = (uint32_t)(lg * 4 * row_bytes + (size_t)col * 2);   // the host checks 16 rows of B < 4 GiB
  const int m = rb * kBM + l16;
  const bool m_ok = m < M;
  const char* ap = P.a + axis_off(P.a_row, (uint32_t)min(m, M - 1)) * 2;

  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  // B rows of a tile: load j is contraction slot j of the lane group, row (j>>2)*16 + lg*4 + (j&3);
  // rows past k_end repeat the last valid row and meet a zero in A.  Three register sets: the
  // loads of the next two tiles are in flight while one tile is multiplied (a wave has only a
  // few tiles, so the depth of this pipeline is what hides the memory latency).
  Regs16 bst[3][8];
  uint2 a_lo[3], a_hi[3];
  auto issue = [&](int tile, auto set) {
    constexpr int S = decltype(set)::value;
    if (tile >= n_tiles) return;
    const int k0 = k_begin + tile * kTileK;
    if (k0 + kTileK <= k_end) {
      // a full tile: one wave-uniform base per load plus ONE per-lane offset
      const char* wb = P.b + (size_t)k0 * row_bytes;
#pragma unroll
      for (int j = 0; j < 8; ++j) bst[S][j] = load16(wb + (size_t)((j >> 2) * 16 + (j & 3)) * row_bytes + lane_off);
    } else {
      const int last = k_end - 1 - k0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int r = min((j >> 2) * 16 + lg * 4 + (j & 3), last);
        bst[S][j] = load16(bp + (size_t)(k0 + r) * row_bytes);
      }
    }
    // A^T fragment: k = k0 + lg*4 + (0..3) and k0 + 16 + lg*4 + (0..3) of row m (K % 8 == 0, so
    // a group of 4 is valid or not as a whole)
    a_lo[S] = make_uint2(0, 0);
    a_hi[S] = make_uint2(0, 0);
    if (m_ok && k0 + lg * 4 < k_end) a_lo[S] = *reinterpret_cast<const uint2*>(ap + (size_t)(k0 + lg * 4) * 2);
    if (m_ok && k0 + 16 + lg * 4 < k_end) a_hi[S] = *reinterpret_cast<const uint2*>(ap + (size_t)(k0 + 16 + lg * 4) * 2);
  };
  auto multiply = [&](auto set) {
    constexpr int S = decltype(set)::value;
    const opvec aop = __builtin_bit_cast(opvec, make_uint4(a_lo[S].x, a_lo[S].y, a_hi[S].x, a_hi[S].y));
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
      uint32_t w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) w[u] = __builtin_amdgcn_perm(bst[S][2 * u + 1].w[e >> 1], bst[S][2 * u].w[e >> 1], sel);
      acc[e] = M_::run(__builtin_bit_cast(opvec, make_uint4(w[0], w[1], w[2], w[3])), aop, acc[e]);
    }
  };
  typedef std::integral_constant<int, 0> S0;
  typedef std::integral_constant<int, 1> S1;
  typedef std::integral_constant<int, 2> S2;
  // this wave's tiles: wave, wave + kWaves, ...
  issue(wave, S0{});
  issue(wave + kWaves, S1{});
  for (int tile = wave; tile < n_tiles; tile += 3 * kWaves) {
    issue(tile + 2 * kWaves, S2{});
    multiply(S0{});
    VT_PROF_ONCE(1);
    if (tile + kWaves >= n_tiles) break;
    issue(tile + 3 * kWaves, S0{});
    multiply(S1{});
    if (tile + 2 * kWaves >= n_tiles) break;
    issue(tile + 4 * kWaves, S1{});
    multiply(S2{});
  }

  // what the rest of the kernel needs from the arguments, fetched in one batch and pinned in
  // registers (the empty statement makes the values opaque, so they are not fetched again in
  // front of each of the dependent steps below)
  uint32_t* a_tickets = P.tickets;
  float* a_partial = P.partial;
  int a_ns = P.n_splits, a_nout = P.n_out;
  asm volatile("" : "+s"(a_tickets), "+s"(a_partial), "+s"(a_ns), "+s"(a_nout));

  // ---- sum the waves through LDS.  acc[e][i] is C[m = l16][n = (lg*4 + i)*8 + e] of the block.
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][l16 * kBN + (lg * 4 + i) * 8 + e] = acc[e][i];
  __syncthreads();
  VT_PROF(2);
  const size_t blk = (size_t)rb * gridDim.y + cb;
  float* mine = a_partial + (blk * a_ns + split) * (kBM * kBN);
  const int n_valid = min(kBM, M - rb * kBM) * kBN;     // rows past M are neither summed nor stored
  // four consecutive columns per thread: 16-byte device-coherent stores, whole lines per wave
  for (int idx = threadIdx.x * 4; idx < n_valid; idx += kWaves * 64 * 4) {
    float4 s = *reinterpret_cast<const float4*>(&red[0][idx]);
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      const float4 t = *reinterpret_cast<const float4*>(&red[w][idx]);
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    store_device_b128(&mine[idx], __builtin_bit_cast(u32x4_t, s));
  }
  // ---- the last workgroup of this block to arrive adds the K slices and stores.  The barrier
  // waits for every wave's stores to complete before one thread takes the ticket; atomicInc
  // wraps to 0 at n_splits - 1, which leaves the counter ready for the next launch.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  VT_PROF(3);
  if (threadIdx.x == 0) ticket_sh = atomicInc(&a_tickets[blk], (uint32_t)(a_ns - 1));
  __syncthreads();
  VT_PROF(4);
  if (ticket_sh != (uint32_t)(a_ns - 1)) {
    VT_PROF_FLUSH(gemm_store, STORE_WG);
    return;
  }
  const float* all = a_partial + blk * a_ns * (kBM * kBN);
  for (int idx = threadIdx.x * 4; idx < n_valid; idx += kWaves * 64 * 4) {
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int sp0 = 0; sp0 < a_ns; sp0 += 4) {      // slices in order: the sum is reproducible
      u32x4_t v[4];
      const float* q[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) q[u] = &all[(size_t)min(sp0 + u, a_ns - 1) * (kBM * kBN) + idx];
      load_device_4xb128(q[0], q[1], q[2], q[3], v);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (sp0 + u < a_ns) {
          const float4 t = __builtin_bit_cast(float4, v[u]);
          s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
    }
    const float sv[4] = {s.x, s.y, s.z, s.w};
    const int mm = rb * kBM + idx / kBN;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int n = cb * kBN + idx % kBN + c;
      if (n >= N) continue;
      // stage 3 through the map: which physical tensor holds column n, and where
      int pc = 0;
#pragma unroll
      for (int i = 1; i < kMaxOutPieces; ++i)
        if (i < a_nout && n >= out_sh[i].col_lo) pc = i;
      const OutPiece& o = out_sh[pc];
      const int64_t off = axis_off(o.row, (uint32_t)mm) + axis_off(o.col, (uint32_t)(n - o.col_lo));
      *reinterpret_cast<T*>(o.base + off * 2) = from_float<T>(sv[c]);
    }
  }
#ifdef VT_PROFILE
  __builtin_amdgcn_s_waitcnt(0);
  VT_PROF(5);
  VT_PROF_FLUSH(gemm_store, STORE_WG);
#endif
}

__global__ void k_zero_store_ws(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// Slices of K per block: as many as keep every workgroup on a compute unit of its own (one unit
// draws only about 40 GB/s from memory, so the matrix has to be spread over all of them, and a
// second workgroup on a unit would finish last; measured on the 4096 x 6144 projection, 48 column
// blocks: 4 slices 14.75 us, 5: 14.5, 6: 16.7, 7: 16.6, 8: 15.9), at least one tile per wave, at
// most 64.  The slices are whole tiles and need not be equal.
int choose_k_splits(int64_t blocks, int64_t K) {
  static const int n_cu = [] {
    int dev = 0, n = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 256;
    return n > 0 ? n : 256;
  }();
  const int64_t max_splits = std::max<int64_t>(1, K / (kTileK * kWaves));
  return (int)std::min<int64_t>(std::min(std::max<int64_t>(1, n_cu / blocks), max_splits), 64);
}

size_t ticket_area(int64_t blocks) { return (size_t)((blocks * 4 + 255) / 256 * 256); }

}  // namespace

extern "C" {

size_t vt_gemm_store_workspace(int64_t M, int64_t N, int64_t K) {
  if (M < 1 || N < 1 || K < 1) return 0;
  const int64_t blocks = ((M + kBM - 1) / kBM) * ((N + kBN - 1) / kBN);
  return ticket_area(blocks) + (size_t)blocks * choose_k_splits(blocks, K) * kBM * kBN * sizeof(float);
}

int vt_gemm_store_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace || (uintptr_t)workspace % 16) return fail(VT_ERR_INVALID_ARG, "vt_gemm_store_workspace_init: NULL or misaligned workspace");
  const size_t words = workspace_bytes / 4;
  if (words == 0) return VT_OK;
  hipLaunchKernelGGL(k_zero_store_ws, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream, (uint32_t*)workspace, words);
  return check_launch("vt_gemm_store_workspace_init");
}

int vt_gemm_store(const vt_desc* A, const vt_desc* B, const vt_desc* C, void* workspace, size_t workspace_bytes,
                  void* stream) {
  if (!A || !B || !C || !workspace) return fail(VT_ERR_INVALID_ARG, "vt_gemm_store: NULL argument");
  if (A->dtype == VT_F32 || B->dtype != A->dtype || C->dtype != A->dtype)
    return fail(VT_ERR_INVALID_ARG, "vt_gemm_store: A, B and the output must share a 16-bit dtype");
  if (A->shape.size() != 2 || B->shape.size() != 2 || C->shape.size() != 2)
    return fail(VT_ERR_SHAPE, "vt_gemm_store: A [M,K], B [K,N] and the output [M,N] must be 2-D");
  const int64_t M = A->shape[0], K = A->shape[1], N = B->shape[1];
  if (B->shape[0] != K || C->shape[0] != M || C->shape[1] != N) return fail(VT_ERR_SHAPE, "vt_gemm_store: shapes do not match");
  if (M < 1 || N < 8 || K < 8 || N % 8 || K % 8) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: N and K must be multiples of 8");
  if (M >= (1ll << 20) || N >= (1ll << 30) || K >= (1ll << 30)) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: extents too large");

  int rc0 = check_store_map(*C, "vt_gemm_store");
  if (rc0 != VT_OK) return rc0;
  // many rows: the tiled GEMM with the map applied in its store stage (this kernel would read B
  // once per 16 rows)
  if (M > kTiledFrom) return gemm_store_launch(*A, *B, *C, (hipStream_t)stream);

  StoreParams P;
  memset(&P, 0, sizeof(P));
  // A: one piece, rows through a map, K contiguous
  if (A->pieces.size() != 1 || !A->pieces[0].v.lower.empty()) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: A must be a single piece with one index stage");
  {
    const Piece& p = A->pieces[0];
    int rc = make_axis(*A, p, 0, 1, &P.a_row, "vt_gemm_store: A rows");
    if (rc != VT_OK) return rc;
    AxisMap<3> ac;
    rc = make_axis(*A, p, 1, 2, &ac, "vt_gemm_store: A columns");
    if (rc != VT_OK) return rc;
    const vt_source& s = A->sources[p.src];
    if (!s.ptr) return fail(VT_ERR_INVALID_ARG, "vt_gemm_store: A source without a device pointer");
    P.a = static_cast<const char*>(s.ptr) + p.v.base * 2;
    if (!(ac.nd == 1 && ac.stride[2] == 1) || (uintptr_t)P.a % 8 || !strides_multiple_of(P.a_row, 4, 0))
      return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: rows of A must be contiguous and 8-byte aligned");
  }
  // B: a plain row-major matrix (rows one stride apart, columns contiguous)
  if (B->pieces.size() != 1 || !B->pieces[0].v.lower.empty()) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: B must be a single piece with one index stage");
  {
    const Piece& p = B->pieces[0];
    AxisMap<3> br, bc;
    int rc = make_axis(*B, p, 0, 1, &br, "vt_gemm_store: B rows");
    if (rc != VT_OK) return rc;
    rc = make_axis(*B, p, 1, 2, &bc, "vt_gemm_store: B columns");
    if (rc != VT_OK) return rc;
    const vt_source& s = B->sources[p.src];
    if (!s.ptr) return fail(VT_ERR_INVALID_ARG, "vt_gemm_store: B source without a device pointer");
    P.b = static_cast<const char*>(s.ptr) + p.v.base * 2;
    if (br.nd != 1 || !(bc.nd == 1 && bc.stride[2] == 1) || br.stride[2] % 8 || br.stride[2] < 0 || (uintptr_t)P.b % 16)
      return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: B must be a row-major matrix with 16-byte aligned rows");
    P.ldb = br.stride[2];
    if (P.ldb * 2 * 16 + N * 2 >= (1ll << 32)) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: rows of B too far apart");
  }
  // the output: pieces that split the columns
  int rc = VT_OK;
  if (C->pieces.size() > (size_t)kMaxOutPieces) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: more than 4 output pieces");
  {
    std::vector<const Piece*> ps;
    for (const Piece& p : C->pieces) ps.push_back(&p);
    std::sort(ps.begin(), ps.end(), [](const Piece* x, const Piece* y) { return x->lo[1] < y->lo[1]; });
    int64_t expect = 0;
    for (size_t i = 0; i < ps.size(); ++i) {
      const Piece& p = *ps[i];
      if (p.lo[0] != 0 || p.hi[0] != M || p.lo[1] != expect) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: output pieces must split the columns only");
      expect = p.hi[1];
      OutPiece& o = P.out[i];
      rc = make_axis(*C, p, 0, 1, &o.row, "vt_gemm_store: output rows");
      if (rc != VT_OK) return rc;
      rc = make_axis(*C, p, 1, 2, &o.col, "vt_gemm_store: output columns");
      if (rc != VT_OK) return rc;
      const vt_source& s = C->sources[p.src];
      if (!s.ptr) return fail(VT_ERR_INVALID_ARG, "vt_gemm_store: output tensor without a device pointer");
      o.base = static_cast<char*>(s.ptr) + p.v.base * 2;
      o.col_lo = (int32_t)p.lo[1];
      o.col_hi = (int32_t)p.hi[1];
    }
    if (expect != N) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: output pieces do not cover the columns");
    P.n_out = (int32_t)ps.size();
  }
  const int64_t rbs = (M + kBM - 1) / kBM, cbs = (N + kBN - 1) / kBN;
  if (rbs > 65535 || cbs > 65535) return fail(VT_ERR_UNSUPPORTED, "vt_gemm_store: too many blocks");
  const int ns = choose_k_splits(rbs * cbs, K);
  int kps = (int)((K + ns - 1) / ns);
  kps = (kps + kTileK - 1) / kTileK * kTileK;
  const int ns_eff = (int)((K + kps - 1) / kps);
  const size_t need = ticket_area(rbs * cbs) + (size_t)rbs * cbs * ns_eff * kBM * kBN * sizeof(float);
  if (workspace_bytes < need) return fail(VT_ERR_INVALID_ARG, "vt_gemm_store: workspace too small");
  if ((uintptr_t)workspace % 16) return fail(VT_ERR_INVALID_ARG, "vt_gemm_store: misaligned workspace");
  P.M = (int32_t)M;
  P.N = (int32_t)N;
  P.K = (int32_t)K;
  P.n_splits = ns_eff;
  P.k_per_split = kps;
  P.tickets = static_cast<uint32_t*>(workspace);
  P.partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + ticket_area(rbs * cbs));
  dim3 grid((unsigned)ns_eff, (unsigned)cbs, (unsigned)rbs);
  hipStream_t st = (hipStream_t)stream;
  if (A->dtype == VT_BF16) hipLaunchKernelGGL((k_gemm_store<bf16_t>), grid, dim3(kWaves * 64), 0, st, P);
  else hipLaunchKernelGGL((k_gemm_store<f16_t>), grid, dim3(kWaves * 64), 0, st, P);
  return check_launch("vt_gemm_store");
}

}  // extern "C"
