// Split-K flash-decoding attention for grouped queries that reads Q, K and V through
// virtual-tensor descriptors (Sec. 3.1: the attention kernel reads the un-expanded cache and
// the freshly projected K/V rows where the producer left them).  gfx950, wave64, MFMA.
//
// Work split: one workgroup per (batch b, kv head g, context split s); WAVES waves share the
// split's rows in tiles of 32.  All G query heads of the group are served from one read of
// K and V (the broadcast digit of the descriptor, i.e. the Expand that is never executed).
//
// Per tile of 32 context rows and per wave:
//   S^T = K . Q^T   on v_mfma_f32_16x16x32 (rows = context, cols = the group's heads, padded
//                   to 16).  K rows are fetched with fully coalesced 16-byte loads (16 lanes
//                   per 256-byte row), staged through an XOR-swizzled LDS tile and read back in
//                   the matrix-core operand layout without bank conflicts.
//   online softmax  in the accumulator layout (lane = head, 4 rows per 16-row block).
//   O^T += V^T . P^T on the same instruction.  V never touches LDS: each lane loads 8 rows of
//                   its own 8-column chunk (again whole rows per 16 lanes), transposes the 8x8
//                   block inside its registers (v_perm_b32) and feeds it as the A operand;
//                   the contraction index is permuted identically for P, which the softmax
//                   already holds in exactly that layout.
// A second, tiny kernel merges the per-split partial results.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

#include "vt_device.h"
#include "vt_numeric.h"

using namespace vt;

namespace {

constexpr int kD = 128;          // head dim
constexpr int kTile = 32;        // context rows per wave step
constexpr int kMaxAttnPieces = 4;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct AttnPiece {
  const char* ptr;       // element (b=0, g=0, t=t_lo, d=0)
  int64_t sb, sh;        // bytes per batch / per kv head
  uint32_t st;           // bytes per context row
  int32_t t_lo, t_hi;
};
struct AttnOperand {
  AttnPiece pc[kMaxAttnPieces];
  int32_t n;
};
struct AttnParams {
  AttnOperand K, V;
  const char* q_ptr;
  int64_t q_sb, q_sh;    // bytes
  int32_t B, Hkv, G, S, n_splits, rows_per_split;
  float scale_log2;      // softmax scale * log2(e)
  float* ws_o;           // [B, Hkv, n_splits, G, D]
  float* ws_ml;          // [B, Hkv, n_splits, G, 2]
};

template <typename T>
struct Mfma;
template <>
struct Mfma<bf16_t> {
  typedef bf16x8 vec;
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
  }
};
template <>
struct Mfma<f16_t> {
  typedef f16x8 vec;
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    _Float16 l = (_Float16)lo, h = (_Float16)hi;
    return (uint32_t)__builtin_bit_cast(uint16_t, l) | ((uint32_t)__builtin_bit_cast(uint16_t, h) << 16);
  }
};

// Address of context row t of operand X for (b, g); t is clamped by the caller to [0, S).
__device__ __forceinline__ const char* row_address(const AttnOperand& X, int b, int g, int t) {
  const char* base = X.pc[0].ptr + b * X.pc[0].sb + g * X.pc[0].sh;
  uint32_t st = X.pc[0].st;
  int lo = X.pc[0].t_lo;
#pragma unroll
  for (int i = 1; i < kMaxAttnPieces; ++i) {
    if (i < X.n && t >= X.pc[i].t_lo) {
      base = X.pc[i].ptr + b * X.pc[i].sb + g * X.pc[i].sh;
      st = X.pc[i].st;
      lo = X.pc[i].t_lo;
    }
  }
  return base + (uint64_t)(uint32_t)(t - lo) * st;
}

template <typename T, int WAVES>
__global__ void __launch_bounds__(WAVES * 64) k_decode_attn(const AttnParams P) {
  typedef Mfma<T> M;
  typedef typename M::vec opvec;
  __shared__ uint4 lds[WAVES][kTile * 16];   // per wave: 32 rows x 16 chunks of 16 bytes, swizzled

  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int l16 = lane & 15, lg = lane >> 4;
  const int t_begin = split * P.rows_per_split;
  const int t_end = min(P.S, t_begin + P.rows_per_split);
  const int n_tiles = (t_end - t_begin + kTile - 1) / kTile;

  // Q^T operand: lane (head l16, k-group lg) holds 8 consecutive d for each of the 4 k-steps
  opvec qreg[4];
  {
    const char* qp = P.q_ptr + b * P.q_sb + (int64_t)(g * P.G + l16) * P.q_sh;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (l16 < P.G) raw = *reinterpret_cast<const uint4*>(qp + (kk * 32 + lg * 8) * 2);
      qreg[kk] = __builtin_bit_cast(opvec, raw);
    }
  }

  float m_run = -1.0e30f;   // running max (log2 domain) of head l16, identical in the 4 lane groups
  float l_run = 0.0f;       // this lane's share of the running denominator
  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint4 kst[8], vst[8];
  auto issue_loads = [&](int tile) {
    const int r0 = t_begin + tile * kTile;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int tk = min(r0 + 4 * j + lg, t_end - 1);                          // K: instruction j covers rows 4j..4j+3
      kst[j] = *reinterpret_cast<const uint4*>(row_address(P.K, b, g, tk) + l16 * 16);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int tv = min(r0 + (j >> 2) * 16 + lg * 4 + (j & 3), t_end - 1);    // V: contraction slot j of lane group lg
      vst[j] = *reinterpret_cast<const uint4*>(row_address(P.V, b, g, tv) + l16 * 16);
    }
  };

  uint4* my_lds = lds[wave];
  if (wave < n_tiles) issue_loads(wave);
  for (int tile = wave; tile < n_tiles; tile += WAVES) {
    const int r0 = t_begin + tile * kTile;
    // ---- stage K through LDS (swizzle: chunk c of row r sits at unit c ^ (r & 15))
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int r = 4 * j + lg;
      my_lds[r * 16 + (l16 ^ (r & 15))] = kst[j];
    }
    uint4 vcur[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) vcur[j] = vst[j];
    if (tile + WAVES < n_tiles) issue_loads(tile + WAVES);

    // ---- S^T = K . Q^T : two 16-row blocks, 4 k-steps each
    f32x4 s[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      int r = u * 16 + l16;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        uint4 raw = my_lds[r * 16 + ((kk * 4 + lg) ^ l16)];
        s[u] = M::run(__builtin_bit_cast(opvec, raw), qreg[kk], s[u]);
      }
    }
    // ---- online softmax; lane holds head l16, rows r0 + u*16 + lg*4 + i
    float sv[8];
    float tmax = -1.0e30f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int t = r0 + u * 16 + lg * 4 + i;
        float x = s[u][i] * P.scale_log2;
        x = t < t_end ? x : -1.0e30f;
        sv[u * 4 + i] = x;
        tmax = fmaxf(tmax, x);
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    float pv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int t = r0 + (j >> 2) * 16 + lg * 4 + (j & 3);
      float p = t < t_end ? exp2f(sv[j] - m_new) : 0.f;
      pv[j] = p;
      psum += p;
    }
    l_run = l_run * alpha + psum;
    uint4 praw = make_uint4(M::pack2(pv[0], pv[1]), M::pack2(pv[2], pv[3]), M::pack2(pv[4], pv[5]),
                            M::pack2(pv[6], pv[7]));
    const opvec pop = __builtin_bit_cast(opvec, praw);
    // ---- O^T += V^T . P^T : transpose the lane's 8x8 block, one MFMA per column e
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
      uint32_t w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t* lo = reinterpret_cast<const uint32_t*>(&vcur[2 * u]);
        const uint32_t* hi = reinterpret_cast<const uint32_t*>(&vcur[2 * u + 1]);
        w[u] = __builtin_amdgcn_perm(hi[e >> 1], lo[e >> 1], sel);
      }
      uint4 traw = make_uint4(w[0], w[1], w[2], w[3]);
      f32x4 a = acc[e];
      a[0] *= alpha; a[1] *= alpha; a[2] *= alpha; a[3] *= alpha;
      acc[e] = M::run(__builtin_bit_cast(opvec, traw), pop, a);
    }
  }

  // ---- merge the waves of the workgroup through LDS, then write the split's partial result
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  __syncthreads();                       // every wave is done with its K tile
  __shared__ float red_ml[WAVES * 16 * 2];                // [WAVES][16][2]
  float* red_o = reinterpret_cast<float*>(&lds[0][0]);    // [WAVES][G][D] floats: at most the K tiles' 32 KB
  const int G = P.G;
  if (l16 < G) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
      for (int i = 0; i < 4; ++i) red_o[(wave * G + l16) * kD + (lg * 4 + i) * 8 + e] = acc[e][i];
    if (lg == 0) {
      red_ml[(wave * 16 + l16) * 2 + 0] = m_run;
      red_ml[(wave * 16 + l16) * 2 + 1] = l_run;
    }
  }
  __syncthreads();
  const size_t unit = ((size_t)(b * P.Hkv + g) * P.n_splits + split);
  for (int idx = threadIdx.x; idx < G * kD; idx += WAVES * 64) {
    int h = idx / kD;
    float mx = -1.0e30f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) mx = fmaxf(mx, red_ml[(w * 16 + h) * 2]);
    float o = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      float sc = exp2f(red_ml[(w * 16 + h) * 2] - mx);
      o += red_o[(w * G + h) * kD + (idx - h * kD)] * sc;
      l += red_ml[(w * 16 + h) * 2 + 1] * sc;
    }
    P.ws_o[unit * G * kD + idx] = o;
    if (idx == h * kD) {
      P.ws_ml[(unit * G + h) * 2 + 0] = mx;
      P.ws_ml[(unit * G + h) * 2 + 1] = l;
    }
  }
}

// out[b, hq, :] = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M); one block of 128 threads per head.
template <typename T>
__global__ void __launch_bounds__(kD) k_decode_combine(const float* __restrict__ ws_o, const float* __restrict__ ws_ml,
                                                       T* __restrict__ out, float* __restrict__ lse, int G, int n_splits) {
  const int hq = blockIdx.x;            // b * Hq + h
  const int unit = hq / G, j = hq - unit * G;
  const int d = threadIdx.x;
  float mx = -1.0e30f;
  for (int s = 0; s < n_splits; ++s) mx = fmaxf(mx, ws_ml[(((size_t)unit * n_splits + s) * G + j) * 2]);
  float o = 0.f, l = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    size_t u = (size_t)unit * n_splits + s;
    float sc = exp2f(ws_ml[(u * G + j) * 2] - mx);
    o += ws_o[(u * G + j) * kD + d] * sc;
    l += ws_ml[(u * G + j) * 2 + 1] * sc;
  }
  out[(size_t)hq * kD + d] = from_float<T>(o / l);
  if (lse && d == 0) lse[hq] = (mx + log2f(l)) * 0.6931471805599453f;
}

// ---------------------------------------------------------------- host: descriptor -> plan
struct HeadMap {
  int64_t stride;   // elements per kv head
  int64_t G;        // query heads per kv head (trailing broadcast digits)
};

bool single_plain(const std::vector<Digit>& g, int64_t* stride) {
  if (g.empty()) {
    *stride = 0;
    return true;
  }
  if (g.size() == 1 && g[0].table < 0) {
    *stride = g[0].stride;
    return true;
  }
  return false;
}

// Trailing zero-stride digits of the head group = heads that share rows.
int64_t broadcast_factor(const std::vector<Digit>& g) {
  int64_t f = 1;
  for (int k = (int)g.size() - 1; k >= 0 && g[k].stride == 0 && g[k].table < 0; --k) f *= g[k].radix;
  return f;
}

int plan_operand(const vt_desc& d, const char* name, int64_t G, AttnOperand* out) {
  const int esz = 2;
  if (d.pieces.size() > (size_t)kMaxAttnPieces) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": more than 4 pieces along the context");
  std::vector<const Piece*> ps;
  for (const Piece& p : d.pieces) ps.push_back(&p);
  std::sort(ps.begin(), ps.end(), [](const Piece* a, const Piece* b) { return a->lo[2] < b->lo[2]; });
  int64_t expect = 0;
  out->n = (int)ps.size();
  for (size_t i = 0; i < ps.size(); ++i) {
    const Piece& p = *ps[i];
    for (int dim : {0, 1, 3})
      if (p.lo[dim] != 0 || p.hi[dim] != d.shape[dim]) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": pieces must split the context dim only");
    if (p.lo[2] != expect) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": pieces do not tile the context");
    expect = p.hi[2];
    if (!p.v.lower.empty()) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": stacked index stages");
    int64_t sb, st, sd;
    if (!single_plain(p.v.groups[0], &sb) || !single_plain(p.v.groups[2], &st) || !single_plain(p.v.groups[3], &sd))
      return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": batch, context and feature dims must each be one strided digit");
    if (sd != 1) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": rows must be contiguous along the head dim");
    // head group: [kv heads (stride sh)] x [G broadcast]
    std::vector<Digit> hg = p.v.groups[1];
    int64_t left = G;
    while (left > 1) {
      if (hg.empty() || hg.back().stride != 0 || hg.back().table >= 0 || (left % hg.back().radix != 0 && hg.back().radix % left != 0))
        return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": head broadcast structure not recognised");
      if (hg.back().radix <= left) {
        left /= hg.back().radix;
        hg.pop_back();
      } else {
        hg.back().radix /= left;
        left = 1;
      }
    }
    int64_t sh;
    if (!single_plain(hg, &sh)) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": kv-head dim must be one strided digit");
    const vt_source& src = d.sources[p.src];
    if (!src.ptr) return fail(VT_ERR_INVALID_ARG, std::string(name) + ": source without a device pointer");
    AttnPiece& a = out->pc[i];
    a.ptr = static_cast<const char*>(src.ptr) + p.v.base * esz;
    a.sb = sb * esz;
    a.sh = sh * esz;
    if (st * esz >= (1ll << 32) || st < 0) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": context stride too large");
    a.st = (uint32_t)(st * esz);
    a.t_lo = (int32_t)p.lo[2];
    a.t_hi = (int32_t)p.hi[2];
    if ((uintptr_t)a.ptr % 16 || a.sb % 16 || a.sh % 16 || a.st % 16)
      return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": rows are not 16-byte aligned");
  }
  if (expect != d.shape[2]) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": pieces do not cover the context");
  return VT_OK;
}

// About two workgroups per compute unit, and at least one 32-row tile per wave.
int choose_splits(int units, int S, int n_splits) {
  if (n_splits > 0) return n_splits;
  int max_splits = std::max(1, (S + 127) / 128);
  int want = std::max(1, (512 + units - 1) / units);
  return std::min(want, max_splits);
}

constexpr int kWaves = 4;

}  // namespace

extern "C" {

size_t vt_decode_attn_workspace(int B, int Hq, int D, int S, int n_splits) {
  if (B < 1 || Hq < 1 || D < 1 || S < 1 || n_splits < 0) return 0;
  // an upper bound that does not need the grouping: the fewest kv heads (16 query heads each)
  // give the most splits
  int ns = choose_splits(B * std::max(1, Hq / 16), S, n_splits);
  return (size_t)B * Hq * ns * ((size_t)D + 2) * sizeof(float);
}

int vt_decode_attn(const vt_desc* Q, const vt_desc* K, const vt_desc* V, float scale, void* out, float* lse,
                   void* workspace, size_t workspace_bytes, int n_splits, void* stream) {
  if (!Q || !K || !V || !out || !workspace) return fail(VT_ERR_INVALID_ARG, "vt_decode_attn: NULL argument");
  if (Q->dtype == VT_F32 || K->dtype != Q->dtype || V->dtype != Q->dtype)
    return fail(VT_ERR_INVALID_ARG, "vt_decode_attn: Q, K, V must share a 16-bit dtype");
  if (Q->shape.size() != 4 || K->shape.size() != 4 || V->shape != K->shape)
    return fail(VT_ERR_SHAPE, "vt_decode_attn: Q must be [B,Hq,1,D], K and V [B,Hq,S,D]");
  const int64_t B = K->shape[0], Hq = K->shape[1], S = K->shape[2], D = K->shape[3];
  if (Q->shape[0] != B || Q->shape[1] != Hq || Q->shape[2] != 1 || Q->shape[3] != D)
    return fail(VT_ERR_SHAPE, "vt_decode_attn: Q does not match K");
  if (D != kD) return fail(VT_ERR_UNSUPPORTED, "vt_decode_attn: head dim must be 128");
  if (B > 65535 || Hq > 65535 || S >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, "vt_decode_attn: extents too large");
  if (n_splits < 0) return fail(VT_ERR_INVALID_ARG, "vt_decode_attn: n_splits < 0");

  // query heads that share K/V rows: common broadcast factor over all pieces of K and V
  int64_t G = 0;
  for (const vt_desc* X : {K, V})
    for (const Piece& p : X->pieces) {
      int64_t f = broadcast_factor(p.v.groups[1]);
      G = G == 0 ? f : std::gcd(G, f);
    }
  if (G < 1) G = 1;
  while (G > 16 || Hq % G) --G;      // the matrix-core tile holds at most 16 heads
  AttnParams P;
  memset(&P, 0, sizeof(P));
  int rc = plan_operand(*K, "K", G, &P.K);
  if (rc != VT_OK) return rc;
  rc = plan_operand(*V, "V", G, &P.V);
  if (rc != VT_OK) return rc;
  // Q: one piece, one stage, contiguous rows
  if (Q->pieces.size() != 1 || !Q->pieces[0].v.lower.empty()) return fail(VT_ERR_UNSUPPORTED, "Q: must be a single strided piece");
  {
    const Piece& p = Q->pieces[0];
    int64_t sb, sh, sd;
    if (!single_plain(p.v.groups[0], &sb) || !single_plain(p.v.groups[1], &sh) || !single_plain(p.v.groups[3], &sd) || sd != 1)
      return fail(VT_ERR_UNSUPPORTED, "Q: batch and head dims must each be one strided digit, rows contiguous");
    const vt_source& src = Q->sources[p.src];
    if (!src.ptr) return fail(VT_ERR_INVALID_ARG, "Q: source without a device pointer");
    P.q_ptr = static_cast<const char*>(src.ptr) + p.v.base * 2;
    P.q_sb = sb * 2;
    P.q_sh = sh * 2;
    if ((uintptr_t)P.q_ptr % 16 || P.q_sb % 16 || P.q_sh % 16) return fail(VT_ERR_UNSUPPORTED, "Q: rows are not 16-byte aligned");
  }
  const int Hkv = (int)(Hq / G);
  const int ns = choose_splits((int)B * Hkv, (int)S, n_splits);
  int rows = (int)((S + ns - 1) / ns);
  rows = (rows + kTile - 1) / kTile * kTile;
  const int ns_eff = (int)((S + rows - 1) / rows);
  const size_t need = (size_t)B * Hq * ns_eff * ((size_t)kD + 2) * sizeof(float);
  if (workspace_bytes < need) return fail(VT_ERR_INVALID_ARG, "vt_decode_attn: workspace too small");
  if ((uintptr_t)workspace % 16 || (uintptr_t)out % 2) return fail(VT_ERR_INVALID_ARG, "vt_decode_attn: misaligned workspace or out");
  P.B = (int)B;
  P.Hkv = Hkv;
  P.G = (int)G;
  P.S = (int)S;
  P.n_splits = ns_eff;
  P.rows_per_split = rows;
  P.scale_log2 = scale * 1.4426950408889634f;
  P.ws_o = static_cast<float*>(workspace);
  P.ws_ml = P.ws_o + (size_t)B * Hq * ns_eff * kD;
  hipStream_t st = (hipStream_t)stream;
  dim3 grid(ns_eff, Hkv, (unsigned)B);
  if (Q->dtype == VT_BF16) {
    hipLaunchKernelGGL((k_decode_attn<bf16_t, kWaves>), grid, dim3(kWaves * 64), 0, st, P);
  } else {
    hipLaunchKernelGGL((k_decode_attn<f16_t, kWaves>), grid, dim3(kWaves * 64), 0, st, P);
  }
  rc = check_launch("vt_decode_attn");
  if (rc != VT_OK) return rc;
  if (Q->dtype == VT_BF16) {
    hipLaunchKernelGGL(k_decode_combine<bf16_t>, dim3((unsigned)(B * Hq)), dim3(kD), 0, st, P.ws_o, P.ws_ml, (bf16_t*)out, lse,
                       (int)G, ns_eff);
  } else {
    hipLaunchKernelGGL(k_decode_combine<f16_t>, dim3((unsigned)(B * Hq)), dim3(kD), 0, st, P.ws_o, P.ws_ml, (f16_t*)out, lse,
                       (int)G, ns_eff);
  }
  return check_launch("vt_decode_attn(combine)");
}

}  // extern "C"
