// Pure data movement through a descriptor (vt_materialize, vt_copy_op) and the
// elementwise / reduction consumer (vt_elementwise).  gfx950, wave64.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "vt_device.h"
#include "vt_kernarg.h"
#include "vt_numeric.h"
#include "vt_profile.h"

using namespace vt;

// ------------------------------------------------------------------------------------------
// Gather-copy: thread t moves one vector of VB bytes.  The host guarantees that aligned
// vectors never straddle a piece, a run or a row of the virtual tensor.
// ------------------------------------------------------------------------------------------
template <typename V>
__global__ void __launch_bounds__(256) k_materialize(const DevDesc D, V* __restrict__ dst, uint32_t inner_vecs,
                                                     uint32_t vec_elems, uint32_t outer) {
  __shared__ DevDesc map[1];
  {
    const DevDesc* const from[1] = {&D};
    stage_maps(map, from);
  }
  const DevDesc& M = map[0];
  uint32_t vi = blockIdx.x * 256u + threadIdx.x;
  if (vi >= inner_vecs) return;
  for (uint32_t o = blockIdx.y; o < outer; o += gridDim.y) {
    int64_t off;
    const void* ptr;
    vtd_eval(M, o, vi * vec_elems, &off, &ptr);
    dst[(size_t)o * inner_vecs + vi] = ld_global<V>(static_cast<const char*>(ptr) + off * M.elem_size);
  }
}

// The reverse direction: every element of the virtual tensor S is written to the place the map
// of D names (D one to one).  The explicit Split / Reshape / ScatterND of the materialized path.
template <typename V>
__global__ void __launch_bounds__(256) k_scatter(const DevDesc S, const DevDesc D, uint32_t inner_vecs, uint32_t vec_elems,
                                                 uint32_t outer) {
  __shared__ DevDesc maps[2];
  {
    const DevDesc* const from[2] = {&S, &D};
    stage_maps(maps, from);
  }
  uint32_t vi = blockIdx.x * 256u + threadIdx.x;
  if (vi >= inner_vecs) return;
  for (uint32_t o = blockIdx.y; o < outer; o += gridDim.y) {
    int64_t so, dof;
    const void *sp, *dp;
    vtd_eval(maps[0], o, vi * vec_elems, &so, &sp);
    vtd_eval(maps[1], o, vi * vec_elems, &dof, &dp);
    st_global<V>(static_cast<char*>(const_cast<void*>(dp)) + dof * maps[1].elem_size,
                 ld_global<V>(static_cast<const char*>(sp) + so * maps[0].elem_size));
  }
}

// ------------------------------------------------------------------------------------------
// Block-wise copy (Sec. 4.2, block-wise virtual tensor I/O): the tensor is cut into aligned
// blocks of BL * 16 bytes, each one contiguous range of one source (the host's block analysis
// guarantees it).  A wave takes `rb` consecutive blocks per round: every lane applies the map
// ONCE, to the first element of "its" block; the block addresses are then handed round with
// lane shuffles and all 64 lanes move 64 / BL blocks per instruction, 16 bytes each, so that the
// index arithmetic is paid once per block and not once per vector.  SCATTER: the destination
// goes through a map as well (store direction), otherwise it is dense.
// ------------------------------------------------------------------------------------------
// Every byte a copy moves is read once: streaming loads keep it from displacing other lines
// (blocks of 256 bytes and less measured faster with ordinary loads).
template <bool STREAM = true>
__device__ __forceinline__ uint4 load_once(uint64_t addr) { return ld_global<uint4, STREAM>(addr); }

__device__ __forceinline__ uint64_t shfl_u64(uint64_t v, int src_lane) {
  const uint32_t lo = __shfl((uint32_t)v, src_lane, 64), hi = __shfl((uint32_t)(v >> 32), src_lane, 64);
  return ((uint64_t)hi << 32) | lo;
}

typedef __attribute__((address_space(4))) const BlockWalk* kernarg_block_walk_t;   // a walk inside the kernel-argument segment

// The body shared by the two kernels below: src_of(o, blk) / dst_of(o, blk) give the address of a block.
template <int BL, bool SCATTER, typename SrcOf, typename DstOf>
__device__ __forceinline__ void copy_blocks_body(char* __restrict__ dst, uint32_t inner_blocks, uint32_t rb, uint32_t outer, SrcOf src_of,
                                                 DstOf dst_of) {
  constexpr int G = 64 / BL;                         // blocks moved by one instruction
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wv = blockIdx.x * 4u + (threadIdx.x >> 6);
  const uint32_t first = wv * rb;                    // this wave's blocks: [first, first + rb)
  if (first >= inner_blocks) return;
  const uint32_t n_here = min(rb, inner_blocks - first);
  const uint32_t sub = lane / BL, c16 = (lane % BL) * 16u;
  const uint32_t iters = (n_here + G - 1) / G;
  // the address of block `blk` of this round, from the lane that applied the map to it
  auto addr_of = [&](uint64_t mine, uint32_t blk) -> uint64_t {
    if (BL == 64) {                                  // one block per instruction: a wave-uniform address
      const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)mine, (int)blk), hi = __builtin_amdgcn_readlane((uint32_t)(mine >> 32), (int)blk);
      return ((uint64_t)hi << 32) | lo;
    }
    return shfl_u64(mine, (int)min(blk, 63u));
  };
  for (uint32_t o = blockIdx.y; o < outer; o += gridDim.y) {
    const uint32_t mine = first + min(lane, n_here - 1);
    const uint64_t src_addr = src_of(o, mine);
    uint64_t dst_addr = 0;
    if (SCATTER) dst_addr = dst_of(o, mine);
    // dense destination: block b of the round sits at a fixed distance from the round's first block
    const uint64_t dense0 = reinterpret_cast<uint64_t>(dst) + ((uint64_t)o * inner_blocks + first) * (uint64_t)(BL * 16) + c16;
    uint32_t j0 = 0;
    // whole batches of sixteen instructions, nothing to guard: sixteen loads in flight, then their stores
    for (; j0 + 16 <= iters && (j0 + 16) * G <= n_here; j0 += 16) {
      uint4 v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = load_once<(BL >= 32)>(addr_of(src_addr, (j0 + u) * G + sub) + c16);
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const uint32_t blk = (j0 + u) * G + sub;
        const uint64_t a = SCATTER ? addr_of(dst_addr, blk) + c16 : dense0 + (uint64_t)blk * (BL * 16);
        st_global<uint4>(a, v[u]);
      }
    }
    for (; j0 < iters; j0 += 4) {                     // the remainder, four at a time, guarded
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t blk = (j0 + u) * G + sub;
        const uint64_t a = addr_of(src_addr, min(blk, n_here - 1)) + c16;
        if (blk < n_here) v[u] = load_once<(BL >= 32)>(a);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t blk = (j0 + u) * G + sub;
        const uint64_t a = SCATTER ? addr_of(dst_addr, min(blk, n_here - 1)) + c16 : dense0 + (uint64_t)blk * (BL * 16);
        if (blk < n_here) st_global<uint4>(a, v[u]);
      }
    }
  }
}

template <int BL, bool SCATTER>
__global__ void __launch_bounds__(256) k_copy_blocks(const DevDesc S, const DevDesc D, char* __restrict__ dst,
                                                     uint32_t inner_blocks, uint32_t block_elems, uint32_t rb, uint32_t outer) {
  // Small blocks: the maps are evaluated often for the bytes moved, and are read from an LDS copy.
  // Blocks of 1 KB: one evaluation moves a kilobyte, and the copy to LDS with its barrier costs
  // more than it saves (measured on the gather of 28 KB rows: 10 % slower with it).
  constexpr bool STAGE = BL < 64;
  __shared__ DevDesc staged[STAGE ? (SCATTER ? 2 : 1) : 1];
  if (STAGE) {
    if (SCATTER) {
      const DevDesc* const from[2] = {&S, &D};
      stage_maps(reinterpret_cast<DevDesc*>(staged), from);
    } else {
      const DevDesc* const from[1] = {&S};
      stage_maps(reinterpret_cast<DevDesc*>(staged), from);
    }
  }
  const DevDesc& MS = STAGE ? staged[0] : S;
  const DevDesc& MD = STAGE ? staged[SCATTER ? 1 : 0] : D;
  auto at = [&](const DevDesc& M, uint32_t o, uint32_t blk) -> uint64_t {
    int64_t off;
    const void* ptr;
    vtd_eval(M, o, blk * block_elems, &off, &ptr);
    return reinterpret_cast<uint64_t>(ptr) + (uint64_t)(off * M.elem_size);
  };
  copy_blocks_body<BL, SCATTER>(dst, inner_blocks, rb, outer, [&](uint32_t o, uint32_t blk) { return at(MS, o, blk); },
                                [&](uint32_t o, uint32_t blk) { return at(MD, o, blk); });
}

// The same copy for maps that resolve into the term form (BlockWalk): a block's address costs a
// dozen instructions per term, the terms are read from the arguments where they are used.
template <int BL, bool SCATTER>
__global__ void __launch_bounds__(256) k_copy_blocks_walk(const BlockWalk WS, const BlockWalk WD, char* __restrict__ dst,
                                                          uint32_t inner_blocks, uint32_t rb) {
  // the pieces are read one after the other, each a few wide reads: all their lines are requested at once first
  static_assert(2 * sizeof(BlockWalk) >= 26 * 64 + 4 && 2 * sizeof(BlockWalk) <= 27 * 64, "the lines requested below are those of the two walks");
  warm_kernarg_27();
  kernarg_block_walk_t kw = (kernarg_block_walk_t)__builtin_amdgcn_kernarg_segment_ptr();   // WS, then WD
  asm volatile("" : "+s"(kw));
  (void)WS, (void)WD;
  copy_blocks_body<BL, SCATTER>(dst, inner_blocks, rb, 1u, [&](uint32_t, uint32_t blk) { return walk_address(kw, blk); },
                                [&](uint32_t, uint32_t blk) { return walk_address(kw + 1, blk); });
}

// A map that is one contiguous range of one source (Def. 5 with minimal contiguous dimension 1:
// a Reshape, a Slice or Split along the outermost dim, ...): a plain vector copy, no index work.
__global__ void __launch_bounds__(256) k_copy_flat(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n_vec) {
  // a workgroup moves consecutive 16 KB chunks: four loads of 4 KB in flight per wave, then their stores
  const size_t chunks = n_vec / 1024;
  for (size_t c = blockIdx.x; c < chunks; c += gridDim.x) {
    const size_t i = c * 1024 + threadIdx.x;
    const uint4 a = ld_global<uint4, true>(src + i), b = ld_global<uint4, true>(src + i + 256), e = ld_global<uint4, true>(src + i + 512),
                d = ld_global<uint4, true>(src + i + 768);
    dst[i] = a;
    dst[i + 256] = b;
    dst[i + 512] = e;
    dst[i + 768] = d;
  }
  if (blockIdx.x == gridDim.x - 1)                    // the last, partial chunk
    for (size_t i = chunks * 1024 + threadIdx.x; i < n_vec; i += 256) dst[i] = ld_global<uint4, true>(src + i);
}

// Picks the block size and launches k_copy_blocks; returns false if the maps allow no block of
// at least 32 bytes (the caller then moves single vectors).
static bool launch_copy_blocks(const vt_desc& s, const vt_desc* d, const DevDesc& S, const DevDesc& D, void* dst, int64_t outer,
                               int64_t inner, hipStream_t stream) {
  const int esz = dtype_size(s.dtype);
  if (vector_width(s) * esz != 16 || (d && vector_width(*d) * esz != 16) || (!d && (uintptr_t)dst % 16)) return false;
  int64_t be = block_elems(s, 1024 / esz);
  if (d) be = std::min(be, block_elems(*d, 1024 / esz));
  while (be > 1 && inner % be) be >>= 1;
  const int bl = (int)(be * esz / 16);
  if (bl < 2) return false;
  const int64_t blocks = inner / be;
  if (blocks >= (1ll << 31)) return false;
  // blocks per wave: sixteen instructions' worth (the map is then applied once per 16 KB at most),
  // fewer while that leaves less than about 16384 waves (two full rounds of the chip), never
  // less than one instruction's worth
  const uint32_t want_waves = 16384;
  uint32_t rb = std::min<uint32_t>(64, 16 * (64 / bl));
  while (rb > (uint32_t)(64 / bl) && blocks / rb < want_waves) rb >>= 1;
  const int64_t waves = (blocks + rb - 1) / rb;
  dim3 grid((unsigned)((waves + 3) / 4), (unsigned)std::min<int64_t>(outer, 65535));
  // block addresses from the maps' term form when both resolve
  BlockWalk WS, WD;
  memset(&WD, 0, sizeof(WD));
  const bool walk = outer == 1 && resolve_block_walk(s, be, &WS) && (!d || resolve_block_walk(*d, be, &WD));
  if (walk) {
#define VT_COPY_WALK(BLV)                                                                                              \
  case BLV:                                                                                                            \
    if (d) hipLaunchKernelGGL((k_copy_blocks_walk<BLV, true>), grid, dim3(256), 0, stream, WS, WD, (char*)nullptr,     \
                              (uint32_t)blocks, rb);                                                                   \
    else hipLaunchKernelGGL((k_copy_blocks_walk<BLV, false>), grid, dim3(256), 0, stream, WS, WD, (char*)dst,          \
                            (uint32_t)blocks, rb);                                                                     \
    break;
    switch (bl) {
      VT_COPY_WALK(2)
      VT_COPY_WALK(4)
      VT_COPY_WALK(8)
      VT_COPY_WALK(16)
      VT_COPY_WALK(32)
      VT_COPY_WALK(64)
      default: return false;
    }
#undef VT_COPY_WALK
    return true;
  }
#define VT_COPY_BLOCKS(BLV)                                                                                         \
  case BLV:                                                                                                         \
    if (d) hipLaunchKernelGGL((k_copy_blocks<BLV, true>), grid, dim3(256), 0, stream, S, D, (char*)nullptr,         \
                              (uint32_t)blocks, (uint32_t)be, rb, (uint32_t)outer);                                 \
    else hipLaunchKernelGGL((k_copy_blocks<BLV, false>), grid, dim3(256), 0, stream, S, S, (char*)dst,              \
                            (uint32_t)blocks, (uint32_t)be, rb, (uint32_t)outer);                                   \
    break;
  switch (bl) {
    VT_COPY_BLOCKS(2)
    VT_COPY_BLOCKS(4)
    VT_COPY_BLOCKS(8)
    VT_COPY_BLOCKS(16)
    VT_COPY_BLOCKS(32)
    VT_COPY_BLOCKS(64)
    default: return false;
  }
#undef VT_COPY_BLOCKS
  return true;
}

static int launch_scatter(const vt_desc& s, const vt_desc& d, hipStream_t stream) {
  DevDesc S, D;
  int64_t outer, inner, outer2, inner2;
  int rc = to_device(s, &S, &outer, &inner);
  if (rc != VT_OK) return rc;
  rc = to_device(d, &D, &outer2, &inner2);
  if (rc != VT_OK) return rc;
  if (outer == outer2 && inner == inner2 && launch_copy_blocks(s, &d, S, D, nullptr, outer, inner, stream)) return check_launch("vt_scatter");
  const int vec = std::min(vector_width(s), vector_width(d));
  const uint32_t inner_vecs = (uint32_t)(inner / vec);
  dim3 grid((inner_vecs + 255) / 256, (unsigned)std::min<int64_t>(outer, 65535));
  switch (vec * dtype_size(s.dtype)) {
    case 16:
      hipLaunchKernelGGL(k_scatter<uint4>, grid, dim3(256), 0, stream, S, D, inner_vecs, (uint32_t)vec, (uint32_t)outer);
      break;
    case 8:
      hipLaunchKernelGGL(k_scatter<uint2>, grid, dim3(256), 0, stream, S, D, inner_vecs, (uint32_t)vec, (uint32_t)outer);
      break;
    case 4:
      hipLaunchKernelGGL(k_scatter<uint32_t>, grid, dim3(256), 0, stream, S, D, inner_vecs, (uint32_t)vec, (uint32_t)outer);
      break;
    default:
      hipLaunchKernelGGL(k_scatter<uint16_t>, grid, dim3(256), 0, stream, S, D, inner_vecs, (uint32_t)vec, (uint32_t)outer);
      break;
  }
  return check_launch("vt_scatter");
}

// ------------------------------------------------------------------------------------------
// Transposing copy.  A map whose source runs along another virtual dim than the innermost one
// (a Transpose of the last dims: contiguous runs of one element, the case block-wise I/O cannot
// help) is copied in 64 x 64 tiles through LDS: a tile is read along the source's contiguous
// direction and written along the destination's, both coalesced.  The two directions and the
// remaining ones come from the map's term form (one piece, no test, the terms being exactly the
// digits of the virtual index): term 0 is the destination's innermost digit, `s` the digit whose
// coefficient is one element.
// ------------------------------------------------------------------------------------------
constexpr int kTrTile = 64;
struct TransposeParams {
  uint64_t src;             // address of virtual element 0
  char* dst;
  uint32_t md, ms;          // extents of the destination-contiguous and the source-contiguous digit
  uint32_t coef_d;          // bytes between consecutive values of the destination-contiguous digit in the source
  uint32_t div_s;           // virtual elements between consecutive values of the source-contiguous digit
  int32_t n_other;
  uint32_t o_mod[kWalkTerms], o_coef[kWalkTerms], o_div[kWalkTerms];   // the other digits: extent, source bytes, virtual elements
  uint32_t batch;           // product of the other digits' extents
};

template <typename T>
__global__ void __launch_bounds__(256) k_copy_transpose(const TransposeParams P) {
  __shared__ T tile[kTrTile][kTrTile + 1];
  const uint32_t lane = threadIdx.x & 63u, quarter = threadIdx.x >> 6;
  const uint32_t d0 = blockIdx.x * kTrTile, s0 = blockIdx.y * kTrTile;
  for (uint32_t bz = blockIdx.z; bz < P.batch; bz += gridDim.z) {
    uint64_t rest_src = 0, rest_u = 0;
    uint32_t b = bz;
    for (int k = 0; k < P.n_other; ++k) {
      const uint32_t q = b / P.o_mod[k], i = b - q * P.o_mod[k];
      b = q;
      rest_src += (uint64_t)i * P.o_coef[k];
      rest_u += (uint64_t)i * P.o_div[k];
    }
    // read: lanes along the source's contiguous digit
#pragma unroll
    for (int r = 0; r < kTrTile / 4; ++r) {
      const uint32_t id = r * 4 + quarter, is = lane;
      if (d0 + id < P.md && s0 + is < P.ms)
        tile[id][is] = ld_global<T, true>(P.src + rest_src + (uint64_t)(d0 + id) * P.coef_d + (uint64_t)(s0 + is) * sizeof(T));
    }
    __syncthreads();
    // write: lanes along the destination's contiguous digit
#pragma unroll
    for (int r = 0; r < kTrTile / 4; ++r) {
      const uint32_t is = r * 4 + quarter, id = lane;
      if (d0 + id < P.md && s0 + is < P.ms)
        reinterpret_cast<T*>(P.dst)[rest_u + (uint64_t)(s0 + is) * P.div_s + (d0 + id)] = tile[id][is];
    }
    __syncthreads();
  }
}

// Launches k_copy_transpose if the map has the form described above; false otherwise.
static bool launch_transpose(const vt_desc& d, void* dst, hipStream_t stream) {
  const int esz = dtype_size(d.dtype);
  BlockWalk W;
  if (!resolve_block_walk(d, 1, &W) || W.n != 1 || W.piece[0].has_test) return false;
  const WalkPiece& pc = W.piece[0];
  int64_t numel = 1;
  for (int64_t e : d.shape) numel *= e;
  const int nt = pc.n_terms;
  if (nt < 2) return false;
  // the terms must be the digits of the virtual index: div 1, then each the product of those before
  int64_t mods[kWalkTerms];
  int64_t expect = 1;
  for (int t = 0; t < nt; ++t) {
    if (pc.term[t].on_coord || (int64_t)pc.term[t].div.d != expect) return false;
    mods[t] = pc.term[t].mod.d ? (int64_t)pc.term[t].mod.d : numel / expect;
    expect *= mods[t];
  }
  if (expect != numel) return false;
  if (pc.term[0].coef == (uint32_t)esz) return false;    // the source runs along the innermost digit: not a transpose
  int ts = -1;
  for (int t = 1; t < nt; ++t)
    if (pc.term[t].coef == (uint32_t)esz) ts = t;
  if (ts < 0 || mods[0] < 16 || mods[ts] < 16) return false;   // short digits: tiles would be mostly empty
  TransposeParams P;
  memset(&P, 0, sizeof(P));
  P.src = pc.base;
  P.dst = static_cast<char*>(dst);
  P.md = (uint32_t)mods[0];
  P.ms = (uint32_t)mods[ts];
  P.coef_d = pc.term[0].coef;
  P.div_s = pc.term[ts].div.d;
  int64_t batch = 1;
  for (int t = 1; t < nt; ++t) {
    if (t == ts) continue;
    P.o_mod[P.n_other] = (uint32_t)mods[t];
    P.o_coef[P.n_other] = pc.term[t].coef;
    P.o_div[P.n_other] = pc.term[t].div.d;
    ++P.n_other;
    batch *= mods[t];
  }
  P.batch = (uint32_t)batch;
  const int64_t td = (mods[0] + kTrTile - 1) / kTrTile, tsn = (mods[ts] + kTrTile - 1) / kTrTile;
  if (tsn > 65535) return false;
  dim3 grid((unsigned)td, (unsigned)tsn, (unsigned)std::min<int64_t>(batch, 65535));
  if (esz == 4) hipLaunchKernelGGL(k_copy_transpose<uint32_t>, grid, dim3(256), 0, stream, P);
  else hipLaunchKernelGGL(k_copy_transpose<uint16_t>, grid, dim3(256), 0, stream, P);
  return true;
}

static int launch_materialize(const vt_desc& d, void* dst, hipStream_t stream) {
  DevDesc D;
  int64_t outer, inner;
  int rc = to_device(d, &D, &outer, &inner);
  if (rc != VT_OK) return rc;
  {
    int64_t numel = 1;
    for (int64_t e : d.shape) numel *= e;
    const int64_t bytes_total = numel * dtype_size(d.dtype);
    if (d.pieces.size() == 1 && d.run >= numel && bytes_total % 16 == 0 && (uintptr_t)dst % 16 == 0) {
      const Piece& p = d.pieces[0];
      int64_t base = p.v.base;
      for (const Stage& st : p.v.lower) base = st.base + base;     // a fully contiguous piece: stages only add their bases
      const char* src = static_cast<const char*>(d.sources[p.src].ptr) + base * dtype_size(d.dtype);
      if ((uintptr_t)src % 16 == 0 && p.v.lower.empty()) {
        const size_t n_vec = (size_t)(bytes_total / 16);
        const unsigned blocks = (unsigned)std::min<size_t>((n_vec + 1023) / 1024, 1u << 20);
        hipLaunchKernelGGL(k_copy_flat, dim3(std::max(1u, blocks)), dim3(256), 0, stream, reinterpret_cast<const uint4*>(src),
                           reinterpret_cast<uint4*>(dst), n_vec);
        return check_launch("vt_materialize");
      }
    }
  }
  if (launch_copy_blocks(d, nullptr, D, D, dst, outer, inner, stream)) return check_launch("vt_materialize");
  if (outer == 1 && launch_transpose(d, dst, stream)) return check_launch("vt_materialize");
  int vec = vector_width(d);
  if ((uintptr_t)dst % 16) vec = 1;
  int esz = dtype_size(d.dtype);
  uint32_t inner_vecs = (uint32_t)(inner / vec);
  dim3 grid((inner_vecs + 255) / 256, (unsigned)std::min<int64_t>(outer, 65535));
  int bytes = vec * esz;
  switch (bytes) {
    case 16:
      hipLaunchKernelGGL(k_materialize<uint4>, grid, dim3(256), 0, stream, D, (uint4*)dst, inner_vecs, (uint32_t)vec, (uint32_t)outer);
      break;
    case 8:
      hipLaunchKernelGGL(k_materialize<uint2>, grid, dim3(256), 0, stream, D, (uint2*)dst, inner_vecs, (uint32_t)vec, (uint32_t)outer);
      break;
    case 4:
      hipLaunchKernelGGL(k_materialize<uint32_t>, grid, dim3(256), 0, stream, D, (uint32_t*)dst, inner_vecs, (uint32_t)vec, (uint32_t)outer);
      break;
    default:
      hipLaunchKernelGGL(k_materialize<uint16_t>, grid, dim3(256), 0, stream, D, (uint16_t*)dst, inner_vecs, (uint32_t)vec, (uint32_t)outer);
      break;
  }
  return check_launch("vt_materialize");
}

// ------------------------------------------------------------------------------------------
// out[r] = sum_c (x[r,c] + y[r,c]), fp32.  One wave per row.  Lane l owns the columns
// c = l, l+64, ... in ascending order starting from +0; the 64 partial sums are combined by
// the butterfly p[l] += p[l xor s], s = 32..1, and lane 0 stores.  This order is part of the
// contract (it is what makes the result reproducible bit for bit).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_add_rowsum(const DevDesc X, const DevDesc Y, float* __restrict__ out,
                                                    uint32_t R, uint32_t C) {
  __shared__ DevDesc maps[2];
  {
    const DevDesc* const src[2] = {&X, &Y};
    stage_maps(maps, src);
  }
  uint32_t lane = threadIdx.x & 63u;
  uint32_t row = blockIdx.x * 4u + (threadIdx.x >> 6);
  if (row >= R) return;
  float p = 0.0f;
  for (uint32_t c = lane; c < C; c += 64u) {
    int64_t ox, oy;
    const void *px, *py;
    vtd_eval(maps[0], 0, row * C + c, &ox, &px);
    vtd_eval(maps[1], 0, row * C + c, &oy, &py);
    float t = ld_global<float>(static_cast<const float*>(px) + ox) + ld_global<float>(static_cast<const float*>(py) + oy);
    p = p + t;
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) p = p + __shfl_xor(p, s, 64);
  if (lane == 0) out[row] = p;
}

// The same sum, same order, with block-wise virtual tensor I/O (Sec. 4.2): where the maps keep
// aligned blocks of 2^bx (x) and 2^by (y) columns contiguous, a lane applies a map once per block
// (to the block's first element; 64 blocks per round, one per lane) and the element addresses of
// each 64-column window follow from lane shuffles.  Lane l still owns the columns l, l + 64, ...
// and adds them in ascending order, so the result has the bits of k_add_rowsum.
struct BlockCursor {
  uint64_t addr;      // this lane's block: address of its first element
  uint32_t first;     // first block the 64 lanes hold
};

__device__ __forceinline__ void cursor_load(const DevDesc& X, uint32_t row, uint32_t C, uint32_t blog, uint32_t blk0, uint32_t lane,
                                            BlockCursor& cur) {
  const uint32_t nb = C >> blog;
  const uint32_t b = min(blk0 + lane, nb - 1);
  int64_t off;
  const void* ptr;
  vtd_eval(X, 0, row * C + (b << blog), &off, &ptr);
  cur.addr = reinterpret_cast<uint64_t>(ptr) + (uint64_t)off * 4u;
  cur.first = blk0;
}

__device__ __forceinline__ float cursor_read(const BlockCursor& cur, uint32_t col, uint32_t blog) {
  const uint64_t a = shfl_u64(cur.addr, (int)((col >> blog) - cur.first));
  return ld_global<float, true>(a + (uint64_t)(col & ((1u << blog) - 1u)) * 4u);   // read once: streaming
}

// The same for a window of 64 columns starting at the wave-uniform column c0 when blocks hold at
// least 64 columns: the whole window lies in one block, whose address is read from the owning
// lane into scalar registers; a lane adds its own column.
__device__ __forceinline__ float cursor_read_window(const BlockCursor& cur, uint32_t c0, uint32_t lane, uint32_t blog) {
  const int owner = (int)((c0 >> blog) - cur.first);
  const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)cur.addr, owner), hi = __builtin_amdgcn_readlane((uint32_t)(cur.addr >> 32), owner);
  const uint64_t base = ((uint64_t)hi << 32) | lo;
  return ld_global<float, true>(base + (uint64_t)((c0 & ((1u << blog) - 1u)) + lane) * 4u);   // read once: streaming
}

typedef __attribute__((address_space(4))) const RowWalk* kernarg_walk_t;   // a walk inside the kernel-argument segment

__device__ __forceinline__ void cursor_walk(kernarg_walk_t Wp, uint32_t row, uint32_t C, uint32_t blog, uint32_t blk0, uint32_t lane,
                                            BlockCursor& cur) {
  // The segments are read here, where they are used, and not kept in registers over the kernel's
  // main loop (the pointer is made opaque so that the reads cannot be moved out of this place).
  asm volatile("" : "+s"(Wp));
  const uint32_t nb = C >> blog;
  const uint32_t b = min(blk0 + lane, nb - 1);
  // Few instructions matter here: every wave of the launch runs this before its first load.  A
  // lane first picks the fields of the segment that holds its block (the tests on the row are
  // uniform), then the address is computed once, the block's part in 32 bits.
  uint64_t base = 0;
  uint32_t j = 0, bs = 0, gs = 0;
  FastDiv g = {0, 0, 0};
  const int n = Wp->n, two_level = Wp->two_level;
#pragma unroll
  for (int k = 0; k < kRowSegs; ++k) {
    if (k < n) {
      const __attribute__((address_space(4))) RowSeg* sg = &Wp->seg[k];
      if (row >= sg->row_lo && row < sg->row_hi) {
        const uint64_t row_base = sg->base + (uint64_t)((int64_t)(row - sg->row_lo) * sg->row_stride);
        const bool in = b >= sg->blk_lo && b < sg->blk_hi;
        base = in ? row_base : base;
        j = in ? b - sg->blk_lo : j;
        bs = in ? sg->blk_stride : bs;
        if (two_level) {
          gs = in ? sg->group_stride : gs;
          g.d = in ? sg->blk_group.d : g.d;
          g.magic = in ? sg->blk_group.magic : g.magic;
          g.shift = in ? sg->blk_group.shift : g.shift;
        }
      }
    }
  }
  uint32_t off = j * bs;
  if (two_level) {
    const uint32_t hi = g.d ? fdiv(j, g) : 0u, lo = j - hi * g.d;
    off = g.d ? lo * bs + hi * gs : off;
  }
  cur.addr = base + off;
  cur.first = blk0;
}

VT_PROF_DECLARE(add_rowsum)

// WIDE: both operands keep blocks of at least 64 columns.  WALK: block addresses from the host's
// segments (wx, wy) instead of the evaluator on X and Y.
template <bool WIDE, bool WALK>
__global__ void __launch_bounds__(256) k_add_rowsum_blocks(const RowWalk wx, const RowWalk wy, float* __restrict__ out, uint32_t R, uint32_t C,
                                                           uint32_t bx, uint32_t by, const DevDesc X, const DevDesc Y) {
  VT_PROF_BEGIN();
  VT_PROF(0);
  if (WALK) {
    // the segments and the scalars are read in several rounds, each a miss of the scalar cache:
    // their eight lines are requested at once (0.4 us of 56 on the 335 MB chain)
    static_assert(2 * sizeof(RowWalk) + sizeof(float*) + 4 * sizeof(uint32_t) <= 512, "the walked arguments lie in the first eight lines");
    warm_kernarg_8();
  }
  // wx and wy are the first two arguments
  const kernarg_walk_t kwalk = (kernarg_walk_t)__builtin_amdgcn_kernarg_segment_ptr();
  (void)wx, (void)wy;
  __shared__ DevDesc maps[2];                         // unused (and not allocated) with WALK
  if (!WALK) {
    const DevDesc* const src[2] = {&X, &Y};
    stage_maps(maps, src);
  }
  VT_PROF(1);
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t row = blockIdx.x * 4u + (threadIdx.x >> 6);
  if (row >= R) return;                              // never the workgroup's first wave
  // columns after which the 64 cached blocks of an operand are used up
  const uint32_t span_x = 64u << bx, span_y = 64u << by;
  float p = 0.0f;
  BlockCursor cx, cy;
  for (uint32_t c0 = 0; c0 < C;) {
    if (c0 % span_x == 0) {
      if (WALK) cursor_walk(kwalk, row, C, bx, c0 >> bx, lane, cx);
      else cursor_load(maps[0], row, C, bx, c0 >> bx, lane, cx);
    }
    if (c0 % span_y == 0) {
      if (WALK) cursor_walk(kwalk + 1, row, C, by, c0 >> by, lane, cy);
      else cursor_load(maps[1], row, C, by, c0 >> by, lane, cy);
    }
    const uint32_t end = min(C, min((c0 / span_x + 1) * span_x, (c0 / span_y + 1) * span_y));
    VT_PROF_ONCE(2);
    // whole windows of 64 columns, eight at a time so that sixteen loads are in flight per lane
    // (thirty-two measured the same)
    for (; c0 + 512 <= end; c0 += 512) {
      float xv[8], yv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        xv[u] = WIDE ? cursor_read_window(cx, c0 + 64 * u, lane, bx) : cursor_read(cx, c0 + 64 * u + lane, bx);
        yv[u] = WIDE ? cursor_read_window(cy, c0 + 64 * u, lane, by) : cursor_read(cy, c0 + 64 * u + lane, by);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) p = p + (xv[u] + yv[u]);
      VT_PROF_ONCE(3);
    }
    for (; c0 < end; c0 += 64) {
      const uint32_t col = min(c0 + lane, C - 1);     // every lane shuffles; lanes past the row add nothing
      const float t = cursor_read(cx, col, bx) + cursor_read(cy, col, by);
      if (c0 + lane < C) p = p + t;
    }
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) p = p + __shfl_xor(p, s, 64);
  if (lane == 0) out[row] = p;
  VT_PROF(4);
  VT_PROF_FLUSH(add_rowsum, blockIdx.x);
}

// ------------------------------------------------------------------------------------------
// Per-row LayerNorm over the last dim (gamma = 1, beta = 0, biased variance), fp32 math.
// LPR lanes share a row; each lane keeps up to 4 vectors of VEC elements in registers.
// ------------------------------------------------------------------------------------------
template <typename T, int VEC>
__global__ void __launch_bounds__(256) k_layernorm(const DevDesc X, T* __restrict__ out, uint32_t rows, uint32_t C,
                                                   uint32_t lpr_log2, float eps, uint32_t outer, uint32_t rows_inner) {
  __shared__ DevDesc map[1];
  {
    const DevDesc* const from[1] = {&X};
    stage_maps(map, from);
  }
  const uint32_t lpr = 1u << lpr_log2;
  const uint32_t rpw = 64u >> lpr_log2;                 // rows per wave
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t sub = lane & (lpr - 1u);
  const uint32_t row = (blockIdx.x * 4u + (threadIdx.x >> 6)) * rpw + (lane >> lpr_log2);
  const uint32_t nvec = C / VEC;
  const bool live = row < rows;
  float v[4][VEC];
  float sum = 0.0f;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    uint32_t j = sub + it * lpr;
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[it][e] = 0.0f;
    if (live && j < nvec) {
      uint32_t o = row / rows_inner, ri = row - o * rows_inner;
      int64_t off;
      const void* ptr;
      vtd_eval(map[0], o, ri * C + j * VEC, &off, &ptr);
      Vec<T, VEC> raw = ld_global<Vec<T, VEC>>(static_cast<const T*>(ptr) + off);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        v[it][e] = to_float(raw.v[e]);
        sum += v[it][e];
      }
    }
  }
  for (uint32_t s = lpr >> 1; s >= 1; s >>= 1) sum += __shfl_xor(sum, (int)s, 64);
  const float mean = sum / (float)C;
  float sq = 0.0f;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    uint32_t j = sub + it * lpr;
    if (j < nvec) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        float dlt = v[it][e] - mean;
        sq += dlt * dlt;
      }
    }
  }
  for (uint32_t s = lpr >> 1; s >= 1; s >>= 1) sq += __shfl_xor(sq, (int)s, 64);
  const float rstd = 1.0f / sqrtf(sq / (float)C + eps);
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    uint32_t j = sub + it * lpr;
    if (live && j < nvec) {
      Vec<T, VEC> o;
#pragma unroll
      for (int e = 0; e < VEC; ++e) o.v[e] = from_float<T>((v[it][e] - mean) * rstd);
      *reinterpret_cast<Vec<T, VEC>*>(out + (size_t)row * C + (size_t)j * VEC) = o;
    }
  }
  (void)outer;
}

// The same LayerNorm, same lane-to-element assignment (the sums over a row's lanes may be taken in
// another order), for maps that keep every row one contiguous range of a source: the map is applied once
// per ROW instead of once per vector.  A wave takes 32 consecutive rows; lane l evaluates the
// address of row l (one evaluation serves 32 rows where the kernel above needs one per group of
// 64 / lpr rows: the evaluator's several hundred instructions, not the memory, bound that kernel),
// and the rows are then read in passes of 64 / lpr rows, their addresses handed round by shuffle,
// eight vectors per lane in flight.  ITS = vectors per lane and row (1, 2 or 4).
// (Row addresses from the map's term form, as in the block copies, were measured here as well:
// 20-22 us against 17.5 us on the window-partitioned rows, equal on dense rows; the evaluator stays.)
constexpr uint32_t kLnRowsPerWave = 32;   // (or one pass's rows, if that is more)
VT_PROF_DECLARE(layernorm)

template <typename T, int VEC, int ITS>
__global__ void __launch_bounds__(256) k_layernorm_rows(const DevDesc X, T* __restrict__ out, uint32_t rows, uint32_t C,
                                                        uint32_t lpr_log2, float eps, uint32_t rows_inner) {
  VT_PROF_BEGIN();
  VT_PROF(0);
  __shared__ DevDesc map[1];
  {
    const DevDesc* const from[1] = {&X};
    stage_maps(map, from);
  }
  VT_PROF(1);
  constexpr int U = 8 / ITS;                            // passes in flight
  const uint32_t lpr = 1u << lpr_log2;
  const uint32_t rpw = 64u >> lpr_log2;                 // rows per pass
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t sub = lane & (lpr - 1u);
  const uint32_t rw = max(kLnRowsPerWave, rpw);          // rows of this wave
  const uint32_t row0 = (blockIdx.x * 4u + (threadIdx.x >> 6)) * rw;
  if (row0 >= rows) return;
  const uint32_t nvec = C / VEC;
  uint64_t row_addr;
  {
    const uint32_t r = min(row0 + (lane & (rw - 1u)), rows - 1u);
    const uint32_t o = r / rows_inner, ri = r - o * rows_inner;
    int64_t off;
    const void* ptr;
    vtd_eval(map[0], o, ri * C, &off, &ptr);
    row_addr = reinterpret_cast<uint64_t>(ptr) + (uint64_t)(off * (int64_t)sizeof(T));
  }
  VT_PROF(2);
  const uint32_t passes = rw / rpw;
  // Sum over the lpr lanes of a row, for the U passes at once.  Rows of 16 or 8 lanes (the usual
  // ones: 128 or 64 elements of 16 bits) use the VALU's lane permutes; a shuffle through LDS costs
  // a round trip per step, and the compiler waits for each one before it issues the next.
  auto reduce_rows = [&](float (&x)[U]) {
    if (lpr == 16) {
#pragma unroll
      for (int u = 0; u < U; ++u) x[u] = group_sum<16>(x[u]);
    } else if (lpr == 8) {
#pragma unroll
      for (int u = 0; u < U; ++u) x[u] = group_sum<8>(x[u]);
    } else {
      for (uint32_t s = lpr >> 1; s >= 1; s >>= 1) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] += __shfl_xor(x[u], (int)s, 64);
      }
    }
  };
  for (uint32_t p0 = 0; p0 < passes; p0 += U) {
    Vec<T, VEC> raw[U][ITS];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t rl = min((p0 + u) * rpw + (lane >> lpr_log2), rw - 1u);
      live[u] = p0 + u < passes && row0 + rl < rows;
      const uint64_t a = shfl_u64(row_addr, (int)rl);
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        // unconditional (a lane without a vector of its own reads a valid one again and drops it:
        // rows past the end were clamped to the last row above), so that all loads of the round
        // are in flight together
        const uint32_t j = min(sub + it * lpr, nvec - 1u);
        raw[u][it] = ld_global<Vec<T, VEC>, true>(a + (uint64_t)j * (VEC * sizeof(T)));
      }
    }
    // The U passes are independent: every step below is done for all of them before the next one.
    float v[U][ITS][VEC];
    float sum[U], sq[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      sum[u] = 0.0f;
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        const bool mine = live[u] && sub + it * lpr < nvec;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          v[u][it][e] = mine ? to_float(raw[u][it].v[e]) : 0.0f;
          if (mine) sum[u] += v[u][it][e];
        }
      }
    }
    VT_PROF_ONCE(3);
    reduce_rows(sum);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float mean = sum[u] / (float)C;
      sum[u] = mean;
      sq[u] = 0.0f;
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        if (sub + it * lpr < nvec) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            float dlt = v[u][it][e] - mean;
            sq[u] += dlt * dlt;
          }
        }
      }
    }
    reduce_rows(sq);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float mean = sum[u];
      const float rstd = 1.0f / sqrtf(sq[u] / (float)C + eps);
      const uint32_t row = row0 + (p0 + u) * rpw + (lane >> lpr_log2);
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        const uint32_t j = sub + it * lpr;
        if (live[u] && j < nvec) {
          Vec<T, VEC> o;
#pragma unroll
          for (int e = 0; e < VEC; ++e) o.v[e] = from_float<T>((v[u][it][e] - mean) * rstd);
          // (an ordinary store: a streaming one ends the kernel 2 us earlier, since no dirty lines
          // have to drain, but the consumer that follows then reads the rows from memory instead
          // of the cache: LayerNorm + GEMM measured 71.0 against 70.1 us)
          *reinterpret_cast<Vec<T, VEC>*>(out + (size_t)row * C + (size_t)j * VEC) = o;
        }
      }
    }
    VT_PROF_ONCE(4);
  }
#ifdef VT_PROFILE
  __builtin_amdgcn_s_waitcnt(0);
  VT_PROF(5);
  VT_PROF_FLUSH(layernorm, blockIdx.x);
#endif
}

template <typename T>
static int launch_layernorm_t(const vt_desc& d, const DevDesc& D, void* out, float eps, int64_t outer, int64_t inner,
                              hipStream_t stream) {
  int n = (int)d.shape.size();
  int64_t C = d.shape[n - 1];
  int vec = vector_width(d);
  if ((uintptr_t)out % 16) vec = 1;
  int64_t nvec = C / vec;
  uint32_t lpr_log2 = 0;
  while ((1 << lpr_log2) < nvec && lpr_log2 < 6) ++lpr_log2;
  if (nvec > (int64_t)(4 << lpr_log2)) return fail(VT_ERR_UNSUPPORTED, "layernorm: row too long for the register-resident kernel");
  int64_t rows = outer * inner / C;
  if (rows >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, "layernorm: too many rows");
  uint32_t rows_inner = (uint32_t)(inner / C);
  // every row one contiguous range of a source: one evaluation of the map per row
  bool rows_contiguous = d.run % C == 0;
  for (const Piece& p : d.pieces) rows_contiguous = rows_contiguous && p.lo[n - 1] == 0 && p.hi[n - 1] == C;
  if ((C & (C - 1)) == 0 && block_elems(d, C) == C) rows_contiguous = true;
  if (rows_contiguous && vec * (int)sizeof(T) == 16) {   // full 16-byte vectors only: the other widths keep the kernel above
    const int its = nvec <= (int64_t)(1 << lpr_log2) ? 1 : nvec <= (int64_t)(2 << lpr_log2) ? 2 : 4;
    constexpr int V16 = 16 / (int)sizeof(T);
    const int64_t rows_per_wg = 4 * (int64_t)std::max<uint32_t>(kLnRowsPerWave, 64u >> lpr_log2);
    dim3 grid_rows((unsigned)((rows + rows_per_wg - 1) / rows_per_wg));
#define LN_ROWS(I)                                                                                                            \
  hipLaunchKernelGGL((k_layernorm_rows<T, V16, I>), grid_rows, dim3(256), 0, stream, D, (T*)out, (uint32_t)rows, (uint32_t)C, \
                     lpr_log2, eps, rows_inner)
    if (its == 1) LN_ROWS(1);
    else if (its == 2) LN_ROWS(2);
    else LN_ROWS(4);
#undef LN_ROWS
    return check_launch("vt_elementwise(layernorm)");
  }
  uint32_t rpw = 64u >> lpr_log2;
  dim3 grid((unsigned)((rows + 4 * rpw - 1) / (4 * rpw)));
#define LN_LAUNCH(V)                                                                                          \
  hipLaunchKernelGGL((k_layernorm<T, V>), grid, dim3(256), 0, stream, D, (T*)out, (uint32_t)rows, (uint32_t)C, \
                     lpr_log2, eps, (uint32_t)outer, rows_inner)
  switch (vec) {
    case 8:
      if constexpr (sizeof(T) == 2) { LN_LAUNCH(8); break; }
      [[fallthrough]];
    case 4: LN_LAUNCH(4); break;
    case 2: LN_LAUNCH(2); break;
    default: LN_LAUNCH(1); break;
  }
#undef LN_LAUNCH
  return check_launch("vt_elementwise(layernorm)");
}

// ------------------------------------------------------------------------------------------
// out[r, :] = w[r][0] * x[r, :] + w[r][1] * y[r, :]   (the combine step of a mixture of experts:
// x and y are the two expert outputs of token r, gathered through row tables).  fp32 arithmetic,
// 16-bit storage.  Rows that are contiguous in their sources (the usual case: whole rows are
// gathered) take the row kernel: the map is applied once per row, on values that are uniform in
// the workgroup, and the row streams through 16-byte nontemporal loads and stores (every byte is
// touched once).  Anything else goes through the generic evaluator per vector.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) k_weighted_sum_rows(const DevDesc X, const DevDesc Y, const float* __restrict__ w,
                                                           T* __restrict__ out, uint32_t R, uint32_t C) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  for (uint32_t row = blockIdx.x; row < R; row += gridDim.x) {
    int64_t ox, oy;
    const void *px, *py;
    vtd_eval(X, 0, row * C, &ox, &px);
    vtd_eval(Y, 0, row * C, &oy, &py);
    const u32x4* xr = reinterpret_cast<const u32x4*>(static_cast<const T*>(px) + ox);
    const u32x4* yr = reinterpret_cast<const u32x4*>(static_cast<const T*>(py) + oy);
    u32x4* orow = reinterpret_cast<u32x4*>(out + (size_t)row * C);
    const float wx = w[2 * row], wy = w[2 * row + 1];
    for (uint32_t v = threadIdx.x; v < C / 8; v += 256) {
      const Vec<T, 8> a = __builtin_bit_cast(Vec<T, 8>, __builtin_nontemporal_load(xr + v));
      const Vec<T, 8> b = __builtin_bit_cast(Vec<T, 8>, __builtin_nontemporal_load(yr + v));
      Vec<T, 8> o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o.v[e] = from_float<T>(wx * to_float(a.v[e]) + wy * to_float(b.v[e]));
      __builtin_nontemporal_store(__builtin_bit_cast(u32x4, o), orow + v);
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(256) k_weighted_sum_generic(const DevDesc X, const DevDesc Y, const float* __restrict__ w,
                                                              T* __restrict__ out, uint32_t n, uint32_t C) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= n) return;
  int64_t ox, oy;
  const void *px, *py;
  vtd_eval(X, 0, i, &ox, &px);
  vtd_eval(Y, 0, i, &oy, &py);
  const uint32_t row = i / C;
  out[i] = from_float<T>(w[2 * row] * to_float(static_cast<const T*>(px)[ox]) + w[2 * row + 1] * to_float(static_cast<const T*>(py)[oy]));
}

template <typename T>
static int launch_weighted_sum(const vt_desc& x, const vt_desc& y, const DevDesc& X, const DevDesc& Y, const float* w, void* out,
                               hipStream_t st) {
  const uint32_t R = (uint32_t)x.shape[0], C = (uint32_t)x.shape[1];
  bool rows_ok = C % 8 == 0 && (uintptr_t)out % 16 == 0 && vector_width(x) == 8 && vector_width(y) == 8;
  for (const vt_desc* d : {&x, &y})
    for (const Piece& p : d->pieces)
      rows_ok = rows_ok && p.run % C == 0 && p.lo[1] == 0 && p.hi[1] == (int64_t)C;   // whole rows, each contiguous in its source
  if (rows_ok) {
    hipLaunchKernelGGL((k_weighted_sum_rows<T>), dim3(std::min<uint32_t>(R, 65535u * 16u)), dim3(256), 0, st, X, Y, w, (T*)out, R, C);
  } else {
    const uint32_t n = R * C;
    hipLaunchKernelGGL((k_weighted_sum_generic<T>), dim3((n + 255) / 256), dim3(256), 0, st, X, Y, w, (T*)out, n, C);
  }
  return check_launch("vt_weighted_sum");
}

extern "C" {

int vt_materialize(const vt_desc* d, void* dst, void* stream) {
  if (!d || !dst) return fail(VT_ERR_INVALID_ARG, "vt_materialize: NULL argument");
  return launch_materialize(*d, dst, (hipStream_t)stream);
}

int vt_scatter(const vt_desc* src, const vt_desc* dst, void* stream) {
  if (!src || !dst) return fail(VT_ERR_INVALID_ARG, "vt_scatter: NULL argument");
  if (src->shape != dst->shape || src->dtype != dst->dtype) return fail(VT_ERR_SHAPE, "vt_scatter: source and destination differ in shape or dtype");
  int rc = check_store_map(*dst, "vt_scatter");
  if (rc != VT_OK) return rc;
  for (const Piece& p : dst->pieces)
    if (!dst->sources[p.src].ptr) return fail(VT_ERR_INVALID_ARG, "vt_scatter: destination tensor without a device pointer");
  return launch_scatter(*src, *dst, (hipStream_t)stream);
}

int vt_weighted_sum(const vt_desc* x, const vt_desc* y, const float* weights, void* out, void* stream) {
  if (!x || !y || !weights || !out) return fail(VT_ERR_INVALID_ARG, "vt_weighted_sum: NULL argument");
  if (x->dtype == VT_F32 || y->dtype != x->dtype) return fail(VT_ERR_INVALID_ARG, "vt_weighted_sum: x and y must share a 16-bit dtype");
  if (x->shape.size() != 2 || x->shape != y->shape) return fail(VT_ERR_SHAPE, "vt_weighted_sum: x and y must be [R,C] of equal shape");
  DevDesc X, Y;
  int64_t ox, ix, oy, iy;
  int rc = to_device(*x, &X, &ox, &ix);
  if (rc != VT_OK) return rc;
  rc = to_device(*y, &Y, &oy, &iy);
  if (rc != VT_OK) return rc;
  if (ox != 1 || oy != 1) return fail(VT_ERR_UNSUPPORTED, "vt_weighted_sum: 2^31 elements or more");
  if (x->dtype == VT_BF16) return launch_weighted_sum<bf16_t>(*x, *y, X, Y, weights, out, (hipStream_t)stream);
  return launch_weighted_sum<f16_t>(*x, *y, X, Y, weights, out, (hipStream_t)stream);
}

int vt_copy_op(const vt_source* in, int n_in, const vt_op* op, void* dst, void* stream) {
  if (!in || !op || !dst || n_in < 1) return fail(VT_ERR_INVALID_ARG, "vt_copy_op: NULL argument");
  vt_op local = *op;
  if (local.n_in != n_in) return fail(VT_ERR_INVALID_ARG, "vt_copy_op: n_in differs from the statement's");
  for (int i = 0; i < n_in; ++i) local.in[i] = -1 - i;
  vt_desc* d = nullptr;
  int rc = vt_build(in, n_in, &local, 1, 0, &d);
  if (rc != VT_OK) return rc;
  rc = launch_materialize(*d, dst, (hipStream_t)stream);
  vt_free(d);
  return rc;
}

int vt_elementwise(int kind, const vt_desc* x, const vt_desc* y, float eps, void* out, void* stream) {
  if (!x || !out) return fail(VT_ERR_INVALID_ARG, "vt_elementwise: NULL argument");
  hipStream_t st = (hipStream_t)stream;
  if (kind == VT_EW_ADD_ROWSUM) {
    if (!y) return fail(VT_ERR_INVALID_ARG, "vt_elementwise(add_rowsum): y is NULL");
    if (x->dtype != VT_F32 || y->dtype != VT_F32) return fail(VT_ERR_INVALID_ARG, "vt_elementwise(add_rowsum): fp32 only");
    if (x->shape.size() != 2 || x->shape != y->shape) return fail(VT_ERR_SHAPE, "vt_elementwise(add_rowsum): x and y must be [R,C] of equal shape");
    DevDesc X, Y;
    int64_t ox, ix, oy, iy;
    int rc = to_device(*x, &X, &ox, &ix);
    if (rc != VT_OK) return rc;
    rc = to_device(*y, &Y, &oy, &iy);
    if (rc != VT_OK) return rc;
    if (ox != 1 || oy != 1) return fail(VT_ERR_UNSUPPORTED, "vt_elementwise(add_rowsum): 2^31 elements or more");
    uint32_t R = (uint32_t)x->shape[0], C = (uint32_t)x->shape[1];
    // block-wise path: both maps keep aligned blocks of at least 16 columns contiguous inside a row
    auto block_log2 = [&](const vt_desc& d) {
      int64_t b = block_elems(d, 1 << 20);
      while (b > 1 && C % b) b >>= 1;
      uint32_t l = 0;
      while ((2ll << l) <= b) ++l;
      return l;
    };
    const uint32_t bx = block_log2(*x), by = block_log2(*y);
    const dim3 grid((R + 3) / 4);
    // Block addresses from host-resolved segments whenever both maps have that form, whatever the
    // block size (single elements included: a dozen instructions per address instead of the
    // evaluator); else the evaluator once per block of at least 16 columns, else once per element.
    RowWalk wx, wy;
    const bool walk = resolve_row_walk(*x, 1ll << bx, &wx) && resolve_row_walk(*y, 1ll << by, &wy);
    if (walk || (bx >= 4 && by >= 4)) {
      const bool wide = bx >= 6 && by >= 6;
#define VT_ROWSUM(WIDE, WALK) \
  hipLaunchKernelGGL((k_add_rowsum_blocks<WIDE, WALK>), grid, dim3(256), 0, st, wx, wy, (float*)out, R, C, bx, by, X, Y)
      if (wide && walk) VT_ROWSUM(true, true);
      else if (wide) VT_ROWSUM(true, false);
      else if (walk) VT_ROWSUM(false, true);
      else VT_ROWSUM(false, false);
#undef VT_ROWSUM
    } else hipLaunchKernelGGL(k_add_rowsum, grid, dim3(256), 0, st, X, Y, (float*)out, R, C);
    return check_launch("vt_elementwise(add_rowsum)");
  }
  if (kind == VT_EW_LAYERNORM) {
    if (y) return fail(VT_ERR_INVALID_ARG, "vt_elementwise(layernorm): y must be NULL");
    DevDesc X;
    int64_t outer, inner;
    int rc = to_device(*x, &X, &outer, &inner);
    if (rc != VT_OK) return rc;
    if (inner % x->shape.back()) return fail(VT_ERR_UNSUPPORTED, "vt_elementwise(layernorm): row of 2^31 elements or more");
    switch (x->dtype) {
      case VT_F32: return launch_layernorm_t<float>(*x, X, out, eps, outer, inner, st);
      case VT_F16: return launch_layernorm_t<f16_t>(*x, X, out, eps, outer, inner, st);
      default: return launch_layernorm_t<bf16_t>(*x, X, out, eps, outer, inner, st);
    }
  }
  return fail(VT_ERR_INVALID_ARG, "vt_elementwise: unknown kind");
}

}  // extern "C"
