// Fused self-attention of one tensor-parallel shard (paper section 2.3: heads split over the ranks;
// section 4.2: scale + mask + softmax fused, with the implicit causal mask or a general byte mask;
// here the two batched GEMMs Q K^T and P V of the appendix are fused in as well, so the s x s matrix
// never reaches HBM).
//
// qkv is [s, b, 3*hp] with columns [Q heads | K heads | V heads]; for sample j and local head e the
// row of token i starts at qkv + (i*b + j)*3*hp + {0, hp, 2hp} + e*dh.
//
// bf16 forward: S^T = K Q^T and O^T = V^T P^T on v_mfma_f32_32x32x16_bf16, so that the softmax
// probabilities leave the first MFMA already in the register layout the second one wants as its
// B operand.  One wave owns 32 queries; a block of 2 waves shares 64-key K and V tiles in LDS.
// The "rowwise" kernels are the plain formulation (one wave per row): they are the fp32 path.
#include "common.h"

namespace ptdp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

template <typename T> __device__ __forceinline__ float ld(const T* p);
template <> __device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void st(T* p, float v);
template <> __device__ __forceinline__ void st<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// ------------------------------------------------------------------------------------------------
// rowwise kernels: grid (s, heads, b), one wave per block; lane owns dims lane, lane+64, ... (dh <= 256)
// ------------------------------------------------------------------------------------------------
constexpr int kMaxDimsPerLane = 4;
// General mask (section 4.2: the fused softmax "with general masking"): a hidden score is replaced
// by this value before the softmax, so a row without any visible key attends uniformly, and no
// gradient flows to q and k through a hidden score.  mask is [b, s, s] bytes, nonzero = hidden.
constexpr float kMaskFill = -10000.f;

template <typename T>
__global__ void __launch_bounds__(64)
attn_fwd_rowwise(const T* __restrict__ qkv, T* __restrict__ ctx, float* __restrict__ lse, int s, int b, int heads,
                 int dh, const uint8_t* __restrict__ mask, int causal) {
  const int i = blockIdx.x, e = blockIdx.y, j = blockIdx.z, lane = threadIdx.x;
  const int hp = heads * dh;
  const size_t rs = (size_t)b * 3 * hp;  // token stride
  const T* base = qkv + (size_t)j * 3 * hp + (size_t)e * dh;
  const float scale = rsqrtf((float)dh);
  float q[kMaxDimsPerLane], acc[kMaxDimsPerLane];
#pragma unroll
  for (int c = 0; c < kMaxDimsPerLane; ++c) {
    const int d = lane + 64 * c;
    q[c] = d < dh ? ld(base + (size_t)i * rs + d) : 0.f;
    acc[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int kend = causal ? i : s - 1;
  const uint8_t* mrow = (!causal && mask) ? mask + ((size_t)j * s + i) * s : nullptr;
  for (int kk = 0; kk <= kend; ++kk) {
    const T* kr = base + (size_t)kk * rs + hp;
    const T* vr = kr + hp;
    float dot = 0.f;
#pragma unroll
    for (int c = 0; c < kMaxDimsPerLane; ++c) {
      const int d = lane + 64 * c;
      if (d < dh) dot += q[c] * ld(kr + d);
    }
    float sc = wave_sum(dot) * scale;
    if (mrow && mrow[kk]) sc = kMaskFill;
    const float mn = fmaxf(m, sc);
    const float corr = __expf(m - mn), p = __expf(sc - mn);
    l = l * corr + p;
#pragma unroll
    for (int c = 0; c < kMaxDimsPerLane; ++c) {
      const int d = lane + 64 * c;
      if (d < dh) acc[c] = acc[c] * corr + p * ld(vr + d);
    }
    m = mn;
  }
#pragma unroll
  for (int c = 0; c < kMaxDimsPerLane; ++c) {
    const int d = lane + 64 * c;
    if (d < dh) st(ctx + ((size_t)i * b + j) * hp + (size_t)e * dh + d, acc[c] / l);
  }
  if (lane == 0) lse[((size_t)j * heads + e) * s + i] = m + __logf(l);
}

// delta[j][e][i] = sum_d dctx * ctx
template <typename T>
__global__ void __launch_bounds__(64)
attn_delta_rowwise(const T* __restrict__ ctx, const T* __restrict__ dctx, float* __restrict__ delta, int s, int b,
                   int heads, int dh) {
  const int i = blockIdx.x, e = blockIdx.y, j = blockIdx.z, lane = threadIdx.x;
  const size_t off = ((size_t)i * b + j) * heads * dh + (size_t)e * dh;
  float a = 0.f;
  for (int d = lane; d < dh; d += 64) a += ld(ctx + off + d) * ld(dctx + off + d);
  a = wave_sum(a);
  if (lane == 0) delta[((size_t)j * heads + e) * s + i] = a;
}

// dQ of query row i: sum over keys kk <= i of dS[i][kk] K[kk] / sqrt(dh)
template <typename T>
__global__ void __launch_bounds__(64)
attn_bwd_dq_rowwise(const T* __restrict__ qkv, const T* __restrict__ dctx, const float* __restrict__ lse,
                    const float* __restrict__ delta, T* __restrict__ dqkv, int s, int b, int heads, int dh,
                    const uint8_t* __restrict__ mask, int causal) {
  const int i = blockIdx.x, e = blockIdx.y, j = blockIdx.z, lane = threadIdx.x;
  const int hp = heads * dh;
  const size_t rs = (size_t)b * 3 * hp;
  const T* base = qkv + (size_t)j * 3 * hp + (size_t)e * dh;
  const float scale = rsqrtf((float)dh);
  const float L = lse[((size_t)j * heads + e) * s + i], D = delta[((size_t)j * heads + e) * s + i];
  float q[kMaxDimsPerLane], dc[kMaxDimsPerLane], acc[kMaxDimsPerLane];
#pragma unroll
  for (int c = 0; c < kMaxDimsPerLane; ++c) {
    const int d = lane + 64 * c;
    q[c] = d < dh ? ld(base + (size_t)i * rs + d) : 0.f;
    dc[c] = d < dh ? ld(dctx + ((size_t)i * b + j) * hp + (size_t)e * dh + d) : 0.f;
    acc[c] = 0.f;
  }
  const int kend = causal ? i : s - 1;
  const uint8_t* mrow = (!causal && mask) ? mask + ((size_t)j * s + i) * s : nullptr;
  for (int kk = 0; kk <= kend; ++kk) {
    const T* kr = base + (size_t)kk * rs + hp;
    const T* vr = kr + hp;
    float dot = 0.f, dpv = 0.f;
    float kv[kMaxDimsPerLane];
#pragma unroll
    for (int c = 0; c < kMaxDimsPerLane; ++c) {
      const int d = lane + 64 * c;
      kv[c] = d < dh ? ld(kr + d) : 0.f;
      dot += q[c] * kv[c];
      if (d < dh) dpv += dc[c] * ld(vr + d);
    }
    const bool hidden = mrow && mrow[kk];
    const float p = __expf((hidden ? kMaskFill : wave_sum(dot) * scale) - L);
    const float ds = hidden ? 0.f : p * (wave_sum(dpv) - D) * scale;
#pragma unroll
    for (int c = 0; c < kMaxDimsPerLane; ++c) acc[c] += ds * kv[c];
  }
#pragma unroll
  for (int c = 0; c < kMaxDimsPerLane; ++c) {
    const int d = lane + 64 * c;
    if (d < dh) st(dqkv + (size_t)i * rs + (size_t)j * 3 * hp + (size_t)e * dh + d, acc[c]);
  }
}

// dK, dV of key row kk: sums over queries i >= kk
template <typename T>
__global__ void __launch_bounds__(64)
attn_bwd_dkv_rowwise(const T* __restrict__ qkv, const T* __restrict__ dctx, const float* __restrict__ lse,
                     const float* __restrict__ delta, T* __restrict__ dqkv, int s, int b, int heads, int dh,
                     const uint8_t* __restrict__ mask, int causal) {
  const int kk = blockIdx.x, e = blockIdx.y, j = blockIdx.z, lane = threadIdx.x;
  const int hp = heads * dh;
  const size_t rs = (size_t)b * 3 * hp;
  const T* base = qkv + (size_t)j * 3 * hp + (size_t)e * dh;
  const float scale = rsqrtf((float)dh);
  float kv[kMaxDimsPerLane], vv[kMaxDimsPerLane], dk[kMaxDimsPerLane], dv[kMaxDimsPerLane];
#pragma unroll
  for (int c = 0; c < kMaxDimsPerLane; ++c) {
    const int d = lane + 64 * c;
    kv[c] = d < dh ? ld(base + (size_t)kk * rs + hp + d) : 0.f;
    vv[c] = d < dh ? ld(base + (size_t)kk * rs + 2 * hp + d) : 0.f;
    dk[c] = dv[c] = 0.f;
  }
  for (int i = causal ? kk : 0; i < s; ++i) {
    const T* qr = base + (size_t)i * rs;
    const T* dr = dctx + ((size_t)i * b + j) * hp + (size_t)e * dh;
    float qv[kMaxDimsPerLane], dc[kMaxDimsPerLane];
    float dot = 0.f, dpv = 0.f;
#pragma unroll
    for (int c = 0; c < kMaxDimsPerLane; ++c) {
      const int d = lane + 64 * c;
      qv[c] = d < dh ? ld(qr + d) : 0.f;
      dc[c] = d < dh ? ld(dr + d) : 0.f;
      dot += qv[c] * kv[c];
      dpv += dc[c] * vv[c];
    }
    const size_t st_i = ((size_t)j * heads + e) * s + i;
    const bool hidden = !causal && mask && mask[((size_t)j * s + i) * s + kk];
    const float p = __expf((hidden ? kMaskFill : wave_sum(dot) * scale) - lse[st_i]);
    const float ds = hidden ? 0.f : p * (wave_sum(dpv) - delta[st_i]) * scale;
#pragma unroll
    for (int c = 0; c < kMaxDimsPerLane; ++c) {
      dv[c] += p * dc[c];
      dk[c] += ds * qv[c];
    }
  }
#pragma unroll
  for (int c = 0; c < kMaxDimsPerLane; ++c) {
    const int d = lane + 64 * c;
    if (d < dh) {
      st(dqkv + (size_t)kk * rs + (size_t)j * 3 * hp + hp + (size_t)e * dh + d, dk[c]);
      st(dqkv + (size_t)kk * rs + (size_t)j * 3 * hp + 2 * hp + (size_t)e * dh + d, dv[c]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernels.  A workgroup is 2 waves and owns 64 queries (forward, dQ) or 64 keys (dK/dV); the
// other side streams through LDS in tiles of 64 rows kept in memory order [row][dh].  Operands whose
// contraction index is the tile row (V^T, K^T, Q^T, dO^T) are gathered from those same tiles with
// transposing LDS reads, so nothing is transposed in registers and every tile is stored once.
// ------------------------------------------------------------------------------------------------
constexpr int kBQ = 64;            // rows owned by a workgroup (2 waves x 32)
constexpr int kBKV = 64;           // rows per streamed LDS tile
constexpr int kAttnThreads = 128;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;

// bytes per LDS tile row: padded so that both the 16-byte fragment reads of 16 neighbouring rows and
// the 4-row x 32-byte gathers of the transposing reads spread over the banks
template <int DH> struct TileGeom {
  static constexpr int STRIDE = DH * 2 + (DH == 128 ? 32 : 16);
  static constexpr int BYTES = kBKV * STRIDE;
  static constexpr int NCH = kBKV * (DH / 8) / kAttnThreads;  // 16-byte chunks per thread and tile
};

// One 64-row tile of one head on its way global -> registers -> LDS (rows >= s read as zeros).
template <int DH> struct TileRegs {
  uint4 v[TileGeom<DH>::NCH];
  __device__ __forceinline__ void load(const bf16_t* __restrict__ src, size_t rs, int row0, int s) {
#pragma unroll
    for (int i = 0; i < TileGeom<DH>::NCH; ++i) {
      const int c = (threadIdx.x & (kAttnThreads - 1)) + i * kAttnThreads;
      const int row = c / (DH / 8), ch = c % (DH / 8);
      // branch-free: read a clamped (always valid) row, then blank it if it is past the end, so that
      // the loads of a tile are issued back to back
      const int rr = min(row0 + row, s - 1);
      const uint4 t = *reinterpret_cast<const uint4*>(src + (size_t)rr * rs + ch * 8);
      const bool ok = row0 + row < s;
      v[i] = make_uint4(ok ? t.x : 0u, ok ? t.y : 0u, ok ? t.z : 0u, ok ? t.w : 0u);
    }
  }
  __device__ __forceinline__ void store(char* lds) const {
#pragma unroll
    for (int i = 0; i < TileGeom<DH>::NCH; ++i) {
      const int c = (threadIdx.x & (kAttnThreads - 1)) + i * kAttnThreads;
      const int row = c / (DH / 8), ch = c % (DH / 8);
      *reinterpret_cast<uint4*>(lds + row * TileGeom<DH>::STRIDE + ch * 16) = v[i];
    }
  }
};

// This thread's chunk positions inside a tile, computed once: element offsets for the loads (rows rs
// apart) and byte offsets for the LDS stores.  A tile that lies wholly inside the sequence is then
// loaded with one add per chunk; the last, ragged tile takes TileRegs::load.
template <int DH> struct TileMap {
  uint32_t src[TileGeom<DH>::NCH];
  uint32_t dst[TileGeom<DH>::NCH];
  __device__ __forceinline__ void init(size_t rs) {
#pragma unroll
    for (int i = 0; i < TileGeom<DH>::NCH; ++i) {
      const int c = (threadIdx.x & (kAttnThreads - 1)) + i * kAttnThreads;
      const int row = c / (DH / 8), ch = c % (DH / 8);
      src[i] = (uint32_t)(row * rs + ch * 8);
      dst[i] = (uint32_t)(row * TileGeom<DH>::STRIDE + ch * 16);
    }
  }
  // rows row0 .. row0+63 of src (row pitch rs); s = number of valid rows
  __device__ __forceinline__ void load(TileRegs<DH>& t, const bf16_t* __restrict__ src_base, size_t rs, int row0,
                                       int s) const {
    if (row0 + kBKV <= s) {
      const bf16_t* p = src_base + (size_t)row0 * rs;
#pragma unroll
      for (int i = 0; i < TileGeom<DH>::NCH; ++i) t.v[i] = *reinterpret_cast<const uint4*>(p + src[i]);
    } else {
      t.load(src_base, rs, row0, s);
    }
  }
  __device__ __forceinline__ void store(const TileRegs<DH>& t, char* lds) const {
#pragma unroll
    for (int i = 0; i < TileGeom<DH>::NCH; ++i) *reinterpret_cast<uint4*>(lds + dst[i]) = t.v[i];
  }
};

// MFMA fragment with the tile row as the MFMA row: row = sub*32 + (lane & 31), eight consecutive dh of k16 step kk.
template <int DH>
__device__ __forceinline__ bf16x8_t frag_direct(const char* lds, int sub, int kk, int l31, int half) {
  return *reinterpret_cast<const bf16x8_t*>(lds + (sub * 32 + l31) * TileGeom<DH>::STRIDE + (kk * 2 + half) * 16);
}
// MFMA fragment with dh as the MFMA row (d*32 + (lane & 31)) and tile rows as the contraction index, taken in
// the order of the 32x32 accumulator rows that feed the other operand: rows 16*ks + 4*half + 0..3 and
// 16*ks + 8 + 4*half + 0..3 of 32-row half `sub`.  ds_read_b64_tr_b16: within 16 lanes, lane i receives
// element (i & 3) of the 8-byte rows addressed by lanes (i >> 2) + {0, 4, 8, 12}.
template <int DH>
__device__ __forceinline__ bf16x8_t frag_tr(const char* lds, int d, int sub, int ks, int lane) {
  const int r = lane & 15, G = lane >> 4;
  const int dh0 = d * 32 + 16 * (G & 1) + 4 * (r & 3);
  const int row = sub * 32 + ks * 16 + 4 * (G >> 1) + (r >> 2);
  const char* p = lds + row * TileGeom<DH>::STRIDE + dh0 * 2;
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
  const s16x4_t hi =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p + 8 * TileGeom<DH>::STRIDE));
  typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;
  s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return *reinterpret_cast<bf16x8_t*>(&v);
}
// Registers 8*ks .. 8*ks+7 of a 32x32 accumulator as a bf16 B-operand fragment.
__device__ __forceinline__ bf16x8_t pack_frag(const f32x16_t& a, int ks) {
  uint4 t = make_uint4(pack_bf16x2(a[ks * 8 + 0], a[ks * 8 + 1]), pack_bf16x2(a[ks * 8 + 2], a[ks * 8 + 3]),
                       pack_bf16x2(a[ks * 8 + 4], a[ks * 8 + 5]), pack_bf16x2(a[ks * 8 + 6], a[ks * 8 + 7]));
  return *reinterpret_cast<bf16x8_t*>(&t);
}
__device__ __forceinline__ f32x16_t zero16() {
  f32x16_t z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}
// lane's 8 consecutive dh (k16 step kk) of one token row, as a B-operand fragment straight from HBM
// (`row` must be readable; `ok` false blanks the fragment)
__device__ __forceinline__ bf16x8_t frag_global(const bf16_t* row, bool ok, int kk, int half) {
  const uint4 r = *reinterpret_cast<const uint4*>(row + kk * 16 + half * 8);
  uint4 t = make_uint4(ok ? r.x : 0u, ok ? r.y : 0u, ok ? r.z : 0u, ok ? r.w : 0u);
  return *reinterpret_cast<bf16x8_t*>(&t);
}
// accumulator rows (dh) of lane's column (token) -> 8-byte stores of 4 consecutive dh
template <int NDT>
__device__ __forceinline__ void store_cols(bf16_t* out_row, const f32x16_t (&acc)[NDT], float mul, int half) {
#pragma unroll
  for (int d = 0; d < NDT; ++d)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 w;
      w.x = pack_bf16x2(acc[d][4 * g] * mul, acc[d][4 * g + 1] * mul);
      w.y = pack_bf16x2(acc[d][4 * g + 2] * mul, acc[d][4 * g + 3] * mul);
      *reinterpret_cast<uint2*>(out_row + d * 32 + 8 * g + 4 * half) = w;
    }
}

// Hidden flags of keys key .. key+3 of one mask row as the four bytes of a word (keys >= s read as 0).
__device__ __forceinline__ uint32_t mask_word(const uint8_t* __restrict__ mrow, int key, int s, bool aligned) {
  if (aligned && key < s) return *reinterpret_cast<const uint32_t*>(mrow + key);   // s % 4 == 0: key + 3 < s
  uint32_t w = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (key + i < s) w |= (uint32_t)mrow[key + i] << (8 * i);
  return w;
}

// Work assignment.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: every block of one
// (sample, head) pair goes to the same XCD so that the pair's K and V stay in that L2, and each XCD
// takes its pairs one after the other - as long as whole rounds of 8 pairs remain.  The last heads * b mod 8 pairs
// are dealt block by block instead (block-major, so that each XCD gets the same share of every block index and
// with it of the causal triangle's work): 20 heads would otherwise leave four XCDs with three pairs and four
// with two.  Returns false for surplus ids.  `blk` counts up within a pair.
__device__ __forceinline__ bool attn_map(int id, int nblk, int heads, int b, int* blk, int* e, int* j) {
  const int xcd = id & 7, local = id >> 3;
  const int pairs = heads * b, whole = pairs >> 3, rest = pairs & 7;
  int pair;
  if (local < whole * nblk) {
    pair = xcd + 8 * (local / nblk);
    *blk = local % nblk;
  } else {
    const int g = (local - whole * nblk) * 8 + xcd;   // index into the remaining pairs' blocks, block-major
    if (g >= rest * nblk) return false;
    pair = 8 * whole + g % rest;
    *blk = g / rest;
  }
  *e = pair % heads;
  *j = pair / heads;
  return true;
}
inline int attn_grid(int nblk, int heads, int b) {
  const int pairs = heads * b, whole = pairs >> 3, rest = pairs & 7;
  return 8 * (whole * nblk + (rest * nblk + 7) / 8);
}

// Forward: S^T = K Q^T and O^T = V^T P^T, so that the probabilities leave the first MFMA in the register
// layout the second one takes as its B operand.  One tile's worth of registers carries V of the
// current step (requested before the score MFMAs, stored to LDS after the softmax) and then K of the
// next step (requested before the P V MFMAs), so both loads overlap arithmetic.  The loop is bound by
// vector ALU work, not by MFMA: the output is rescaled only when some row's running maximum moved,
// the mask is applied only on tiles that touch the diagonal, and exponentials and bf16 conversions
// are single instructions.
// NP = 2: the workgroup is two pairs of waves; pair p walks every second key tile with tiles of its own in LDS, and
// at the end pair 0 merges pair 1's running maximum, sum and output into its own (the usual rescaling of two
// partial softmax results).  For launches with so few workgroups that the longest one sets the time.
template <int DH, bool CAUSAL, int NP>
__global__ void __launch_bounds__(NP * kAttnThreads, DH > 128 ? 1 : 2)
attn_fwd_mfma(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx, float* __restrict__ lse, int s, int b,
              int heads, const uint8_t* __restrict__ mask) {
  constexpr int NKK = DH / 16, NDT = DH / 32;
  extern __shared__ __attribute__((aligned(16))) char smem_all[];
  const int pair = NP == 2 ? threadIdx.x >> 7 : 0;
  char* smem = smem_all + pair * 2 * TileGeom<DH>::BYTES;
  char* k_lds = smem;
  char* v_lds = smem + TileGeom<DH>::BYTES;

  const int nqb = (s + kBQ - 1) / kBQ;
  int qblk, e, j;
  if (!attn_map(blockIdx.x, nqb, heads, b, &qblk, &e, &j)) return;
  qblk = nqb - 1 - qblk;  // long rows first
  const int wave = (threadIdx.x >> 6) & 1, lane = threadIdx.x & 63, half = lane >> 5, l31 = lane & 31;
  const int hp = heads * DH;
  const size_t rs = (size_t)b * 3 * hp;
  const bf16_t* base = qkv + (size_t)j * 3 * hp + (size_t)e * DH;
  const int q_first = qblk * kBQ + wave * 32;  // first query of this wave
  const int my_q = q_first + l31;
  const float c2 = rsqrtf((float)DH) * 1.4426950408889634f;  // scale * log2(e)

  bf16x8_t qf[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) qf[kk] = frag_global(base + (size_t)min(my_q, s - 1) * rs, my_q < s, kk, half);

  f32x16_t o[NDT];
#pragma unroll
  for (int d = 0; d < NDT; ++d) o[d] = zero16();
  float m_run = -INFINITY, l_run = 0.f;

  const int q_last_blk = min(s, (qblk + 1) * kBQ) - 1;
  const int ntiles = CAUSAL ? q_last_blk / kBKV + 1 : (s + kBKV - 1) / kBKV;
  const uint8_t* mrow = (!CAUSAL && mask) ? mask + ((size_t)j * s + min(my_q, s - 1)) * s : nullptr;
  const bool aligned = (s & 3) == 0;
  const float fill = kMaskFill * sqrtf((float)DH);   // times 1/sqrt(dh) gives the fill value
  TileMap<DH> map;
  map.init(rs);
  TileRegs<DH> tr;
  if (pair < ntiles) {
    map.load(tr, base + hp, rs, pair * kBKV, s);
    map.store(tr, k_lds);
  }
  __syncthreads();
  // both pairs take the same number of steps (the barriers are the workgroup's); a pair without a tile idles
  for (int kt0 = 0; kt0 < ntiles; kt0 += NP) {
    const int kt = kt0 + pair;
    const bool have = kt < ntiles;
    const int key0 = kt * kBKV;
    const bool active = have && (!CAUSAL || key0 <= q_first + 31);  // else every key of the tile is in this wave's future
    if (have) map.load(tr, base + 2 * hp, rs, key0, s);
    uint32_t mw[2][4];
    if (!CAUSAL && mrow) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int g = 0; g < 4; ++g) mw[sub][g] = mask_word(mrow, key0 + sub * 32 + 8 * g + 4 * half, s, aligned);
    }

    bf16x8_t pf[2][2];
    if (active) {
      f32x16_t sacc[2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        sacc[sub] = zero16();
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
          sacc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct<DH>(k_lds, sub, kk, l31, half), qf[kk],
                                                              sacc[sub], 0, 0, 0);
      }
      if (CAUSAL) {
        // causal mask (also hides keys >= s, which are > every valid query); only tiles on the diagonal need it
        if (key0 + kBKV - 1 > q_first) {
#pragma unroll
          for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = key0 + sub * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
              sacc[sub][r] = key > my_q ? -INFINITY : sacc[sub][r];
            }
        }
      } else {
        if (mrow) {
#pragma unroll
          for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              sacc[sub][r] = ((mw[sub][r >> 2] >> (8 * (r & 3))) & 0xffu) ? fill : sacc[sub][r];
        }
        if (key0 + kBKV > s) {   // keys past the end of the sequence do not exist
#pragma unroll
          for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = key0 + sub * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
              sacc[sub][r] = key >= s ? -INFINITY : sacc[sub][r];
            }
        }
      }
      float mx = m_run;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[sub][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      if (__any(mx > m_run)) {   // some row's maximum moved: rescale what has been accumulated
        const float corr = __builtin_amdgcn_exp2f((m_run - mx) * c2);
        m_run = mx;
        l_run *= corr;
#pragma unroll
        for (int d = 0; d < NDT; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= corr;
      }
      const float mc = mx * c2;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          sacc[sub][r] = __builtin_amdgcn_exp2f(sacc[sub][r] * c2 - mc);
          l_run += sacc[sub][r];
        }
        pf[sub][0] = pack_frag(sacc[sub], 0);
        pf[sub][1] = pack_frag(sacc[sub], 1);
      }
    }
    if (have) map.store(tr, v_lds);
    __syncthreads();   // V visible; every wave is done with K of this step
    if (kt + NP < ntiles) map.load(tr, base + hp, rs, key0 + NP * kBKV, s);
    if (active) {
#pragma unroll
      for (int d = 0; d < NDT; ++d)
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int ks = 0; ks < 2; ++ks)
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<DH>(v_lds, d, sub, ks, lane), pf[sub][ks], o[d], 0, 0, 0);
    }
    if (kt + NP < ntiles) map.store(tr, k_lds);
    __syncthreads();   // next K visible; every wave is done with V of this step
  }
  l_run += __shfl_xor(l_run, 32, 64);
  if constexpr (NP == 2) {
    // pair 1's partial result joins pair 0's: value v of lane l of wave w at part[w][v][l]
    float* part = reinterpret_cast<float*>(smem_all) + wave * ((2 + NDT * 16) * 64) + lane;
    if (pair == 1) {
      part[0] = m_run;
      part[64] = l_run;
#pragma unroll
      for (int d = 0; d < NDT; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[(2 + d * 16 + r) * 64] = o[d][r];
    }
    __syncthreads();
    if (pair == 1) return;
    const float m1 = part[0], l1 = part[64];
    const float m = fmaxf(m_run, m1);   // pair 0 always has tile 0, whose key 0 every query sees: m_run is finite
    const float a0 = __builtin_amdgcn_exp2f((m_run - m) * c2), a1 = __builtin_amdgcn_exp2f((m1 - m) * c2);
    l_run = l_run * a0 + l1 * a1;
    m_run = m;
#pragma unroll
    for (int d = 0; d < NDT; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[d][r] = o[d][r] * a0 + part[(2 + d * 16 + r) * 64] * a1;
  }
  if (my_q < s) {
    store_cols<NDT>(ctx + ((size_t)my_q * b + j) * hp + (size_t)e * DH, o, 1.f / l_run, half);
    if (half == 0) lse[((size_t)j * heads + e) * s + my_q] = m_run * rsqrtf((float)DH) + __logf(l_run);
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA backward.  P is recomputed from the stashed log-sum-exp; two kernels so that no result
// needs atomics: one owns 64 queries and produces dQ, one owns 64 keys and produces dK and dV.
//   dP = dO V^T, dS = P o (dP - delta), dQ = dS K / sqrt(dh), dK = dS^T Q / sqrt(dh), dV = P^T dO
// ------------------------------------------------------------------------------------------------
// dQ: a workgroup owns 64 queries.  NP = 2: it is two pairs of waves; pair p walks every second 64-key tile with
// tiles of its own in LDS and pair 1 hands its sums to pair 0 at the end (see the dK/dV kernel below for when).
template <int DH, bool CAUSAL, int NP>
__global__ void __launch_bounds__(NP * kAttnThreads, DH >= 96 ? 1 : 2)
attn_bwd_dq_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx, const float* __restrict__ lse,
                 const float* __restrict__ delta, bf16_t* __restrict__ dqkv, int s, int b, int heads,
                 const uint8_t* __restrict__ mask) {
  constexpr int NKK = DH / 16, NDT = DH / 32;
  extern __shared__ __attribute__((aligned(16))) char smem_all[];
  const int pair = NP == 2 ? threadIdx.x >> 7 : 0;
  char* smem = smem_all + pair * 2 * TileGeom<DH>::BYTES;
  char* k_lds = smem;                          // K [key][dh]: S^T = K Q^T directly, dQ^T = K^T dS^T through tr reads
  char* v_lds = smem + TileGeom<DH>::BYTES;    // V [key][dh]: dP^T = V dO^T

  const int nqb = (s + kBQ - 1) / kBQ;
  int qblk, e, j;
  if (!attn_map(blockIdx.x, nqb, heads, b, &qblk, &e, &j)) return;
  qblk = nqb - 1 - qblk;
  const int wave = (threadIdx.x >> 6) & 1, lane = threadIdx.x & 63, half = lane >> 5, l31 = lane & 31;
  const int hp = heads * DH;
  const size_t rs = (size_t)b * 3 * hp;
  const bf16_t* base = qkv + (size_t)j * 3 * hp + (size_t)e * DH;
  const int q_first = qblk * kBQ + wave * 32;
  const int my_q = q_first + l31;
  const bool valid = my_q < s;
  const float scale = rsqrtf((float)DH), c2 = scale * 1.4426950408889634f;
  const size_t stat = ((size_t)j * heads + e) * s + my_q;
  const float L2 = valid ? lse[stat] * 1.4426950408889634f : 0.f;
  const float D = valid ? delta[stat] : 0.f;

  bf16x8_t qf[NKK], dof[NKK];
  const bf16_t* dorow = dctx + ((size_t)min(my_q, s - 1) * b + j) * hp + (size_t)e * DH;
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    qf[kk] = frag_global(base + (size_t)min(my_q, s - 1) * rs, valid, kk, half);
    dof[kk] = frag_global(dorow, valid, kk, half);
  }
  f32x16_t acc[NDT];
#pragma unroll
  for (int d = 0; d < NDT; ++d) acc[d] = zero16();

  const int q_last_blk = min(s, (qblk + 1) * kBQ) - 1;
  const int ntiles = CAUSAL ? q_last_blk / kBKV + 1 : (s + kBKV - 1) / kBKV;
  const uint8_t* mrow = (!CAUSAL && mask) ? mask + ((size_t)j * s + min(my_q, s - 1)) * s : nullptr;
  const bool aligned = (s & 3) == 0;
  const float fill = kMaskFill * sqrtf((float)DH);
  // the next K and V tiles travel in registers while this step's arithmetic runs
  TileMap<DH> map;
  map.init(rs);
  TileRegs<DH> kr, vr;
  if (pair < ntiles) {
    map.load(kr, base + hp, rs, pair * kBKV, s);
    map.load(vr, base + 2 * hp, rs, pair * kBKV, s);
  }
  // both pairs take the same number of steps (the barriers are the workgroup's); a pair without a tile idles
  for (int kt0 = 0; kt0 < ntiles; kt0 += NP) {
    const int kt = kt0 + pair;
    const bool have = kt < ntiles;
    const int key0 = kt * kBKV;
    __syncthreads();
    if (have) {
      map.store(kr, k_lds);
      map.store(vr, v_lds);
    }
    __syncthreads();
    if (!have) continue;
    if (kt + NP < ntiles) {
      map.load(kr, base + hp, rs, key0 + NP * kBKV, s);
      map.load(vr, base + 2 * hp, rs, key0 + NP * kBKV, s);
    }
    if (CAUSAL && key0 > q_first + 31) continue;
    const bool diag = key0 + kBKV - 1 > q_first;   // only tiles on the diagonal need the causal mask
    bf16x8_t dsf[2][2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      uint32_t mw[4] = {0u, 0u, 0u, 0u};
      if (!CAUSAL && mrow) {
#pragma unroll
        for (int g = 0; g < 4; ++g) mw[g] = mask_word(mrow, key0 + sub * 32 + 8 * g + 4 * half, s, aligned);
      }
      f32x16_t sacc = zero16(), dp = zero16();
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct<DH>(k_lds, sub, kk, l31, half), qf[kk], sacc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct<DH>(v_lds, sub, kk, l31, half), dof[kk], dp, 0, 0, 0);
      }
      if (!CAUSAL) {
        // a hidden score is the constant fill: its probability counts (through D) but it passes no gradient;
        // keys past the end do not exist (an empty row's lse is so low that their exp2 would overflow)
        const bool tail = key0 + kBKV > s;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + sub * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
          const bool hidden = ((mw[r >> 2] >> (8 * (r & 3))) & 0xffu) || (tail && key >= s);
          sacc[r] = hidden ? 0.f : __builtin_amdgcn_exp2f(sacc[r] * c2 - L2) * (dp[r] - D);
        }
      } else if (diag) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + sub * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
          const float p = __builtin_amdgcn_exp2f(sacc[r] * c2 - L2);
          sacc[r] = key > my_q ? 0.f : p * (dp[r] - D);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = __builtin_amdgcn_exp2f(sacc[r] * c2 - L2) * (dp[r] - D);
      }
      dsf[sub][0] = pack_frag(sacc, 0);
      dsf[sub][1] = pack_frag(sacc, 1);
    }
#pragma unroll
    for (int d = 0; d < NDT; ++d)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
          acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<DH>(k_lds, d, sub, ks, lane), dsf[sub][ks], acc[d], 0, 0, 0);
  }
  if constexpr (NP == 2) {
    // pair 1's sums join pair 0's: register r of lane l of wave w at sum[w][r][l]
    __syncthreads();   // every wave is done with the tiles
    float* sum = reinterpret_cast<float*>(smem_all) + wave * (NDT * 16 * 64) + lane;
    if (pair == 1) {
#pragma unroll
      for (int d = 0; d < NDT; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[(d * 16 + r) * 64] = acc[d][r];
    }
    __syncthreads();
    if (pair == 1) return;
#pragma unroll
    for (int d = 0; d < NDT; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[d][r] += sum[(d * 16 + r) * 64];
  }
  if (valid) store_cols<NDT>(dqkv + (size_t)my_q * rs + (size_t)j * 3 * hp + (size_t)e * DH, acc, scale, half);
}

constexpr int kMaskLdsStride = 68;   // bytes per key row of the staged mask tile ([key][query], padded)

// dK/dV: a workgroup owns 64 keys; wave w of a pair owns keys 32 w .. 32 w + 31.  NP = 1: one pair of waves walks all
// 64-query tiles.  NP = 2: two pairs; pair p walks every second tile (first + p, first + p + 2, ...) with tiles of its
// own in LDS, and at the end pair 1 hands its sums to pair 0 through LDS, added in that fixed order.  The workgroup
// that owns the first keys of a causal head walks all query tiles and the launch lasts at least as long as it does:
// two pairs halve that path, at the price of one barrier domain per CU instead of two independent ones.  The launch
// code takes NP = 2 when all workgroups of the one-pair form would be resident at once (the longest one then sets
// the time: GPT-3-shaped shard, 12 heads: backward 0.213 -> 0.152 ms) and NP = 1 otherwise (1T-shaped shard, 20
// heads of 160: 0.331 against 0.343 ms).
template <int DH, bool CAUSAL> struct DkvLds {
  static constexpr int kPair = 2 * TileGeom<DH>::BYTES + 2 * kBKV * (int)sizeof(float) + (CAUSAL ? 0 : kBQ * kMaskLdsStride);
  static constexpr int kSum = 2 * (DH / 32) * 16 * 64 * (int)sizeof(float);   // one wave's dK and dV
  static constexpr int kBytes2 = 2 * kPair > 2 * kSum ? 2 * kPair : 2 * kSum;
};
template <int DH, bool CAUSAL, int NP>
__global__ void __launch_bounds__(NP * kAttnThreads)
attn_bwd_dkv_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx, const float* __restrict__ lse,
                  const float* __restrict__ delta, bf16_t* __restrict__ dqkv, int s, int b, int heads,
                  const uint8_t* __restrict__ mask) {
  constexpr int NKK = DH / 16, NDT = DH / 32;
  extern __shared__ __attribute__((aligned(16))) char smem_all[];
  const int pair = NP == 2 ? threadIdx.x >> 7 : 0, tid = threadIdx.x & (kAttnThreads - 1);
  char* smem = smem_all + pair * DkvLds<DH, CAUSAL>::kPair;
  char* q_lds = smem;                           // Q  [query][dh]: S = Q K^T directly, dK^T = Q^T dS through tr reads
  char* do_lds = smem + TileGeom<DH>::BYTES;    // dO [query][dh]: dP = dO V^T directly, dV^T = dO^T P through tr reads
  float* lse_lds = reinterpret_cast<float*>(smem + 2 * TileGeom<DH>::BYTES);  // lse * log2(e), +inf past the end
  float* delta_lds = lse_lds + kBKV;
  uint8_t* mask_lds = reinterpret_cast<uint8_t*>(delta_lds + kBKV);   // general mask only: [64 keys][68]
  const bool use_mask = !CAUSAL && mask != nullptr;
  const float fill = kMaskFill * sqrtf((float)DH);

  int kblk, e, j;  // the first key blocks see the most queries and start first
  if (!attn_map(blockIdx.x, (s + kBQ - 1) / kBQ, heads, b, &kblk, &e, &j)) return;
  const int wave = (threadIdx.x >> 6) & 1, lane = threadIdx.x & 63, half = lane >> 5, l31 = lane & 31;
  const int hp = heads * DH;
  const size_t rs = (size_t)b * 3 * hp;
  const bf16_t* base = qkv + (size_t)j * 3 * hp + (size_t)e * DH;
  const bf16_t* dobase = dctx + (size_t)j * hp + (size_t)e * DH;
  const size_t dors = (size_t)b * hp;
  const int key_first = kblk * kBQ + wave * 32;
  const int my_key = key_first + l31;
  const bool valid = my_key < s;
  const float scale = rsqrtf((float)DH), c2 = scale * 1.4426950408889634f;
  const float* lse_h = lse + ((size_t)j * heads + e) * s;
  const float* delta_h = delta + ((size_t)j * heads + e) * s;

  bf16x8_t kf[NKK], vf[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    kf[kk] = frag_global(base + (size_t)min(my_key, s - 1) * rs + hp, valid, kk, half);
    vf[kk] = frag_global(base + (size_t)min(my_key, s - 1) * rs + 2 * hp, valid, kk, half);
  }
  f32x16_t dk[NDT], dv[NDT];
#pragma unroll
  for (int d = 0; d < NDT; ++d) {
    dk[d] = zero16();
    dv[d] = zero16();
  }
  const int nq_tiles = (s + kBKV - 1) / kBKV;
  // the next Q and dO tiles (and their lse, delta) travel in registers while this step's arithmetic runs
  // (not for the largest head size: the tiles would not fit the register file next to dK and dV)
  constexpr bool kPrefetch = DH <= 128;
  TileMap<kPrefetch ? DH : 32> qmap, domap;
  TileRegs<kPrefetch ? DH : 32> qr, dor;
  float lse_r = 0.f, delta_r = 0.f;
  auto fetch = [&](int q0) {
    if constexpr (kPrefetch) {
      qmap.load(qr, base, rs, q0, s);
      domap.load(dor, dobase, dors, q0, s);
      if (tid < kBKV) {
        const int q = q0 + tid;
        lse_r = q < s ? lse_h[q] * 1.4426950408889634f : INFINITY;
        delta_r = q < s ? delta_h[q] : 0.f;
      }
    }
  };
  const int qt_first = CAUSAL ? (kblk * kBQ) / kBKV : 0;
  if constexpr (kPrefetch) {
    qmap.init(rs);
    domap.init(dors);
    if (qt_first + pair < nq_tiles) fetch((qt_first + pair) * kBKV);
  }
  // both pairs take the same number of steps (the barriers are the workgroup's); a pair without a tile idles
  for (int qt0 = qt_first; qt0 < nq_tiles; qt0 += NP) {
    const int qt = qt0 + pair;
    const bool have = qt < nq_tiles;
    const int q0 = qt * kBKV;
    __syncthreads();
    if (have) {
      if constexpr (kPrefetch) {
        qmap.store(qr, q_lds);
        domap.store(dor, do_lds);
        if (tid < kBKV) {
          lse_lds[tid] = lse_r;
          delta_lds[tid] = delta_r;
        }
      } else {
        TileRegs<DH> t;
        t.load(base, rs, q0, s);
        t.store(q_lds);
        t.load(dobase, dors, q0, s);
        t.store(do_lds);
        if (tid < kBKV) {
          const int q = q0 + tid;
          lse_lds[tid] = q < s ? lse_h[q] * 1.4426950408889634f : INFINITY;
          delta_lds[tid] = q < s ? delta_h[q] : 0.f;
        }
      }
      if (use_mask) {   // this tile of the mask, transposed to [key][query] so that a lane reads 4 queries at once
        for (int idx = tid; idx < kBKV * kBQ; idx += kAttnThreads) {
          const int ql = idx / kBQ, kl = idx % kBQ;
          const int q = q0 + ql, key = kblk * kBQ + kl;
          mask_lds[kl * kMaskLdsStride + ql] = (q < s && key < s) ? mask[((size_t)j * s + q) * s + key] : (uint8_t)0;
        }
      }
    }
    __syncthreads();
    if (!have) continue;
    if (qt + NP < nq_tiles) fetch(q0 + NP * kBKV);
    if (CAUSAL && q0 + kBKV - 1 < key_first) continue;  // every query of the tile precedes this wave's keys
    const bool diag = CAUSAL && q0 < key_first + 32;    // some query of the tile precedes some key of this wave
    bf16x8_t pf[2][2], dsf[2][2];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      f32x16_t sacc = zero16(), dp = zero16();
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct<DH>(q_lds, sub, kk, l31, half), kf[kk], sacc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct<DH>(do_lds, sub, kk, l31, half), vf[kk], dp, 0, 0, 0);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ql = sub * 32 + 8 * g + 4 * half;  // local index of the first of 4 consecutive queries
        const float4 L4 = *reinterpret_cast<const float4*>(lse_lds + ql);
        const float4 D4 = *reinterpret_cast<const float4*>(delta_lds + ql);
        const float Ls[4] = {L4.x, L4.y, L4.z, L4.w}, Ds[4] = {D4.x, D4.y, D4.z, D4.w};
        const uint32_t mw = use_mask ? *reinterpret_cast<const uint32_t*>(mask_lds + (wave * 32 + l31) * kMaskLdsStride + ql) : 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = 4 * g + i;
          const bool hidden = (mw >> (8 * i)) & 0xffu;
          float p = __builtin_amdgcn_exp2f((hidden ? fill : sacc[r]) * c2 - Ls[i]);   // lse = +inf past the end gives 0
          if (diag) p = my_key > q0 + ql + i ? 0.f : p;
          sacc[r] = p;
          dp[r] = hidden ? 0.f : p * (dp[r] - Ds[i]);
        }
      }
      pf[sub][0] = pack_frag(sacc, 0);
      pf[sub][1] = pack_frag(sacc, 1);
      dsf[sub][0] = pack_frag(dp, 0);
      dsf[sub][1] = pack_frag(dp, 1);
    }
#pragma unroll
    for (int d = 0; d < NDT; ++d)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          dv[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<DH>(do_lds, d, sub, ks, lane), pf[sub][ks], dv[d], 0, 0, 0);
          dk[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<DH>(q_lds, d, sub, ks, lane), dsf[sub][ks], dk[d], 0, 0, 0);
        }
  }
  if constexpr (NP == 2) {
    // pair 1's sums join pair 0's: register r of lane l of wave w at sum[w][r][l]
    __syncthreads();   // every wave is done with the tiles
    float* sum = reinterpret_cast<float*>(smem_all) + wave * (2 * NDT * 16 * 64) + lane;
    if (pair == 1) {
#pragma unroll
      for (int d = 0; d < NDT; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          sum[(d * 16 + r) * 64] = dk[d][r];
          sum[((NDT + d) * 16 + r) * 64] = dv[d][r];
        }
    }
    __syncthreads();
    if (pair == 1) return;
#pragma unroll
    for (int d = 0; d < NDT; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        dk[d][r] += sum[(d * 16 + r) * 64];
        dv[d][r] += sum[((NDT + d) * 16 + r) * 64];
      }
  }
  if (valid) {
    bf16_t* out = dqkv + (size_t)my_key * rs + (size_t)j * 3 * hp + (size_t)e * DH;
    store_cols<NDT>(out + hp, dk, scale, half);
    store_cols<NDT>(out + 2 * hp, dv, 1.f, half);
  }
}

// delta[j][e][i] = sum_d dctx[i][j][e][d] * ctx[i][j][e][d]; one wave per (token, head), 4 per block
__global__ void __launch_bounds__(256)
attn_delta_bf16(const bf16_t* __restrict__ ctx, const bf16_t* __restrict__ dctx, float* __restrict__ delta, int s, int b,
                int heads, int dh) {
  const int lane = threadIdx.x & 63;
  const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (token, head) pair index
  const size_t nrows = (size_t)s * b * heads;
  if (row >= nrows) return;
  const size_t tok = row / heads;
  const int e = (int)(row % heads);
  const int i = (int)(tok / b), j = (int)(tok % b);
  const bf16_t* c = ctx + row * dh;
  const bf16_t* d = dctx + row * dh;
  float a = 0.f;
  for (int v = lane; v < dh / 8; v += 64) {
    Vec16<bf16_t> x, y;
    float xf[8], yf[8];
    x.load(c + v * 8);
    y.load(d + v * 8);
    x.unpack(xf);
    y.unpack(yf);
#pragma unroll
    for (int t = 0; t < 8; ++t) a += xf[t] * yf[t];
  }
  a = wave_sum(a);
  if (lane == 0) delta[((size_t)j * heads + e) * s + i] = a;
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
bool attn_dh_supported(int dtype, int dh) {
  if (dh <= 0 || dh % 8 != 0) return false;
  if (dtype == PTDP_F32) return dh <= 64 * kMaxDimsPerLane;
  return dh == 32 || dh == 64 || dh == 96 || dh == 128 || dh == 160;
}

static inline double attn_flops(int s, int b, int heads, int dh) { return 4.0 * b * heads * (double)s * s * dh; }

// resident workgroups of the one-pair kernels: two per CU (one wave per SIMD each)
static int attn_resident_pairs() {
  static std::atomic<int> cached[kMaxDevices];   // per device, looked up once
  const int d = device_slot();
  if (d >= 0 && cached[d].load(std::memory_order_relaxed) > 0) return cached[d].load(std::memory_order_relaxed);
  int dev = 0, cu = 256;
  if (hipGetDevice(&dev) == hipSuccess) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cu = v;
  }
  if (d >= 0) cached[d].store(2 * cu, std::memory_order_relaxed);
  return 2 * cu;
}
template <int DH, bool CAUSAL, int NP>
static int attn_fwd_mfma_np(const bf16_t* qkv, bf16_t* ctx, float* lse, int s, int b, int heads, const uint8_t* mask,
                            hipStream_t stream) {
  constexpr int smem = NP * 2 * TileGeom<DH>::BYTES;   // (NP = 2: the partial results, (2 + DH / 2) x 512 bytes, fit in the tiles)
  static once_flag_t done[kMaxDevices];
  if (set_dynamic_smem(reinterpret_cast<const void*>(attn_fwd_mfma<DH, CAUSAL, NP>), smem, done) != PTDP_OK) return PTDP_E_HIP;
  const dim3 grid(attn_grid((s + kBQ - 1) / kBQ, heads, b));
  hipLaunchKernelGGL((attn_fwd_mfma<DH, CAUSAL, NP>), grid, dim3(NP * kAttnThreads), smem, stream, qkv, ctx, lse, s, b, heads,
                     mask);
  return PTDP_OK;
}
template <int DH, bool CAUSAL>
static int attn_fwd_mfma_t(const bf16_t* qkv, bf16_t* ctx, float* lse, int s, int b, int heads, const uint8_t* mask,
                           hipStream_t stream) {
  // few workgroups: the longest one sets the time, so split its walk over two pairs of waves
  const long long wgs = (long long)((s + kBQ - 1) / kBQ) * heads * b;
  if (wgs <= attn_resident_pairs()) return attn_fwd_mfma_np<DH, CAUSAL, 2>(qkv, ctx, lse, s, b, heads, mask, stream);
  return attn_fwd_mfma_np<DH, CAUSAL, 1>(qkv, ctx, lse, s, b, heads, mask, stream);
}

// Without the causal mask every row is a full row: count the whole s x s square as executed too.
int launch_attn_fwd(int dtype, const void* qkv, void* ctx, float* lse, int s, int b, int heads, int dh,
                    const uint8_t* mask, int causal, hipStream_t stream) {
  if (s == 0 || b == 0 || heads == 0) return PTDP_OK;
  if (!attn_dh_supported(dtype, dh)) return PTDP_E_UNSUPPORTED;
  Launch L(PTDP_K_ATTN_FWD, attn_flops(s, b, heads, dh), stream);
  int rc = PTDP_OK;
  if (dtype == PTDP_F32) {
    hipLaunchKernelGGL((attn_fwd_rowwise<float>), dim3(s, heads, b), dim3(64), 0, stream, (const float*)qkv,
                       (float*)ctx, lse, s, b, heads, dh, mask, causal);
  } else {
    const bf16_t* q = (const bf16_t*)qkv;
    bf16_t* c = (bf16_t*)ctx;
#define PTDP_ATTN_FWD(D) \
  rc = causal ? attn_fwd_mfma_t<D, true>(q, c, lse, s, b, heads, mask, stream) \
              : attn_fwd_mfma_t<D, false>(q, c, lse, s, b, heads, mask, stream)
    if (dh == 32) PTDP_ATTN_FWD(32);
    else if (dh == 96) PTDP_ATTN_FWD(96);
    else if (dh == 64) PTDP_ATTN_FWD(64);
    else if (dh == 128) PTDP_ATTN_FWD(128);
    else PTDP_ATTN_FWD(160);
#undef PTDP_ATTN_FWD
  }
  if (rc != PTDP_OK) return rc;
  return L.status();
}

template <typename T>
static int attn_bwd_rowwise_t(const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv,
                              float* delta, int s, int b, int heads, int dh, const uint8_t* mask, int causal,
                              hipStream_t stream) {
  const dim3 grid(s, heads, b);
  hipLaunchKernelGGL((attn_delta_rowwise<T>), grid, dim3(64), 0, stream, (const T*)ctx, (const T*)dctx, delta, s, b,
                     heads, dh);
  hipLaunchKernelGGL((attn_bwd_dq_rowwise<T>), grid, dim3(64), 0, stream, (const T*)qkv, (const T*)dctx, lse, delta,
                     (T*)dqkv, s, b, heads, dh, mask, causal);
  hipLaunchKernelGGL((attn_bwd_dkv_rowwise<T>), grid, dim3(64), 0, stream, (const T*)qkv, (const T*)dctx, lse, delta,
                     (T*)dqkv, s, b, heads, dh, mask, causal);
  return PTDP_OK;
}

template <int DH, bool CAUSAL, int NP>
static int attn_bwd_mfma_np(const bf16_t* qkv, const bf16_t* dctx, const float* lse, const float* delta, bf16_t* dqkv, int s,
                            int b, int heads, const uint8_t* mask, hipStream_t stream) {
  constexpr int smem_dq = NP * 2 * TileGeom<DH>::BYTES;   // (NP = 2: the final sums, 2 x DH x 256 bytes, fit in the tiles)
  constexpr int smem_dkv = NP == 2 ? DkvLds<DH, CAUSAL>::kBytes2 : DkvLds<DH, CAUSAL>::kPair;
  static once_flag_t done_dq[kMaxDevices], done_dkv[kMaxDevices];
  if (set_dynamic_smem(reinterpret_cast<const void*>(attn_bwd_dq_mfma<DH, CAUSAL, NP>), smem_dq, done_dq) != PTDP_OK ||
      set_dynamic_smem(reinterpret_cast<const void*>(attn_bwd_dkv_mfma<DH, CAUSAL, NP>), smem_dkv, done_dkv) != PTDP_OK)
    return PTDP_E_HIP;
  const dim3 grid(attn_grid((s + kBQ - 1) / kBQ, heads, b));
  hipLaunchKernelGGL((attn_bwd_dkv_mfma<DH, CAUSAL, NP>), grid, dim3(NP * kAttnThreads), smem_dkv, stream, qkv, dctx, lse, delta,
                     dqkv, s, b, heads, mask);
  hipLaunchKernelGGL((attn_bwd_dq_mfma<DH, CAUSAL, NP>), grid, dim3(NP * kAttnThreads), smem_dq, stream, qkv, dctx, lse, delta,
                     dqkv, s, b, heads, mask);
  return PTDP_OK;
}
template <int DH, bool CAUSAL>
static int attn_bwd_mfma_t(const bf16_t* qkv, const bf16_t* ctx, const float* lse, const bf16_t* dctx, bf16_t* dqkv,
                           float* delta, int s, int b, int heads, const uint8_t* mask, hipStream_t stream) {
  const size_t nrows = (size_t)s * b * heads;
  hipLaunchKernelGGL(attn_delta_bf16, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, stream, ctx, dctx, delta, s, b,
                     heads, DH);
  // few workgroups: the longest one sets the time, so split its walk over two pairs of waves
  const long long wgs = (long long)((s + kBQ - 1) / kBQ) * heads * b;
  if (wgs <= attn_resident_pairs())
    return attn_bwd_mfma_np<DH, CAUSAL, 2>(qkv, dctx, lse, delta, dqkv, s, b, heads, mask, stream);
  return attn_bwd_mfma_np<DH, CAUSAL, 1>(qkv, dctx, lse, delta, dqkv, s, b, heads, mask, stream);
}

int launch_attn_bwd(int dtype, const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv,
                    float* delta, int s, int b, int heads, int dh, const uint8_t* mask, int causal, hipStream_t stream) {
  if (s == 0 || b == 0 || heads == 0) return PTDP_OK;
  if (!attn_dh_supported(dtype, dh)) return PTDP_E_UNSUPPORTED;
  Launch L(PTDP_K_ATTN_BWD, 2.0 * attn_flops(s, b, heads, dh), stream);
  int rc = PTDP_OK;
  if (dtype == PTDP_F32) {
    rc = attn_bwd_rowwise_t<float>(qkv, ctx, lse, dctx, dqkv, delta, s, b, heads, dh, mask, causal, stream);
  } else {
    const bf16_t* q = (const bf16_t*)qkv;
    const bf16_t* c = (const bf16_t*)ctx;
    const bf16_t* d = (const bf16_t*)dctx;
    bf16_t* o = (bf16_t*)dqkv;
#define PTDP_ATTN_BWD(D) \
  rc = causal ? attn_bwd_mfma_t<D, true>(q, c, lse, d, o, delta, s, b, heads, mask, stream) \
              : attn_bwd_mfma_t<D, false>(q, c, lse, d, o, delta, s, b, heads, mask, stream)
    if (dh == 32) PTDP_ATTN_BWD(32);
    else if (dh == 96) PTDP_ATTN_BWD(96);
    else if (dh == 64) PTDP_ATTN_BWD(64);
    else if (dh == 128) PTDP_ATTN_BWD(128);
    else PTDP_ATTN_BWD(160);
#undef PTDP_ATTN_BWD
  }
  if (rc != PTDP_OK) return rc;
  return L.status();
}

}  // namespace ptdp
