// GEMMs of the layer (paper appendix: QKV, attention output projection, MLP h->4h/t and 4h/t->h, and
// for each the input-gradient and weight-gradient products of the backward pass).
//
//   mode NN: C[M,N] = A[M,K] B[K,N]          forward      Y  = X W
//   mode NT: C[M,N] = A[M,K] B[N,K]^T        input grad   dX = dY W^T
//   mode TN: C[M,N] = A[K,M]^T B[K,N]        weight grad  dW = X^T dY
//
// bf16 path (gfx950): v_mfma_f32_16x16x32_bf16 for NN and NT, v_mfma_f32_32x32x16_bf16 for TN; 256 x 256 block
// tile, two LDS stages of 64 k filled by direct global->LDS loads.  An operand whose reduction index is the slow
// memory index (B in NN, both in TN) stays in its memory order in LDS and is gathered into MFMA fragments by
// transposing LDS reads.
// fp32 path: a plain LDS-tiled FMA kernel (correctness configuration only).
#include "common.h"
#include <type_traits>

namespace ptdp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

// ------------------------------------------------------------------------------------------------
// fp32: 64 x 64 x 16 tile, 256 threads, 4 x 4 outputs per thread, generic strides.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ B, float* C, const float* __restrict__ bias,
                int M, int N, int K, size_t a_rs, size_t a_cs, size_t b_rs, size_t b_cs, int accumulate) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int e = threadIdx.x; e < 16 * 64; e += 256) {
      const int kk = e & 15, r = e >> 4;  // consecutive threads walk k, then rows
      const int m = m0 + r, n = n0 + r, k = k0 + kk;
      As[kk][r] = (m < M && k < K) ? A[(size_t)m * a_rs + (size_t)k * a_cs] : 0.f;
      Bs[kk][r] = (n < N && k < K) ? B[(size_t)k * b_rs + (size_t)n * b_cs] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = As[kk][ty * 4 + i];
        b[i] = Bs[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j] + (bias ? bias[n] : 0.f);
      float* c = C + (size_t)m * N + n;
      *c = accumulate ? *c + v : v;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel: global -> LDS without passing through registers (buffer_load ... lds, 16 bytes
// per lane), 256 x 256 x 64 block tile, 8 waves (2 x 4, 128 x 64 each), two LDS stages.
// Out-of-range lanes use an offset beyond the buffer's num_records, for which the hardware returns
// zeros.
//
// LDS tile layouts:
//   k-contiguous operand: [row][8 chunks of 16 B]; chunk c of row r sits in slot c ^ f(r), f chosen
//     so that 16 neighbouring rows of one fragment read fall into 16 different 16-byte bank groups.
//   k-slow operand (memory [k][row]): [k][32 chunks of 16 B] (512 B per k); chunk c of k-row k sits in
//     slot c ^ (4 * (k & 3)) ^ (2 * ((k >> 3) & 1)): the four k-rows that one group of 16 lanes gathers land in
//     different bank groups, and so do k-rows 8 apart, which the 16x16x32 fragments read in the same cycle.
//     MFMA fragments are gathered with ds_read_b64_tr_b16: within 16 lanes, lane i receives element (i & 3) of
//     the 8-byte rows addressed by lanes (i >> 2) + {0, 4, 8, 12}.
// ------------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) void lds_void_t;

constexpr uint32_t kOob = 0x80000000u;  // beyond any num_records this kernel accepts (< 2 GiB)

// Buffer descriptor (raw, no stride, no swizzle): 48-bit base, bytes, data format dword.
typedef uint32_t rsrc_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(p);
  rsrc_t r = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};
  return r;
}
__device__ __forceinline__ uint32_t lds_offset(const char* p) {
  return (uint32_t)reinterpret_cast<uintptr_t>((lds_void_t*)p);
}

// Global -> LDS loads (16 bytes per lane, lane i lands at dst + 16*i; dst wave-uniform) are written as assembly:
// the compiler makes every LDS read that it cannot prove disjoint (all transposing reads) wait for every such
// load in flight, which would cut the distance between request and use from a k-tile to a fraction of one.  The
// main loops order these loads themselves: an explicit vmcnt(0) wait and a barrier stand between a request and
// the first read of what it brings, and no other vector-memory access is in flight while one of them is.
__device__ __forceinline__ void load_lds_16(rsrc_t r, char* dst, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_offset(dst)), "v"(voff), "s"(r) : "memory", "m0");
}
__device__ __forceinline__ void load_lds_4(rsrc_t r, char* dst, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
               :: "s"(lds_offset(dst)), "v"(voff), "s"(r) : "memory", "m0");
}
// four wave-loads whose destinations lie 1 KiB apart: the instruction's offset field moves the destination (and
// the source: the lane offsets passed in are 0, 1024, 2048, 3072 bytes short); soff is added to the source only
__device__ __forceinline__ void load_lds_16x4(rsrc_t r, char* dst, uint32_t v0, uint32_t v1, uint32_t v2, uint32_t v3,
                                              uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
               "buffer_load_dwordx4 %1, %5, %6 offen lds\n\t"
               "buffer_load_dwordx4 %2, %5, %6 offen offset:1024 lds\n\t"
               "buffer_load_dwordx4 %3, %5, %6 offen offset:2048 lds\n\t"
               "buffer_load_dwordx4 %4, %5, %6 offen offset:3072 lds"
               :: "s"(lds_offset(dst)), "v"(v0), "v"(v1), "v"(v2), "v"(v3), "s"(r), "s"(soff) : "memory", "m0");
}
// two of the four: loads H*2 and H*2+1 of a group (instruction offsets 2048*H and 2048*H + 1024)
template <int H>
__device__ __forceinline__ void load_lds_16x2(rsrc_t r, char* dst, uint32_t v0, uint32_t v1, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
               "buffer_load_dwordx4 %1, %3, %4 offen offset:%5 lds\n\t"
               "buffer_load_dwordx4 %2, %3, %4 offen offset:%6 lds"
               :: "s"(lds_offset(dst)), "v"(v0), "v"(v1), "s"(r), "s"(soff), "n"(H * 2048), "n"(H * 2048 + 1024) : "memory", "m0");
}

// One 256-row operand tile of 64 k (32 KiB) is filled by 32 wave-loads of 1 KiB; wave w of NW issues
// wave-loads w*LPW .. w*LPW+LPW-1.
// A k-tile that lies inside K whole is requested with as few instructions as the hardware allows, because every
// one of them takes an issue slot from the MFMAs: the lane offsets are loop constants, the k advance rides in the
// scalar offset, and the destinations of four consecutive wave-loads differ only in the instruction's offset
// field (which moves the source too, so it is taken out of the lane offset beforehand); the last, partial k-tile
// and operands with rows shorter than 256 elements take the general form with its per-lane checks.
constexpr int BK = 64;
template <bool KSLOW, int NW> struct TileLoad {
  static constexpr int LPW = 32 / NW;
  uint32_t offm[LPW];  // byte offset of the lane's chunk at k-tile 0 minus 1024 * (i % 4), or kOob if its row is out of range
  uint32_t kstep;      // byte advance per k-tile
  int kfirst;          // k of wave-load 0's chunk (k-contiguous: first k of the chunk; k-slow: the k-row)
  bool plain;          // no offset above goes negative

  // the descriptor's base is the block's first row (k-contiguous: base + row0*ld; k-slow: base + row0)
  __device__ __forceinline__ void init(size_t ld, int rows_left, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      const int li = wave * LPW + i;
      const uint32_t imm = (uint32_t)(i & 3) * 1024u;
      if (!KSLOW) {
        const int row = li * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        offm[i] = row < rows_left ? (uint32_t)(((size_t)row * ld + chunk * 8) * 2) - imm : kOob;
      } else {
        const int k = li * 2 + (lane >> 5);
        const int chunk = (lane & 31) ^ (4 * (k & 3)) ^ (2 * ((k >> 3) & 1));
        offm[i] = chunk * 8 < rows_left ? (uint32_t)(((size_t)k * ld + chunk * 8) * 2) - imm : kOob;
      }
    }
    kstep = KSLOW ? (uint32_t)(BK * ld * 2) : (uint32_t)(BK * 2);
    kfirst = KSLOW ? wave * LPW * 2 + (lane >> 5) : 0;
    plain = ld >= 256;   // row (or k-row) i of a wave-load starts at least 1024 * (i % 4) bytes into the block
  }
  // k of the lane's data in wave-load i: k-contiguous -> depends on the row's swizzle, recomputed here
  __device__ __forceinline__ int kpos(int i, int wave, int lane) const {
    if (KSLOW) return kfirst + 2 * i;
    const int row = (wave * LPW + i) * 8 + (lane >> 3);
    return ((lane & 7) ^ ((row >> 1) & 7)) * 8;
  }
  // The same request in two instalments (four loads per wave only): H = 0 issues loads 0 and 1, H = 1 loads 2 and 3;
  // where the lean form does not apply, H = 0 issues everything and H = 1 nothing.
  template <int H> __device__ __forceinline__ void issue_half(rsrc_t r, char* tile, int wave, int lane, int kt, int K) {
    static_assert(LPW == 4, "one group of four loads per wave");
    if (plain && (kt + 1) * BK <= K)
      load_lds_16x2<H>(r, tile + wave * LPW * 1024, offm[2 * H], offm[2 * H + 1], (uint32_t)kt * kstep);
    else if (H == 0)
      issue(r, tile, wave, lane, kt, K);
  }
  // k-tiles past the end of K come back as zeros (every lane out of range)
  __device__ __forceinline__ void issue(rsrc_t r, char* tile, int wave, int lane, int kt, int K) {
    if (plain && (kt + 1) * BK <= K) {
      const uint32_t koff = (uint32_t)kt * kstep;
#pragma unroll
      for (int i = 0; i < LPW; i += 4)
        load_lds_16x4(r, tile + (wave * LPW + i) * 1024, offm[i], offm[i + 1], offm[i + 2], offm[i + 3], koff);
    } else {
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const bool ok = offm[i] != kOob && kt * BK + kpos(i, wave, lane) < K;
        load_lds_16(r, tile + (wave * LPW + i) * 1024, ok ? offm[i] + (uint32_t)(i & 3) * 1024u + (uint32_t)kt * kstep : kOob);
      }
    }
  }
};

// MFMA operand fragment (row = tile row of this lane, 8 k of k16 step kk) from either layout
template <bool KSLOW>
__device__ __forceinline__ bf16x8_t read_frag(const char* tile, int row_base, int kk, int lane) {
  if (!KSLOW) {
    const int row = row_base + (lane & 31);
    const int chunk = (kk * 2 + (lane >> 5)) ^ ((row >> 1) & 7);
    return *reinterpret_cast<const bf16x8_t*>(tile + row * 128 + chunk * 16);
  } else {
    const int r = lane & 15, G = lane >> 4;
    const int n0 = row_base + 16 * (G & 1) + 4 * (r & 3);
    const int k = kk * 16 + 8 * (G >> 1) + (r >> 2);  // (k & 3) == r >> 2 and (k >> 3) & 1 == G >> 1 for both halves
    const int slot = (n0 >> 3) ^ (4 * (r >> 2)) ^ (2 * (G >> 1));
    const char* p = tile + k * 512 + slot * 16 + (n0 & 7) * 2;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p + 4 * 512));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;
    s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return *reinterpret_cast<bf16x8_t*>(&v);
  }
}

// MFMA operand fragment of v_mfma_f32_16x16x32_bf16 from either layout: lane (lane & 15) is the tile row
// (column of C for the B operand) inside the 16-row block starting at row_base, lane >> 4 selects which 8 of
// the 32 k of step ks (0, 1) the lane carries.
template <bool KSLOW>
__device__ __forceinline__ bf16x8_t read_frag16(const char* tile, int row_base, int ks, int lane) {
  if (!KSLOW) {
    const int row = row_base + (lane & 15);
    const int chunk = (ks * 4 + (lane >> 4)) ^ ((row >> 1) & 7);
    return *reinterpret_cast<const bf16x8_t*>(tile + row * 128 + chunk * 16);
  } else {
    const int r = lane & 15, G = lane >> 4;
    const int n0 = row_base + 4 * (r & 3);
    const int k = ks * 32 + 8 * G + (r >> 2);  // (k & 3) == r >> 2 and (k >> 3) & 1 == G & 1 for both halves
    const int slot = (n0 >> 3) ^ (4 * (r >> 2)) ^ (2 * (G & 1));
    const char* p = tile + k * 512 + slot * 16 + (n0 & 7) * 2;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p + 4 * 512));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;
    s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return *reinterpret_cast<bf16x8_t*>(&v);
  }
}

// s_waitcnt vmcnt(0) only (gfx9 encoding: lgkmcnt and expcnt fields left at their maxima)
__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0f70); }

// Operands of one GEMM call as the kernels see them.  N is the number of columns this launch covers;
// ldb / ldc are the row lengths of the full B (k-slow form) and C, so that a launch may cover a column
// range of a larger problem.  a_end / b_end: one past the last byte of the operands (descriptor bounds).
struct GemmArgs {
  const bf16_t* A;
  const bf16_t* B;
  const bf16_t* bias;
  const char* a_end;
  const char* b_end;
  int M, N, K;
  size_t lda, ldb, ldc;
};

constexpr int kBM = 256, kBN = 256;
constexpr int kTileBytes = 256 * BK * 2, kStageBytes = 2 * kTileBytes;

// L2 prefetch of operand panels.  In the data-parallel form the 32 workgroups that an XCD runs at a time cover 8 row
// tiles x 4 column tiles and walk k together, so every line of an A panel is wanted by 4 of them and every line of a
// B panel by 8, within a fraction of a k-tile.  Panels that the launch streams once (the weights, in forward and data
// gradient; the activations of a weight gradient) come from HBM, and a request that misses L2 takes longer than the
// one k-tile by which the main loop requests ahead.  So with its request for k-tile kt each workgroup also touches
// (4 bytes per 128-byte line, into a scratch corner of LDS) its share of the panels' lines of k-tile kt + kTouchAhead:
// sharer c of 4 takes a quarter of the A lines, sharer q of 8 an eighth of the B lines; wave 0 touches A, wave 1 B.
// The demand requests of the next round then hit in L2 (measured at the 1T-shaped layer's shapes: forward and data
// gradient GEMMs 7 % faster on average, 10-12 % where k = 25600).  `share` = q | c << 8, or -1 for no touching.
#ifndef PTDP_GEMM_TOUCH_AHEAD
#define PTDP_GEMM_TOUCH_AHEAD 1
#endif
constexpr int kTouchAhead = PTDP_GEMM_TOUCH_AHEAD;   // 0: off
constexpr int kTouchLdsBytes = 2048;                 // 256 bytes per wave, above the two stages
template <bool TA, bool TB> struct PanelTouch {
  uint32_t off, step;
  bool on, is_a;
  __device__ __forceinline__ void init(const GemmArgs& g, int m0, int n0, int share, int wave, int lane) {
    on = kTouchAhead > 0 && !TA && share >= 0 && wave < 2;   // weight gradients (both operands k-slow, 32 k-tiles per tile): 1.5 % slower with it
    is_a = wave == 0;
    off = kOob;
    step = 0;
    if (!on) return;
    const int q = share & 0xff, c = (share >> 8) & 3;
    if (is_a) {
      if (!TA) {            // k-contiguous: one line per row and k-tile; 64 rows
        const int row = c * 64 + lane;
        off = row < g.M - m0 ? (uint32_t)((size_t)row * g.lda * 2) : kOob;
        step = BK * 2;
      } else {              // k-slow: four lines per k-row; 16 k-rows
        const int kr = c * 16 + (lane >> 2), l = lane & 3;
        off = l * 64 < g.M - m0 ? (uint32_t)(((size_t)kr * g.lda + l * 64) * 2) : kOob;
        step = (uint32_t)(BK * g.lda * 2);
      }
    } else if (lane < 32) {
      if (!TB) {            // 32 rows
        const int row = q * 32 + lane;
        off = row < g.N - n0 ? (uint32_t)((size_t)row * g.ldb * 2) : kOob;
        step = BK * 2;
      } else {              // 8 k-rows
        const int kr = q * 8 + (lane >> 2), l = lane & 3;
        off = l * 64 < g.N - n0 ? (uint32_t)(((size_t)kr * g.ldb + l * 64) * 2) : kOob;
        step = (uint32_t)(BK * g.ldb * 2);
      }
    }
  }
  // kt: the k-tile whose demand request is being issued
  __device__ __forceinline__ void issue(rsrc_t ra, rsrc_t rb, char* smem, int wave, int kt, int kend) const {
    if (!on) return;
    const int kt2 = kt + kTouchAhead;
    const bool ok = off != kOob && kt2 * BK < kend;
    load_lds_4(is_a ? ra : rb, smem + 2 * kStageBytes + wave * 256, ok ? off + (uint32_t)kt2 * step : kOob);
  }
};

// acc += A[m0.., k] B[n0.., k] over k-tiles kt0 .. kt1-1.  WGM x WGN waves, each (256/WGM) x (256/WGN);
// two LDS stages.  Fragments are double-buffered in registers: the reads of k16 step kk+1 (or of the
// next tile's step 0, after the barrier) are issued before the MFMAs of step kk.  The barrier that
// ends the reads of tile kt's stage sits before the last step's MFMAs, and the loads of tile kt+2
// into that stage are issued right there (a whole k-tile ahead of their use) with the wave's
// priority raised, so that the requests leave before the other wave's arithmetic; they go out after the
// next tile's first fragment reads (measured: +9..14 % over issuing them at the top of the next iteration).
// Measured on copies of this loop with parts removed (NT, all 256 CUs busy, per k-tile): MFMAs alone 1.28 us
// (the chip's power limit on changing operands; 0.96 us on a lone CU), fragment reads +0.08, the barrier +0.12,
// the loads +0.27 in the compiler's form (most of it the issue slots of their address arithmetic: see TileLoad);
// the loads have always landed when the barrier is reached (dropping the wait changes nothing), so neither more
// stages nor an earlier request shorten a k-tile.
template <bool TA, bool TB, int WGM, int WGN>
__device__ __forceinline__ void gemm_mainloop(f32x16_t (&acc)[kBM / WGM / 32][kBN / WGN / 32], const GemmArgs& g,
                                              int m0, int n0, int kt0, int kt1, char* smem, int share) {
  constexpr int NW = WGM * WGN, WM = kBM / WGM, WN = kBN / WGN, TM = WM / 32, TN = WN / 32, NKK = BK / 16;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave-uniform: LDS bases and M0 values stay in scalar registers
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  // buffer descriptors start at the block's first row so that lane offsets stay small
  const bf16_t* a_base = TA ? g.A + m0 : g.A + (size_t)m0 * g.lda;
  const bf16_t* b_base = TB ? g.B + n0 : g.B + (size_t)n0 * g.ldb;
  const size_t a_left = (size_t)(g.a_end - reinterpret_cast<const char*>(a_base));
  const size_t b_left = (size_t)(g.b_end - reinterpret_cast<const char*>(b_base));
  const rsrc_t ra = make_rsrc(a_base, (uint32_t)(a_left < 0x7fffffffu ? a_left : 0x7fffffffu));
  const rsrc_t rb = make_rsrc(b_base, (uint32_t)(b_left < 0x7fffffffu ? b_left : 0x7fffffffu));
  const int kend = min(g.K, kt1 * BK);  // k-tiles from kt1 on read as zeros

  TileLoad<TA, NW> la;
  TileLoad<TB, NW> lb;
  la.init(g.lda, g.M - m0, wave, lane);
  lb.init(g.ldb, g.N - n0, wave, lane);
  PanelTouch<TA, TB> touch;
  touch.init(g, m0, n0, share, wave, lane);

  __syncthreads();  // LDS may still be read by a slower wave of the previous tile
  la.issue(ra, smem, wave, lane, kt0, kend);
  lb.issue(rb, smem + kTileBytes, wave, lane, kt0, kend);
  wait_vmcnt0();
  __syncthreads();

  bf16x8_t af[2][TM], bfr[2][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) af[0][i] = read_frag<TA>(smem, wm0 + i * 32, 0, lane);
#pragma unroll
  for (int j = 0; j < TN; ++j) bfr[0][j] = read_frag<TB>(smem + kTileBytes, wn0 + j * 32, 0, lane);

  auto request = [&](char* stage, int kt) {
    __builtin_amdgcn_s_setprio(1);
    la.issue(ra, stage, wave, lane, kt, kend);
    lb.issue(rb, stage + kTileBytes, wave, lane, kt, kend);
    touch.issue(ra, rb, smem, wave, kt, kend);
    __builtin_amdgcn_s_setprio(0);
  };
  request(smem + kStageBytes, kt0 + 1);
  for (int kt = kt0; kt < kt1; ++kt) {
    char* cur = smem + ((kt - kt0) & 1) * kStageBytes;
    char* nxt = smem + ((kt - kt0 + 1) & 1) * kStageBytes;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const int c = kk & 1, n = c ^ 1;
      if (kk + 1 < NKK) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[n][i] = read_frag<TA>(cur, wm0 + i * 32, kk + 1, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[n][j] = read_frag<TB>(cur + kTileBytes, wn0 + j * 32, kk + 1, lane);
      } else {
        // every fragment of `cur` is in registers: the next tile may be consumed, `cur` may be refilled
        wait_vmcnt0();
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TM; ++i) af[n][i] = read_frag<TA>(nxt, wm0 + i * 32, 0, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[n][j] = read_frag<TB>(nxt + kTileBytes, wn0 + j * 32, 0, lane);
        // the refill goes out after the next tile's first fragment reads (ahead of them: data gradients 1-2 % slower,
        // the others the same); nothing is requested past the last tile: no load may be in flight when the epilogue
        // reuses LDS
        if (kt + 2 < kt1) request(cur, kt + 2);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c][i], bfr[c][j], acc[i][j], 0, 0, 0);
      // Scheduling hint: spread this step's LDS reads between its MFMAs instead of ahead of them (measured:
      // +2..5 % with two 16-byte reads per two MFMAs when both operands are k-contiguous, +1 % one to one
      // when B needs transposing reads; when both do - the weight gradients, 12 eight-byte reads for 8 MFMAs -
      // three reads after each of the first four MFMAs: +1.5..2 % at the 1T-shaped layer's shapes, +4 % at w_o's;
      // two after each is slower, four the same, six or all twelve up front slower again).
      if (!TA) {
        constexpr int per = TB ? 1 : 2;
#pragma unroll
        for (int q = 0; q < TM * TN / per; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, per, 0);   // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, per, 0);   // LDS read
        }
      } else {
#pragma unroll
        for (int q = 0; q < TM * TN; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);   // LDS reads
        }
      }
    }
  }
}

// Output forms.  32x32 accumulator layout: lane holds column (lane & 31), rows 8*(r/4) + 4*(lane/32) + r%4.
//   Each wave passes its 32-row slabs through its own LDS patch
//     (the operand stages are free by then) and leaves with 16 consecutive lanes covering one 256-byte
//     row segment: 16-byte fp32 or 8-byte bf16 accesses instead of scalar ones.
enum { OUT_BF16 = 0, OUT_F32_STORE = 1, OUT_F32_RMW = 2 };
constexpr int kEpiStride = 72;  // floats per staged row of 64: rows 4 apart land 32 banks apart
constexpr int kEpiStride16 = 68;  // 16x16 blocks: a store covers rows 0, 4, 8, 12 of a block, which land 16 banks apart

template <int OUT, int WGM, int WGN>
__device__ __forceinline__ void gemm_epilogue(const f32x16_t (&acc)[kBM / WGM / 32][kBN / WGN / 32], void* Cv, size_t ldc,
                                              const bf16_t* bias, int M, int N, int m0, int n0, char* smem) {
  constexpr int WM = kBM / WGM, WN = kBN / WGN, TM = WM / 32, TN = WN / 32;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave-uniform: LDS bases and M0 values stay in scalar registers
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  static_assert(WN == 64, "staging patch is 32 rows x 64 columns per wave");
  float* patch = reinterpret_cast<float*>(smem) + wave * (32 * kEpiStride);
  float bv[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn0 + j * 32 + (lane & 31);
    bv[j] = (bias && n < N) ? bf16_to_f32(bias[n]) : 0.f;
  }
  const int c4 = (lane & 15) * 4;            // first of this lane's 4 columns inside the wave's 64
  const int n = n0 + wn0 + c4;
  // Gradient accumulators are touched once per launch: stream them past the caches.  The old values of
  // slab i + 1 are requested before slab i is staged and added, so two slabs of loads are in flight.
  f32x4_t old[2][8];
  auto fetch_old = [&](int i, f32x4_t (&dst)[8]) {
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int m = m0 + wm0 + i * 32 + it * 4 + (lane >> 4);
      if (m < M && n < N)
        dst[it] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(reinterpret_cast<float*>(Cv) + (size_t)m * ldc + n));
    }
  };
  if (OUT == OUT_F32_RMW) fetch_old(0, old[0]);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (OUT == OUT_F32_RMW && i + 1 < TM) fetch_old(i + 1, old[(i + 1) & 1]);
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        patch[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * kEpiStride + j * 32 + (lane & 31)] = acc[i][j][r] + bv[j];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = it * 4 + (lane >> 4);
      const int m = m0 + wm0 + i * 32 + row;
      const float4 v = *reinterpret_cast<const float4*>(patch + row * kEpiStride + c4);
      if (m < M && n < N) {
        if (OUT == OUT_BF16) {
          uint2 o;
          o.x = pack_bf16x2(v.x, v.y);
          o.y = pack_bf16x2(v.z, v.w);
          *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(Cv) + (size_t)m * ldc + n) = o;
        } else if (OUT == OUT_F32_RMW) {
          f32x4_t o = old[i & 1][it];
          o[0] += v.x; o[1] += v.y; o[2] += v.z; o[3] += v.w;
          __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(Cv) + (size_t)m * ldc + n));
        } else {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(Cv) + (size_t)m * ldc + n) = v;
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

template <int TM, int TN> __device__ __forceinline__ void zero_acc(f32x16_t (&acc)[TM][TN]) {
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}

// ---- the same main loop and output stage on v_mfma_f32_16x16x32_bf16 -------------------------------------------
// On operands that change from instruction to instruction the chip sustains about a tenth more with this
// shape than with 32x32x16 (a register-resident loop: 2.08-2.13 against 1.89 PFLOP/s on random operands; both
// reach 2.46 on constant ones): a 16x16 accumulator block is read and written half as often per FLOP.  Measured
// in the kernel: +4..6 % where operand A is k-contiguous (forward, data gradients), -3..6 % for the weight
// gradients at K = 2048, which therefore stay on 32x32x16.
template <bool TA, bool TB, int WGM, int WGN>
__device__ __forceinline__ void gemm_mainloop16(f32x4_t (&acc)[kBM / WGM / 16][kBN / WGN / 16], const GemmArgs& g,
                                              int m0, int n0, int kt0, int kt1, char* smem, int share) {
  constexpr int NW = WGM * WGN, WM = kBM / WGM, WN = kBN / WGN, RB = WM / 16, CB = WN / 16;
  static_assert(RB == 8 && CB == 4, "four phases per k-tile: two k32 steps x two halves of the wave's 8 row blocks");
  constexpr int HB = RB / 2;   // row blocks per phase
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave-uniform: LDS bases and M0 values stay in scalar registers
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  // buffer descriptors start at the block's first row so that lane offsets stay small
  const bf16_t* a_base = TA ? g.A + m0 : g.A + (size_t)m0 * g.lda;
  const bf16_t* b_base = TB ? g.B + n0 : g.B + (size_t)n0 * g.ldb;
  const size_t a_left = (size_t)(g.a_end - reinterpret_cast<const char*>(a_base));
  const size_t b_left = (size_t)(g.b_end - reinterpret_cast<const char*>(b_base));
  const rsrc_t ra = make_rsrc(a_base, (uint32_t)(a_left < 0x7fffffffu ? a_left : 0x7fffffffu));
  const rsrc_t rb = make_rsrc(b_base, (uint32_t)(b_left < 0x7fffffffu ? b_left : 0x7fffffffu));
  const int kend = min(g.K, kt1 * BK);  // k-tiles from kt1 on read as zeros

  TileLoad<TA, NW> la;
  TileLoad<TB, NW> lb;
  la.init(g.lda, g.M - m0, wave, lane);
  lb.init(g.ldb, g.N - n0, wave, lane);
  PanelTouch<TA, TB> touch;
  touch.init(g, m0, n0, share, wave, lane);

  __syncthreads();  // LDS may still be read by a slower wave of the previous tile
  la.issue(ra, smem, wave, lane, kt0, kend);
  lb.issue(rb, smem + kTileBytes, wave, lane, kt0, kend);
  wait_vmcnt0();
  __syncthreads();

  // phase p = 2 * ks + half: the MFMAs of row blocks half*4 .. half*4+3 against all four column blocks at k32 step ks
  bf16x8_t af[2][HB], bfr[2][CB];
#pragma unroll
  for (int i = 0; i < HB; ++i) af[0][i] = read_frag16<TA>(smem, wm0 + i * 16, 0, lane);
#pragma unroll
  for (int j = 0; j < CB; ++j) bfr[0][j] = read_frag16<TB>(smem + kTileBytes, wn0 + j * 16, 0, lane);

  // A stage is refilled in three instalments - operand A (and the touches) right behind the barrier that frees it,
  // the two halves of operand B at the start of the next tile's phases 0 and 1 - so that a wave's eight loads do
  // not queue up behind each other and the seven other waves' (measured against all eight at the barrier: data
  // gradients +1.5..2.5 %, forward +1 %, -1.5 % at K = 3200; bit-equal).
  auto request_a = [&](char* stage, int kt) {
    __builtin_amdgcn_s_setprio(1);
    la.issue(ra, stage, wave, lane, kt, kend);
    touch.issue(ra, rb, smem, wave, kt, kend);
    __builtin_amdgcn_s_setprio(0);
  };
  auto request_b = [&](char* stage, int kt, auto half) {
    __builtin_amdgcn_s_setprio(1);
    lb.template issue_half<decltype(half)::value>(rb, stage + kTileBytes, wave, lane, kt, kend);
    __builtin_amdgcn_s_setprio(0);
  };
  request_a(smem + kStageBytes, kt0 + 1);
  lb.issue(rb, smem + kStageBytes + kTileBytes, wave, lane, kt0 + 1, kend);
  for (int kt = kt0; kt < kt1; ++kt) {
    char* cur = smem + ((kt - kt0) & 1) * kStageBytes;
    char* nxt = smem + ((kt - kt0 + 1) & 1) * kStageBytes;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int ks = p >> 1, half = p & 1;
      if (p == 0 && kt > kt0 && kt + 1 < kt1) request_b(nxt, kt + 1, std::integral_constant<int, 0>{});
      if (p == 1 && kt > kt0 && kt + 1 < kt1) request_b(nxt, kt + 1, std::integral_constant<int, 1>{});
      if (p < 3) {
        const int q = p + 1, qs = q >> 1, qh = q & 1;
#pragma unroll
        for (int i = 0; i < HB; ++i) af[q & 1][i] = read_frag16<TA>(cur, wm0 + (qh * HB + i) * 16, qs, lane);
        if (qh == 0) {
#pragma unroll
          for (int j = 0; j < CB; ++j) bfr[qs & 1][j] = read_frag16<TB>(cur + kTileBytes, wn0 + j * 16, qs, lane);
        }
      } else {
        // every fragment of `cur` is in registers: the next tile may be consumed, `cur` may be refilled
        wait_vmcnt0();
        __syncthreads();
#pragma unroll
        for (int i = 0; i < HB; ++i) af[0][i] = read_frag16<TA>(nxt, wm0 + i * 16, 0, lane);
#pragma unroll
        for (int j = 0; j < CB; ++j) bfr[0][j] = read_frag16<TB>(nxt + kTileBytes, wn0 + j * 16, 0, lane);
        // the refill goes out after the next tile's first fragment reads (ahead of them: data gradients 1-2 % slower,
        // the others the same); nothing is requested past the last tile: no load may be in flight when the epilogue
        // reuses LDS
        if (kt + 2 < kt1) request_a(cur, kt + 2);
      }
#pragma unroll
      for (int i = 0; i < HB; ++i)
#pragma unroll
        for (int j = 0; j < CB; ++j)
          acc[half * HB + i][j] =
              __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[p & 1][i], bfr[ks & 1][j], acc[half * HB + i][j], 0, 0, 0);
      // Scheduling hint: spread this phase's LDS reads (4 to 12, for 16 MFMAs) between its MFMAs instead of ahead
      // of them, one after each (measured against one after every two: +2..3 % forward, +5 % at K = 3200,
      // +1.5..2.5 % data gradients)
      if (!TA) {
#pragma unroll
        for (int q = 0; q < HB * CB; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
        }
      }
    }
  }
}

template <int OUT, int WGM, int WGN>
__device__ __forceinline__ void gemm_epilogue16(const f32x4_t (&acc)[kBM / WGM / 16][kBN / WGN / 16], void* Cv, size_t ldc,
                                              const bf16_t* bias, int M, int N, int m0, int n0, char* smem) {
  constexpr int WM = kBM / WGM, WN = kBN / WGN, NS = WM / 32, CB = WN / 16;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave-uniform: LDS bases and M0 values stay in scalar registers
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  static_assert(WN == 64, "staging patch is 32 rows x 64 columns per wave");
  float* patch = reinterpret_cast<float*>(smem) + wave * (32 * kEpiStride16);
  float bv[CB];
#pragma unroll
  for (int j = 0; j < CB; ++j) {
    const int n = n0 + wn0 + j * 16 + (lane & 15);
    bv[j] = (bias && n < N) ? bf16_to_f32(bias[n]) : 0.f;
  }
  const int c4 = (lane & 15) * 4;            // first of this lane's 4 columns inside the wave's 64
  const int n = n0 + wn0 + c4;
  // Gradient accumulators are touched once per launch: stream them past the caches.  The old values of
  // slab i + 1 are requested before slab i is staged and added, so two slabs of loads are in flight.
  f32x4_t old[2][8];
  auto fetch_old = [&](int i, f32x4_t (&dst)[8]) {
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int m = m0 + wm0 + i * 32 + it * 4 + (lane >> 4);
      if (m < M && n < N)
        dst[it] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(reinterpret_cast<float*>(Cv) + (size_t)m * ldc + n));
    }
  };
  if (OUT == OUT_F32_RMW) fetch_old(0, old[0]);
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    if (OUT == OUT_F32_RMW && i + 1 < NS) fetch_old(i + 1, old[(i + 1) & 1]);
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int j = 0; j < CB; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          patch[(16 * b + 4 * (lane >> 4) + r) * kEpiStride16 + j * 16 + (lane & 15)] = acc[2 * i + b][j][r] + bv[j];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = it * 4 + (lane >> 4);
      const int m = m0 + wm0 + i * 32 + row;
      const float4 v = *reinterpret_cast<const float4*>(patch + row * kEpiStride16 + c4);
      if (m < M && n < N) {
        if (OUT == OUT_BF16) {
          uint2 o;
          o.x = pack_bf16x2(v.x, v.y);
          o.y = pack_bf16x2(v.z, v.w);
          *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(Cv) + (size_t)m * ldc + n) = o;
        } else if (OUT == OUT_F32_RMW) {
          f32x4_t o = old[i & 1][it];
          o[0] += v.x; o[1] += v.y; o[2] += v.z; o[3] += v.w;
          __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(Cv) + (size_t)m * ldc + n));
        } else {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(Cv) + (size_t)m * ldc + n) = v;
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

template <int TM, int TN> __device__ __forceinline__ void zero_acc(f32x4_t (&acc)[TM][TN]) {
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
}

// One 256 x 256 tile over k-tiles kt0 .. kt1-1, written either in the caller's output form (slab == nullptr) or
// as a dense 256 x 256 fp32 slab.  The MFMA shape follows operand A's layout (see above).
template <bool TA, bool TB, int OUT, int WGM, int WGN>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, void* Cv, float* slab, int m0, int n0, int kt0, int kt1, char* smem,
                                          int share) {
  if constexpr (TA) {
    f32x16_t acc[kBM / WGM / 32][kBN / WGN / 32];
    zero_acc(acc);
    if (kt1 > kt0) gemm_mainloop<TA, TB, WGM, WGN>(acc, g, m0, n0, kt0, kt1, smem, share);
    if (slab) gemm_epilogue<OUT_F32_STORE, WGM, WGN>(acc, slab, kBN, nullptr, kBM, kBN, 0, 0, smem);
    else gemm_epilogue<OUT, WGM, WGN>(acc, Cv, g.ldc, g.bias, g.M, g.N, m0, n0, smem);
  } else {
    f32x4_t acc[kBM / WGM / 16][kBN / WGN / 16];
    zero_acc(acc);
    if (kt1 > kt0) gemm_mainloop16<TA, TB, WGM, WGN>(acc, g, m0, n0, kt0, kt1, smem, share);
    if (slab) gemm_epilogue16<OUT_F32_STORE, WGM, WGN>(acc, slab, kBN, nullptr, kBM, kBN, 0, 0, smem);
    else gemm_epilogue16<OUT, WGM, WGN>(acc, Cv, g.ldc, g.bias, g.M, g.N, m0, n0, smem);
  }
}

// One workgroup per output tile ("data-parallel" form); `id` is the workgroup's index inside its problem.
// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Each XCD owns the column
// tiles x, x+8, ... and works through them in groups of up to 8 row tiles, so that the
// workgroups resident on one XCD share 8 A panels and 4 B panels through that L2.
template <bool TA, bool TB, int OUT, int WGM, int WGN>
__device__ __forceinline__ void gemm_dp_tile(const GemmArgs& g, void* Cv, int id, char* smem) {
  const int tiles_m = (g.M + kBM - 1) / kBM, tiles_n = (g.N + kBN - 1) / kBN;
  const int xcd = id & 7, local = id >> 3;
  const int nx = (tiles_n + 7) / 8;                 // column tiles per XCD (some may be past the end)
  const int per_group = 8 * nx;                     // blocks of one full group of 8 row tiles
  const int grp = local / per_group, in_grp = local % per_group;
  const int gm = min(8, tiles_m - grp * 8);         // row tiles in this group
  const int tile_m = grp * 8 + in_grp % gm, tile_n = (in_grp / gm) * 8 + xcd;
  if (tile_n >= tiles_n) return;
  // place among the workgroups that share this tile's panels: row tile within the group of 8, column tile within the round's 4
  const int share = (in_grp % gm) | (((in_grp / gm) & 3) << 8);
  gemm_tile<TA, TB, OUT, WGM, WGN>(g, Cv, nullptr, tile_m * kBM, tile_n * kBN, 0, (g.K + BK - 1) / BK, smem, share);
}
// workgroups of one problem (a multiple of 8, so that a second problem starts on XCD 0 again)
static inline int dp_blocks(const GemmArgs& g) {
  const int tiles_m = (g.M + kBM - 1) / kBM, tiles_n = (g.N + kBN - 1) / kBN;
  return 8 * tiles_m * ((tiles_n + 7) / 8);  // 8 XCD queues of equal length; surplus workgroups exit at once
}

template <bool TA, bool TB, int OUT, int WGM, int WGN>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_bf16_dp_kernel(GemmArgs g, void* Cv) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  gemm_dp_tile<TA, TB, OUT, WGM, WGN>(g, Cv, blockIdx.x, smem);
}

// Up to four independent problems of the same form in one launch: each later problem's tiles fill the CUs that the
// last, partial round of the ones before it would leave idle.  start[j] = first workgroup index of problem j
// (multiples of 8, so that every problem starts on XCD 0), start[n] = grid size.
constexpr int kMaxMulti = 4;
struct MultiArgs {
  GemmArgs g[kMaxMulti];
  void* C[kMaxMulti];
  int start[kMaxMulti + 1];
  int n;
};
template <bool TA, bool TB, int OUT, int WGM, int WGN>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_bf16_dp_multi_kernel(MultiArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int id = (int)blockIdx.x;
  // constant indices only: the arguments stay in scalar registers
  GemmArgs g = a.g[0];
  void* C = a.C[0];
  int first = a.start[0];
#pragma unroll
  for (int q = 1; q < kMaxMulti; ++q)
    if (q < a.n && id >= a.start[q]) {
      g = a.g[q];
      C = a.C[q];
      first = a.start[q];
    }
  gemm_dp_tile<TA, TB, OUT, WGM, WGN>(g, C, id - first, smem);
}

// Remainder form, for the tiles that do not fill a whole round of the machine.  The remaining tiles are cut into
// at most two groups; a group of s tiles gives each tile to g = floor(CUs / s) workgroups, workgroup (tile, part)
// taking k-steps [nk*part/g, nk*(part+1)/g) of its tile.  All workgroups of one part index walk the same k-range
// at the same time, so neighbouring tiles share their operand panels through an XCD's L2 exactly as whole rounds
// do (ranges that start at unrelated k, one per workgroup, share nothing: every panel then streams from memory
// and the kernel runs at the memory system's rate instead of L2's).  With g = 1 a workgroup writes its tile
// in the caller's output form; with g > 1 it stores a dense 256 x 256 fp32 slab (index part*s + tile inside the
// group) and gemm_split_reduce_kernel sums a tile's g slabs in part order: no atomics, no waits between
// workgroups, bit-reproducible.
constexpr size_t kSlabFloats = (size_t)kBM * kBN;
constexpr int kMaxSplitGroups = 2;

struct SplitPlan {
  int dp_cols;                      // column tiles computed in whole rounds, one workgroup per tile
  int n_groups;                     // groups of remainder tiles (0 .. kMaxSplitGroups)
  int tiles[kMaxSplitGroups];       // tiles of each group (remainder tiles are numbered row tile fastest)
  int parts[kMaxSplitGroups];       // workgroups per tile
};
// device view of the groups: first workgroup, first tile and first slab of each
struct SplitGroups {
  int n;
  int tiles[kMaxSplitGroups], parts[kMaxSplitGroups], block0[kMaxSplitGroups], tile0[kMaxSplitGroups], slab0[kMaxSplitGroups];
};
static inline int split_blocks(int tiles, int parts) { return 8 * ((tiles * parts + 7) / 8); }   // 8 XCD queues of equal length

template <bool TA, bool TB, int OUT, int WGM, int WGN>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_bf16_split_kernel(GemmArgs g, void* Cv, float* slabs, SplitGroups sg) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int j = 0;
  if (sg.n > 1 && (int)blockIdx.x >= sg.block0[1]) j = 1;
  const int id = (int)blockIdx.x - sg.block0[j];
  const int s = sg.tiles[j], parts = sg.parts[j], units = s * parts;
  // each XCD takes a contiguous run of units in part-major order: one part index (or two), neighbouring tiles
  const int per_xcd = (units + 7) / 8;
  const int unit = (id & 7) * per_xcd + (id >> 3);
  if ((id >> 3) >= per_xcd || unit >= units) return;
  const int part = unit / s, t = unit % s;
  const int tiles_m = (g.M + kBM - 1) / kBM;
  const int tile = sg.tile0[j] + t;
  const int m0 = (tile % tiles_m) * kBM, n0 = (tile / tiles_m) * kBN;
  const int nk = (g.K + BK - 1) / BK;
  const int kt0 = (int)((long long)nk * part / parts), kt1 = (int)((long long)nk * (part + 1) / parts);
  // an XCD's run of units is a run of neighbouring tiles of one part: with 8 row tiles that is 8 x 4 tiles on the same
  // k range, the sharing pattern of a whole round (other row counts: the touches cover the panels only in part)
  const int share = ((tile % tiles_m) & 7) | (((tile / tiles_m) & 3) << 8);
  gemm_tile<TA, TB, OUT, WGM, WGN>(g, Cv, parts == 1 ? nullptr : slabs + (size_t)(sg.slab0[j] + unit) * kSlabFloats, m0, n0, kt0, kt1,
                                   smem, share);
}

// One workgroup per (tile of a split group, 16-row band): sums the tile's slabs in part order and writes
// C = sum (+ bias) as bf16, or C += sum as fp32.  `first` = number of (tile, band) workgroups of group 0.
template <bool OUT_F32>
__global__ void __launch_bounds__(256)
gemm_split_reduce_kernel(const float* __restrict__ slabs, void* Cv, const bf16_t* __restrict__ bias, int M, int N, size_t ldc,
                         SplitGroups sg, int j0, int first) {
  int j = j0, b = (int)blockIdx.x;
  if (b >= first) { j = j0 + 1; b -= first; }
  const int t = b >> 4, band = b & 15;
  const int s = sg.tiles[j], parts = sg.parts[j];
  const int tiles_m = (M + kBM - 1) / kBM;
  const int tile = sg.tile0[j] + t;
  const int row = band * 16 + (threadIdx.x >> 4), c4 = (threadIdx.x & 15) * 4;   // 16 rows x 64 float4 per pass
  float4 sum[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) sum[q] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int part = 0; part < parts; ++part) {
    const float* slab = slabs + (size_t)(sg.slab0[j] + part * s + t) * kSlabFloats + (size_t)row * kBN + c4;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 v = *reinterpret_cast<const float4*>(slab + q * 64);
      sum[q].x += v.x; sum[q].y += v.y; sum[q].z += v.z; sum[q].w += v.w;
    }
  }
  const int m = (tile % tiles_m) * kBM + row;
  if (m >= M) return;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int n = (tile / tiles_m) * kBN + q * 64 + c4;
    if (n >= N) continue;
    if (OUT_F32) {
      float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(Cv) + (size_t)m * ldc + n);
      const float4 o = *c;
      *c = make_float4(o.x + sum[q].x, o.y + sum[q].y, o.z + sum[q].z, o.w + sum[q].w);
    } else {
      float b4[4] = {0.f, 0.f, 0.f, 0.f};
      if (bias) {
        const uint2 bb = *reinterpret_cast<const uint2*>(bias + n);
        b4[0] = __uint_as_float(bb.x << 16); b4[1] = __uint_as_float(bb.x & 0xffff0000u);
        b4[2] = __uint_as_float(bb.y << 16); b4[3] = __uint_as_float(bb.y & 0xffff0000u);
      }
      uint2 o;
      o.x = pack_bf16x2(sum[q].x + b4[0], sum[q].y + b4[1]);
      o.y = pack_bf16x2(sum[q].z + b4[2], sum[q].w + b4[3]);
      *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(Cv) + (size_t)m * ldc + n) = o;
    }
  }
}

constexpr int kWGM = 2, kWGN = 4, kGemmThreads = kWGM * kWGN * 64, kGemmSmem = 2 * kStageBytes + kTouchLdsBytes;

template <bool TA, bool TB, int OUT>
static int launch_dp(const GemmArgs& g, void* C, hipStream_t st) {
  auto kern = gemm_bf16_dp_kernel<TA, TB, OUT, kWGM, kWGN>;
  static once_flag_t done[kMaxDevices];
  if (set_dynamic_smem(reinterpret_cast<const void*>(kern), kGemmSmem, done) != PTDP_OK) return PTDP_E_HIP;
  hipLaunchKernelGGL(kern, dim3(dp_blocks(g)), dim3(kGemmThreads), kGemmSmem, st, g, C);
  return PTDP_OK;
}

template <bool TA, bool TB, int OUT>
static int launch_split(const GemmArgs& g, void* C, float* slabs, const SplitGroups& sg, int blocks, hipStream_t st) {
  auto kern = gemm_bf16_split_kernel<TA, TB, OUT, kWGM, kWGN>;
  static once_flag_t done[kMaxDevices];
  if (set_dynamic_smem(reinterpret_cast<const void*>(kern), kGemmSmem, done) != PTDP_OK) return PTDP_E_HIP;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kGemmThreads), kGemmSmem, st, g, C, slabs, sg);
  return PTDP_OK;
}

static int compute_units() {
  static std::atomic<int> n[kMaxDevices];
  const int d = device_slot();
  if (d >= 0 && n[d].load(std::memory_order_relaxed) > 0) return n[d].load(std::memory_order_relaxed);
  hipDeviceProp_t prop;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 256;
  const int cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  if (d >= 0) n[d].store(cu, std::memory_order_relaxed);
  return cu;
}

// every split group stores at most one slab per compute unit
size_t gemm_workspace_bytes() { return (size_t)compute_units() * kMaxSplitGroups * kSlabFloats * sizeof(float); }

// How a call is cut: whole rounds of tiles (whole columns of tiles, so that the remainder is fewer tiles than
// compute units), then the remainder in at most two groups (see gemm_bf16_split_kernel).  A first group of
// 2^a tiles is taken while one group over all remaining tiles would leave more than a tenth of the
// compute units idle; the second group takes what is left.  The split is used when a cost model fitted to
// measurements (1.8 us per k-step; 12 us per group for its first loads and last stores; 0.12 us per slab
// for its trip through memory, 0.3 us when the sums are added into an fp32 C; 8 us for the reduce launch) puts it
// below nine tenths of one more round of whole tiles.
SplitPlan gemm_plan(int M, int N, int K, int out_f32, int accumulate, int has_bias, size_t ws_bytes) {
  const int ncu = compute_units();
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN, nk = (K + BK - 1) / BK;
  const long long tiles = (long long)tiles_m * tiles_n;
  SplitPlan P;
  P.dp_cols = tiles_n;
  P.n_groups = 0;
  for (int j = 0; j < kMaxSplitGroups; ++j) P.tiles[j] = P.parts[j] = 0;
  const bool out_ok = (out_f32 && accumulate && !has_bias) || !out_f32;
  if (tiles % ncu == 0 || !out_ok || ws_bytes < gemm_workspace_bytes() || (out_f32 && nk < 64)) return P;
  // whole columns only: the full rounds' tiles, rounded up to a column boundary
  const long long full = (tiles / ncu) * ncu;
  const int dp_cols = (int)((full + tiles_m - 1) / tiles_m);
  int rem = (int)(tiles - (long long)dp_cols * tiles_m);
  if (dp_cols >= tiles_n || rem <= 0 || rem >= ncu) return P;
  int gt[kMaxSplitGroups], gp[kMaxSplitGroups], n = 0;
  while (rem > 0 && n < kMaxSplitGroups) {
    int take = rem;
    if (n + 1 < kMaxSplitGroups && (long long)rem * (ncu / rem) * 10 < (long long)ncu * 9) {
      take = 1;
      while (take * 2 <= rem) take *= 2;
    }
    gt[n] = take;
    gp[n] = ncu / take < nk ? ncu / take : nk;   // never more parts than k-steps
    if (gp[n] < 1) gp[n] = 1;
    rem -= take;
    ++n;
  }
  double t_split = 0.0;
  bool any = false;
  for (int j = 0; j < n; ++j) {
    t_split += 1.8 * ((nk + gp[j] - 1) / gp[j]) + 12.0;
    if (gp[j] > 1) {
      t_split += (out_f32 ? 0.3 : 0.12) * gt[j] * gp[j];
      any = true;
    }
  }
  if (any) t_split += 8.0;
  if (!any || t_split >= 0.9 * 1.8 * nk) return P;
  P.dp_cols = dp_cols;
  P.n_groups = n;
  for (int j = 0; j < n; ++j) {
    P.tiles[j] = gt[j];
    P.parts[j] = gp[j];
  }
  return P;
}

void gemm_plan_query(int M, int N, int K, int out_f32, int accumulate, int has_bias, size_t ws_bytes, int* dp_cols,
                     int* n_groups, int* tiles, int* parts) {
  const SplitPlan P = gemm_plan(M, N, K, out_f32, accumulate, has_bias, ws_bytes);
  *dp_cols = P.dp_cols;
  *n_groups = P.n_groups;
  for (int j = 0; j < kMaxSplitGroups; ++j) {
    tiles[j] = P.tiles[j];
    parts[j] = P.parts[j];
  }
}

template <bool TA, bool TB>
static int launch_bf16_mode(const void* A, const void* B, void* C, const void* bias, int M, int N, int K, int out_f32,
                            int accumulate, void* ws, size_t ws_bytes, hipStream_t st) {
  // the kernel addresses each operand through a 31-bit byte offset from the block's first row
  if ((size_t)M * K * 2 >= 0x7fffffffull || (size_t)N * K * 2 >= 0x7fffffffull) return PTDP_E_UNSUPPORTED;
  GemmArgs g;
  g.A = (const bf16_t*)A;
  g.B = (const bf16_t*)B;
  g.bias = (const bf16_t*)bias;
  g.a_end = (const char*)A + (size_t)M * K * 2;
  g.b_end = (const char*)B + (size_t)N * K * 2;
  g.M = M; g.N = N; g.K = K;
  g.lda = TA ? (size_t)M : (size_t)K;
  g.ldb = TB ? (size_t)N : (size_t)K;
  g.ldc = (size_t)N;

  const SplitPlan P = gemm_plan(M, N, K, out_f32, accumulate, bias != nullptr, ws != nullptr ? ws_bytes : 0);
  const int ncu = compute_units();
  const int tiles_m = (M + kBM - 1) / kBM, tiles_n = (N + kBN - 1) / kBN;
  const int n_dp = P.dp_cols < tiles_n ? P.dp_cols * kBN : N;
  if (n_dp > 0) {
    GemmArgs d = g;
    d.N = n_dp;
    int rc;
    if (!out_f32) rc = launch_dp<TA, TB, OUT_BF16>(d, C, st);
    else if (accumulate) rc = launch_dp<TA, TB, OUT_F32_RMW>(d, C, st);
    else rc = launch_dp<TA, TB, OUT_F32_STORE>(d, C, st);
    if (rc != PTDP_OK) return rc;
  }
  if (n_dp < N) {
    // the remainder as a problem of its own: columns n_dp .. N-1
    GemmArgs r = g;
    r.N = N - n_dp;
    r.B = TB ? g.B + n_dp : g.B + (size_t)n_dp * K;
    r.bias = bias ? (const bf16_t*)bias + n_dp : nullptr;
    void* Cr = out_f32 ? (void*)((float*)C + n_dp) : (void*)((bf16_t*)C + n_dp);
    SplitGroups sg;
    sg.n = P.n_groups;
    int blocks = 0, tile0 = 0, slab0 = 0;
    for (int j = 0; j < kMaxSplitGroups; ++j) {
      sg.tiles[j] = j < P.n_groups ? P.tiles[j] : 0;
      sg.parts[j] = j < P.n_groups ? P.parts[j] : 1;
      sg.block0[j] = blocks;
      sg.tile0[j] = tile0;
      sg.slab0[j] = slab0;
      if (j < P.n_groups) {
        if (P.tiles[j] * P.parts[j] > ncu) return PTDP_E_STATE;   // a group never needs more than one slab per compute unit
        blocks += split_blocks(P.tiles[j], P.parts[j]);
        tile0 += P.tiles[j];
        if (P.parts[j] > 1) slab0 += P.tiles[j] * P.parts[j];
      }
    }
    if (tile0 != tiles_m * ((r.N + kBN - 1) / kBN)) return PTDP_E_STATE;   // the groups cover the remainder exactly
    int rc;
    if (!out_f32) rc = launch_split<TA, TB, OUT_BF16>(r, Cr, (float*)ws, sg, blocks, st);
    else if (accumulate) rc = launch_split<TA, TB, OUT_F32_RMW>(r, Cr, (float*)ws, sg, blocks, st);
    else rc = launch_split<TA, TB, OUT_F32_STORE>(r, Cr, (float*)ws, sg, blocks, st);
    if (rc != PTDP_OK) return rc;
    // one reduce launch over the groups that were split (they are adjacent: a group with one part comes last, if at all)
    int j0 = -1, first = 0, total = 0;
    for (int j = 0; j < P.n_groups; ++j) {
      if (P.parts[j] <= 1) continue;
      if (j0 < 0) { j0 = j; first = P.tiles[j] * 16; }
      else if (j != j0 + 1) return PTDP_E_STATE;
      total += P.tiles[j] * 16;
    }
    if (j0 >= 0) {
      if (out_f32)
        hipLaunchKernelGGL(gemm_split_reduce_kernel<true>, dim3(total), dim3(256), 0, st, (const float*)ws, Cr,
                           (const bf16_t*)nullptr, M, r.N, (size_t)N, sg, j0, first);
      else
        hipLaunchKernelGGL(gemm_split_reduce_kernel<false>, dim3(total), dim3(256), 0, st, (const float*)ws, Cr, r.bias, M, r.N,
                           (size_t)N, sg, j0, first);
    }
  }
  return PTDP_OK;
}

static GemmArgs tn_args(const void* A, const void* B, int M, int N, int K) {
  GemmArgs g;
  g.A = (const bf16_t*)A;
  g.B = (const bf16_t*)B;
  g.bias = nullptr;
  g.a_end = (const char*)A + (size_t)M * K * 2;
  g.b_end = (const char*)B + (size_t)N * K * 2;
  g.M = M; g.N = N; g.K = K;
  g.lda = (size_t)M;
  g.ldb = (size_t)N;
  g.ldc = (size_t)N;
  return g;
}

// C_j[M_j,N_j] += A_j^T B_j for j < n <= 4 (fp32 C, both operands [K, .]), sharing K: weight gradients whose inputs
// are all at hand.  In bf16 they run as one launch.
int launch_gemm_tn_multi(int dtype, int n, const void* const* A, const void* const* B, float* const* C, const int* M,
                         const int* N, int K, hipStream_t st) {
  if (n <= 0 || n > kMaxMulti) return PTDP_E_INVALID_ARG;
  bool one_by_one = dtype == PTDP_F32;
  double flops = 0.0;
  for (int j = 0; j < n; ++j) {
    if (M[j] == 0 || N[j] == 0 || (size_t)M[j] * K * 2 >= 0x7fffffffull || (size_t)N[j] * K * 2 >= 0x7fffffffull) one_by_one = true;
    flops += 2.0 * K * (double)M[j] * N[j];
  }
  if (one_by_one) {
    for (int j = 0; j < n; ++j) {
      const int rc = launch_gemm(dtype, PTDP_GEMM_TN, A[j], B[j], C[j], nullptr, M[j], N[j], K, 1, 1, nullptr, 0, st);
      if (rc != PTDP_OK) return rc;
    }
    return PTDP_OK;
  }
  Launch L(PTDP_K_GEMM_TN, flops, st);
  MultiArgs a;
  a.n = n;
  int at = 0;
  for (int j = 0; j < kMaxMulti; ++j) {
    const int q = j < n ? j : 0;   // unused slots repeat problem 0 (never selected)
    a.g[j] = tn_args(A[q], B[q], M[q], N[q], K);
    a.C[j] = C[q];
    a.start[j] = at;
    if (j < n) at += dp_blocks(a.g[j]);
  }
  a.start[kMaxMulti] = at;
  auto kern = gemm_bf16_dp_multi_kernel<true, true, OUT_F32_RMW, kWGM, kWGN>;
  static once_flag_t done[kMaxDevices];
  if (set_dynamic_smem(reinterpret_cast<const void*>(kern), kGemmSmem, done) != PTDP_OK) return PTDP_E_HIP;
  hipLaunchKernelGGL(kern, dim3(at), dim3(kGemmThreads), kGemmSmem, st, a);
  return L.status();
}

int launch_gemm(int dtype, int mode, const void* A, const void* B, void* C, const void* bias, int M, int N, int K,
                int out_f32, int accumulate, void* ws, size_t ws_bytes, hipStream_t st) {
  if (M == 0 || N == 0) return PTDP_OK;
  const int fam = mode == PTDP_GEMM_NN ? PTDP_K_GEMM_NN : (mode == PTDP_GEMM_NT ? PTDP_K_GEMM_NT : PTDP_K_GEMM_TN);
  Launch L(fam, 2.0 * M * N * K, st);
  if (dtype == PTDP_F32) {
    size_t a_rs = K, a_cs = 1, b_rs = N, b_cs = 1;
    if (mode == PTDP_GEMM_NT) { b_rs = 1; b_cs = K; }
    if (mode == PTDP_GEMM_TN) { a_rs = 1; a_cs = M; }
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, st, (const float*)A,
                       (const float*)B, (float*)C, (const float*)bias, M, N, K, a_rs, a_cs, b_rs, b_cs, accumulate);
    return L.status();
  }
  int rc;
  switch (mode) {
    case PTDP_GEMM_NN: rc = launch_bf16_mode<false, true>(A, B, C, bias, M, N, K, out_f32, accumulate, ws, ws_bytes, st); break;
    case PTDP_GEMM_NT: rc = launch_bf16_mode<false, false>(A, B, C, bias, M, N, K, out_f32, accumulate, ws, ws_bytes, st); break;
    default: rc = launch_bf16_mode<true, true>(A, B, C, bias, M, N, K, out_f32, accumulate, ws, ws_bytes, st); break;
  }
  if (rc != PTDP_OK) return rc;
  return L.status();
}

}  // namespace ptdp
