// GEMMs of the layer (paper appendix: QKV, attention output projection, MLP h->4h/t and 4h/t->h, and
// for each the input-gradient and weight-gradient products of the backward pass).
//
//   mode NN: C[M,N] = A[M,K] B[K,N]          forward      Y  = X W
//   mode NT: C[M,N] = A[M,K] B[N,K]^T        input grad   dX = dY W^T
//   mode TN: C[M,N] = A[K,M]^T B[K,N]        weight grad  dW = X^T dY
//
// bf16 path: v_mfma_f32_32x32x16_bf16 (gfx950), 256 x 256 x 64 block tile, LDS double buffering,
// register-staged global loads.  An operand whose reduction index is the slow memory index (B in NN,
// both in TN) is transposed in registers (8 x 8 blocks of 16-bit values) on its way into LDS, so that
// every MFMA fragment is one 16-byte LDS read of eight consecutive k.
// fp32 path: a plain LDS-tiled FMA kernel (correctness configuration only).
#include "common.h"

namespace ptdp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

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
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------------
constexpr int BK = 64;  // k per LDS stage: one 128-byte LDS row of eight 16-byte chunks

// LDS tile: R rows (m or n index) x 64 k, 128 bytes per row; chunk c of row r sits at chunk
// c ^ swz(r).  swz mixes bits 0-2 and 3-5 of the row so that (a) the 8 rows read by 8 neighbouring
// lanes of a fragment load and (b) the 8 rows r0+j of neighbouring 8x8 transposed blocks fall into
// different bank groups.
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ swz(row)) << 4); }

// Stages one R x 64 operand tile through registers.
//   TRANS = false: memory is [row][k] (k contiguous):  src + row*ld + k
//   TRANS = true : memory is [k][row] (row contiguous): src + k*ld + row
template <int R, bool TRANS> struct Stage {
  static constexpr int NV = TRANS ? 8 * ((R + 255) / 256) : R / 32;
  uint4 v[NV];

  __device__ __forceinline__ void load(const bf16_t* __restrict__ src, size_t ld, int row0, int row_end, int k0,
                                       int K) {
    const int t = threadIdx.x;
    if (!TRANS) {
      const int chunk = t & 7;
      const int k = k0 + chunk * 8;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int row = row0 + (t >> 3) + i * 32;
        v[i] = (row < row_end && k < K) ? *reinterpret_cast<const uint4*>(src + (size_t)row * ld + k)
                                        : make_uint4(0, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int blk = 0; blk < NV / 8; ++blk) {
        const int id = t + blk * 256;  // 8x8 block id: R/8 row groups x 8 k groups
        const int rg = id % (R / 8), kg = id / (R / 8);
        const int row = row0 + rg * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int k = k0 + kg * 8 + j;
          v[blk * 8 + j] = (id < R && row < row_end && k < K)
                               ? *reinterpret_cast<const uint4*>(src + (size_t)k * ld + row)
                               : make_uint4(0, 0, 0, 0);
        }
      }
    }
  }

  __device__ __forceinline__ void store(char* lds) const {
    const int t = threadIdx.x;
    if (!TRANS) {
      const int chunk = t & 7;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int row = (t >> 3) + i * 32;
        *reinterpret_cast<uint4*>(lds + lds_off(row, chunk)) = v[i];
      }
    } else {
#pragma unroll
      for (int blk = 0; blk < NV / 8; ++blk) {
        const int id = t + blk * 256;
        if (id >= R) continue;
        const int rg = id % (R / 8), kg = id / (R / 8);
        // in[j] holds k = j, rows 0..7 (two per dword); out[r] must hold row r, k = 0..7
        const uint32_t* in = reinterpret_cast<const uint32_t*>(&v[blk * 8]);  // in[j*4 + d]
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          uint32_t o[4];
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const uint32_t x = in[(2 * d) * 4 + (r >> 1)], y = in[(2 * d + 1) * 4 + (r >> 1)];
            o[d] = (r & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
          }
          *reinterpret_cast<uint4*>(lds + lds_off(rg * 8 + r, kg)) = make_uint4(o[0], o[1], o[2], o[3]);
        }
      }
    }
  }
};

// BM x BN block tile, waves arranged (BM/WM) x (BN/WN), each wave WM x WN = (WM/32) x (WN/32) MFMA tiles.
template <int BM, int BN, int WM, int WN, bool TA, bool TB, bool OUT_F32>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
gemm_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, void* Cv, const bf16_t* __restrict__ bias,
                 int M, int N, int K, int accumulate) {
  static_assert((BM / WM) * (BN / WN) == 4, "loaders assume 256 threads");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int TM = WM / 32, TN = WN / 32;

  // tile order: consecutive blocks walk M first so that blocks running together share the B panel
  const int tiles_m = (M + BM - 1) / BM;
  const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const size_t lda = TA ? (size_t)M : (size_t)K;
  const size_t ldb = TB ? (size_t)N : (size_t)K;   // TB: B is [K,N]; else B is [N,K]

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm0 = (wave / (BN / WN)) * WM, wn0 = (wave % (BN / WN)) * WN;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  Stage<BM, TA> sa;
  Stage<BN, TB> sb;
  const int nk = (K + BK - 1) / BK;
  sa.load(A, lda, m0, M, 0, K);
  sb.load(B, ldb, n0, N, 0, K);
  sa.store(smem);
  sb.store(smem + A_BYTES);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * STAGE_BYTES;
    char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
    if (kt + 1 < nk) {
      sa.load(A, lda, m0, M, (kt + 1) * BK, K);
      sb.load(B, ldb, n0, N, (kt + 1) * BK, K);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8_t af[TM], bfr[TN];
      const int chunk = kk * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8_t*>(cur + lds_off(wm0 + i * 32 + (lane & 31), chunk));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8_t*>(cur + A_BYTES + lds_off(wn0 + j * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      sa.store(nxt);
      sb.store(nxt + A_BYTES);
    }
    __syncthreads();
  }

  // epilogue.  32x32 accumulator layout: lane holds column (lane & 31), rows 8*(r/4) + 4*(lane/32) + r%4.
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn0 + j * 32 + (lane & 31);
    if (n >= N) continue;
    const float bv = bias ? bf16_to_f32(bias[n]) : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm0 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m >= M) continue;
        const float val = acc[i][j][r] + bv;
        if (OUT_F32) {
          float* c = reinterpret_cast<float*>(Cv) + (size_t)m * N + n;
          *c = accumulate ? *c + val : val;
        } else {
          reinterpret_cast<bf16_t*>(Cv)[(size_t)m * N + n] = f32_to_bf16(val);
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, bool TA, bool TB, bool OUT_F32>
static int launch_bf16_cfg(const void* A, const void* B, void* C, const void* bias, int M, int N, int K, int accumulate,
                           hipStream_t st) {
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, TA, TB, OUT_F32>;
  constexpr int smem = 2 * (BM + BN) * BK * 2;
  static bool attr_set = false;  // per instantiation; benign race (idempotent call)
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) !=
        hipSuccess)
      return PTDP_E_HIP;
    attr_set = true;
  }
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(256), smem, st, (const bf16_t*)A, (const bf16_t*)B, C,
                     (const bf16_t*)bias, M, N, K, accumulate);
  return PTDP_OK;
}

template <bool TA, bool TB>
static int launch_bf16_mode(const void* A, const void* B, void* C, const void* bias, int M, int N, int K, int out_f32,
                            int accumulate, hipStream_t st) {
  if (out_f32) return launch_bf16_cfg<256, 256, 128, 128, TA, TB, true>(A, B, C, bias, M, N, K, accumulate, st);
  return launch_bf16_cfg<256, 256, 128, 128, TA, TB, false>(A, B, C, bias, M, N, K, accumulate, st);
}

int launch_gemm(int dtype, int mode, const void* A, const void* B, void* C, const void* bias, int M, int N, int K,
                int out_f32, int accumulate, hipStream_t st) {
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
    case PTDP_GEMM_NN: rc = launch_bf16_mode<false, true>(A, B, C, bias, M, N, K, out_f32, accumulate, st); break;
    case PTDP_GEMM_NT: rc = launch_bf16_mode<false, false>(A, B, C, bias, M, N, K, out_f32, accumulate, st); break;
    default: rc = launch_bf16_mode<true, true>(A, B, C, bias, M, N, K, out_f32, accumulate, st); break;
  }
  if (rc != PTDP_OK) return rc;
  return L.status();
}

}  // namespace ptdp
