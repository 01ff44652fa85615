// Internal helpers shared by the HIP translation units of libptdp (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "ptdp.h"

namespace ptdp {

typedef uint16_t bf16_t;  // raw bfloat16 bits

// ---- storage <-> fp32 -------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// fp32 -> bf16, round to nearest even: the hardware's packed conversion (v_cvt_pk_bf16_f32)
typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, hw_bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

// A 16-byte vector of storage elements: 4 floats or 8 bf16.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ __forceinline__ void load(const float* p) { raw = *reinterpret_cast<const float4*>(p); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<float4*>(p) = raw; }
  __device__ __forceinline__ void unpack(float* f) const { f[0] = raw.x; f[1] = raw.y; f[2] = raw.z; f[3] = raw.w; }
  __device__ __forceinline__ void pack(const float* f) { raw = make_float4(f[0], f[1], f[2], f[3]); }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_t* p) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void store(bf16_t* p) const { *reinterpret_cast<uint4*>(p) = raw; }
  __device__ __forceinline__ void unpack(float* f) const {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ __forceinline__ void pack(const float* f) {
    raw.x = pack_bf16x2(f[0], f[1]);
    raw.y = pack_bf16x2(f[2], f[3]);
    raw.z = pack_bf16x2(f[4], f[5]);
    raw.w = pack_bf16x2(f[6], f[7]);
  }
};

// ---- reductions -------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
// Sum over the whole block (blockDim.x a multiple of 64, at most 1024); every thread gets the result.
// smem: at least 16 floats; safe to call repeatedly (leading barrier).
__device__ __forceinline__ float block_sum(float v, float* smem) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) smem[wave] = v;
  __syncthreads();
  float r = 0.f;
  for (int i = 0; i < nw; ++i) r += smem[i];
  return r;
}

// ---- dropout stream (integers only; see ptdp_hash in ptdp.h) -------------------
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
inline uint64_t dropout_key(uint64_t seed, uint32_t layer, uint32_t site, uint64_t microbatch) {
  uint64_t k = mix64(seed);
  k = mix64(k + kGolden * (uint64_t)(2ull * layer + site + 1ull));
  k = mix64(k + kGolden * (microbatch + 1ull));
  return k;
}
inline uint32_t dropout_threshold(float p) { return (uint32_t)((double)p * 65536.0 + 0.5); }
// keep flags of the N elements starting at flat index idx (idx % N == 0, N in {4, 8}).
template <int N> __device__ __forceinline__ void keep_flags(uint64_t key, uint64_t idx, uint32_t thr, bool* keep) {
#pragma unroll
  for (int w = 0; w < N / 4; ++w) {
    const uint64_t r = mix64(key + kGolden * ((idx >> 2) + w));
#pragma unroll
    for (int j = 0; j < 4; ++j) keep[4 * w + j] = (uint32_t)((r >> (16 * j)) & 0xffffu) >= thr;
  }
}

// ---- launch bookkeeping -------------------------------------------------------
// Brackets a launch with an event pair when profiling is on; records launch errors.
struct Launch {
  Launch(int family, double work, hipStream_t stream);
  ~Launch();
  int status();  // call after the launch statement(s): PTDP_OK or PTDP_E_HIP
  hipStream_t stream_;
  int slot_;     // index of the open profiling record, or -1
  int status_;
  bool closed_;
};

// Per-device one-time state (function attributes, device properties): each device of the process keeps its own.
constexpr int kMaxDevices = 64;
inline int device_slot() {
  int d = 0;
  return (hipGetDevice(&d) == hipSuccess && d >= 0 && d < kMaxDevices) ? d : -1;
}
// Raises a kernel's dynamic shared memory limit once per device; `done` is that kernel's flag array.  Threads
// that race here both make the (idempotent) call; the flags are atomics so that the race is a defined one.
typedef std::atomic<bool> once_flag_t;
inline int set_dynamic_smem(const void* kern, int bytes, once_flag_t (&done)[kMaxDevices]) {
  const int d = device_slot();
  if (d >= 0 && done[d].load(std::memory_order_acquire)) return PTDP_OK;
  if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return PTDP_E_HIP;
  if (d >= 0) done[d].store(true, std::memory_order_release);
  return PTDP_OK;
}

// Second stages of column sums that a caller wants run together: a backward kernel given a ColsumBatch only records
// where its partial sums lie and what they are to be added to; launch_colsum_batch then finishes all of them in one
// launch (each recorded job needs scratch of its own until then).
struct ColsumJob {
  const float* part;
  int nparts, stride, width;
  float* out0;
  float* out1;   // second output (the partials' upper half) or null
};
constexpr int kMaxColsumJobs = 8;
struct ColsumBatch {
  ColsumJob job[kMaxColsumJobs];
  int n = 0;
};
int launch_colsum_batch(const ColsumBatch& batch, hipStream_t st);

// kernels (defined in the .hip files; all arguments validated by the callers in api.hip)
int launch_layernorm_fwd(int dtype, const void* x, const void* gain, const void* bias, void* u, float* mu,
                         float* rstd, void* x_copy, int rows, int width, float eps, hipStream_t st);
int launch_layernorm_bwd(int dtype, const void* du, const void* x, const void* gain, const float* mu,
                         const float* rstd, const void* resid, void* dx, float* dgain, float* dbias,
                         void* scratch, int rows, int width, hipStream_t st, ColsumBatch* defer = nullptr);
int launch_bias_gelu_fwd(int dtype, int mode, const void* z, const void* bias, void* g, int rows, int width,
                         hipStream_t st);
int launch_bias_gelu_bwd(int dtype, int mode, const void* dg, const void* z, const void* bias, void* dz,
                         float* dbias, void* scratch, int rows, int width, hipStream_t st, ColsumBatch* defer = nullptr);
int launch_bda_fwd(int dtype, const void* in, const void* bias, const void* resid, void* out, int rows,
                   int width, float p, uint64_t key, hipStream_t st);
int launch_bda_bwd(int dtype, const void* dout, void* din, float* dbias, void* scratch, int rows, int width,
                   float p, uint64_t key, hipStream_t st, ColsumBatch* defer = nullptr);
// same, with the column-sum partials in a static device array of kStaticScratchBytes (allocates nothing)
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
int launch_bda_bwd_static(int dtype, const void* dout, void* din, float* dbias, int rows, int width, float p,
                          uint64_t key, hipStream_t st);
bool profiling_enabled();
int launch_dropout_mask(uint8_t* keep, int64_t n, float p, uint64_t key, hipStream_t st);
size_t colsum_scratch_bytes(int rows, int width);
size_t layernorm_bwd_scratch_bytes(int rows, int width);   // scratch of launch_layernorm_bwd
// out[width] (fp32) += column sums of in[rows, width]
int launch_colsum(int dtype, const void* in, float* out, void* scratch, int rows, int width, hipStream_t st,
                  ColsumBatch* defer = nullptr);
// ws / ws_bytes: optional scratch of gemm_workspace_bytes() for tiles that are split along k (may be null / 0)
size_t gemm_workspace_bytes();
// how a bf16 call is cut (host only): column tiles computed in whole rounds, then up to two groups of remainder
// tiles, group j giving each of its tiles[j] tiles to parts[j] workgroups that split the k range evenly
void gemm_plan_query(int M, int N, int K, int out_f32, int accumulate, int has_bias, size_t ws_bytes, int* dp_cols,
                     int* n_groups, int* tiles, int* parts);
int launch_gemm(int dtype, int mode, const void* A, const void* B, void* C, const void* bias, int M, int N,
                int K, int out_f32, int accumulate, void* ws, size_t ws_bytes, hipStream_t st);
// up to four fp32-accumulating weight gradients C_j += A_j^T B_j with the same K (bf16: one launch)
int launch_gemm_tn_multi(int dtype, int n, const void* const* A, const void* const* B, float* const* C, const int* M,
                         const int* N, int K, hipStream_t st);
// mask: [b, s, s] bytes (nonzero = hidden) or null, used when causal == 0
int launch_attn_fwd(int dtype, const void* qkv, void* ctx, float* lse, int s, int b, int heads, int dh,
                    const uint8_t* mask, int causal, hipStream_t st);
int launch_attn_bwd(int dtype, const void* qkv, const void* ctx, const float* lse, const void* dctx,
                    void* dqkv, float* delta, int s, int b, int heads, int dh, const uint8_t* mask, int causal,
                    hipStream_t st);
bool attn_dh_supported(int dtype, int dh);
// first / last stage extras (lm_stage.hip)
int launch_embed_fwd(int dtype, const int32_t* tokens, const void* e_word, const void* e_pos, void* x, int s, int b,
                     int h, int v0, int vrows, float p, uint64_t key, hipStream_t st);
int launch_embed_bwd(int dtype, const int32_t* tokens, const void* dx, void* dmasked, float* d_e_word, float* d_e_pos,
                     int s, int b, int h, int v0, int vrows, float p, uint64_t key, hipStream_t st);
int launch_xent(int dtype, void* logits, const int32_t* targets, float* token_loss, float* loss, int rows, int vrows,
                int v0, float grad_scale, hipStream_t st);

}  // namespace ptdp
