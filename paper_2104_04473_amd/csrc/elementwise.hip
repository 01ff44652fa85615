// Bandwidth-bound kernels of the layer: LayerNorm, bias+GeLU, bias+dropout+add (paper section 4.2
// names the two fusions; LayerNorm is implied by the 13h term of eq. (2)) and their backward passes.
// All of them move 16 bytes per lane per access, keep fp32 arithmetic, and reduce with wavefront
// shuffles; column sums (bias / LayerNorm parameter gradients) are two-stage and deterministic.
#include "common.h"

namespace ptdp {

static constexpr int kColRows = 32;  // rows per block in the column-sum producers

// The column-sum producers (bias+GeLU backward, bias+dropout+add backward, plain column sums) run 256-thread
// workgroups of 64 column groups (16 bytes each) x 4 row lanes: wave w takes rows r0 + w, r0 + w + 4, ... of
// the block's kColRows rows, a whole 1 KiB run of one row per access, eight rows per thread in flight, and
// width / 512 x rows / 32 workgroups per launch (one thread walking all 32 rows left a 6144-wide bf16 gradient
// with 192 workgroups for 256 CUs).  The four waves' sums meet in LDS and wave 0 adds them in a fixed order.
static constexpr int kColLanes = 4;
static inline dim3 colsum_grid(int nvec, int rows) { return dim3((nvec + 63) / 64, (rows + kColRows - 1) / kColRows); }
template <int N>
__device__ __forceinline__ void colsum_block_store(float (&acc)[N], float* __restrict__ part, int width, int c, bool valid) {
  __shared__ float red[kColLanes - 1][N][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (w > 0) {
#pragma unroll
    for (int j = 0; j < N; ++j) red[w - 1][j][lane] = acc[j];
  }
  __syncthreads();
  if (w == 0 && valid) {
#pragma unroll
    for (int j = 0; j < N; ++j)
      part[(size_t)blockIdx.y * width + (size_t)c * N + j] = (acc[j] + red[0][j][lane]) + (red[1][j][lane] + red[2][j][lane]);
  }
}

// ------------------------------------------------------------------------------------------------
// LayerNorm forward: one block per row, the row lives in registers (VPT 16-byte vectors per thread).
// ------------------------------------------------------------------------------------------------
template <typename T, int VPT>
__global__ void layernorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gain, const T* __restrict__ bias,
                                     T* __restrict__ u, float* __restrict__ mu, float* __restrict__ rstd,
                                     T* __restrict__ x_copy, int width, float eps) {
  constexpr int N = Vec16<T>::N;
  __shared__ float red[16];
  const int nvec = width / N;
  const size_t row = blockIdx.x;
  const T* xr = x + row * width;
  float v[VPT][N];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c = threadIdx.x + i * blockDim.x;
    if (c < nvec) {
      Vec16<T> t;
      t.load(xr + (size_t)c * N);
      if (x_copy) t.store(x_copy + row * width + (size_t)c * N);
      t.unpack(v[i]);
#pragma unroll
      for (int j = 0; j < N; ++j) sum += v[i][j];
    }
  }
  const float mean = block_sum(sum, red) / (float)width;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c = threadIdx.x + i * blockDim.x;
    if (c < nvec) {
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const float d = v[i][j] - mean;
        sq += d * d;
      }
    }
  }
  const float r = rsqrtf(block_sum(sq, red) / (float)width + eps);
  if (threadIdx.x == 0) {
    mu[row] = mean;
    rstd[row] = r;
  }
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c = threadIdx.x + i * blockDim.x;
    if (c < nvec) {
      Vec16<T> g, b, o;
      float gf[N], bf[N], of[N];
      g.load(gain + (size_t)c * N);
      b.load(bias + (size_t)c * N);
      g.unpack(gf);
      b.unpack(bf);
#pragma unroll
      for (int j = 0; j < N; ++j) of[j] = gf[j] * ((v[i][j] - mean) * r) + bf[j];
      o.pack(of);
      o.store(u + row * width + (size_t)c * N);
    }
  }
}

// LayerNorm backward: input gradient and the partial sums of the gain / bias gradients in one pass.
//   xhat = (x-mu)*rstd, dxhat = du*gain, dx = resid + rstd*(dxhat - mean(dxhat) - xhat*mean(dxhat*xhat)),
//   dgain[c] = sum_r du*xhat, dbias[c] = sum_r du.
// A block walks `rpb` consecutive rows; each row of du and x is read once and waits in registers in storage
// form (fp32 copies of both would not fit next to the column accumulators) while the two row means are reduced;
// every lane keeps the running column sums of its own VPT*N columns and stores them once, as row blockIdx.x of
// part[][2*width] (gain part first).  dx may alias du: a lane overwrites only elements it has read itself.
template <typename T, int VPT>
__global__ void __launch_bounds__(512)
layernorm_bwd_kernel(const T* du, const T* __restrict__ x, const T* __restrict__ gain, const float* __restrict__ mu,
                     const float* __restrict__ rstd, const T* resid, T* dx, float* __restrict__ part, int rows, int width,
                     int rpb) {
  constexpr int N = Vec16<T>::N;
  extern __shared__ __attribute__((aligned(16))) char ln_smem[];
  T* gain_s = reinterpret_cast<T*>(ln_smem);   // the gain row, read twice per row of the block
  __shared__ float red[2][16];
  const int nvec = width / N;
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  for (int c = threadIdx.x; c < nvec; c += blockDim.x) {
    Vec16<T> g;
    g.load(gain + (size_t)c * N);
    g.store(gain_s + (size_t)c * N);
  }
  float ag[VPT][N], ab[VPT][N];
#pragma unroll
  for (int i = 0; i < VPT; ++i)
#pragma unroll
    for (int j = 0; j < N; ++j) ag[i][j] = ab[i][j] = 0.f;
  const int r0 = blockIdx.x * rpb, r1 = min(rows, r0 + rpb);
  for (int r = r0; r < r1; ++r) {
    const size_t base = (size_t)r * width;
    const float m = mu[r], rs = rstd[r];
    // the residual gradient is only wanted after the reduction, but requested here: one round trip per row
    Vec16<T> a[VPT], b[VPT], rr[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int c = threadIdx.x + i * blockDim.x;
      if (c < nvec) {
        a[i].load(du + base + (size_t)c * N);
        b[i].load(x + base + (size_t)c * N);
        if (resid) rr[i].load(resid + base + (size_t)c * N);
      }
    }
    __syncthreads();   // gain row visible (first row); `red` of the previous row no longer read
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int c = threadIdx.x + i * blockDim.x;
      if (c < nvec) {
        Vec16<T> g;
        float af[N], xf[N], gf[N];
        g.load(gain_s + (size_t)c * N);
        a[i].unpack(af);
        b[i].unpack(xf);
        g.unpack(gf);
#pragma unroll
        for (int j = 0; j < N; ++j) {
          const float xh = (xf[j] - m) * rs, dxh = af[j] * gf[j];
          s1 += dxh;
          s2 += dxh * xh;
          ag[i][j] += af[j] * xh;
          ab[i][j] += af[j];
        }
      }
    }
    // both row sums through one pair of barriers
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if ((threadIdx.x & 63) == 0) {
      red[0][wave] = s1;
      red[1][wave] = s2;
    }
    __syncthreads();
    float c1 = 0.f, c2 = 0.f;
    for (int w = 0; w < nw; ++w) {
      c1 += red[0][w];
      c2 += red[1][w];
    }
    c1 /= (float)width;
    c2 /= (float)width;
    // the second pass unpacks the stored row again: keeping the first pass's fp32 values alive across the
    // reduction instead would cost two more registers per element and spill
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      asm volatile("" : "+v"(a[i].raw.x), "+v"(a[i].raw.y), "+v"(a[i].raw.z), "+v"(a[i].raw.w));
      asm volatile("" : "+v"(b[i].raw.x), "+v"(b[i].raw.y), "+v"(b[i].raw.z), "+v"(b[i].raw.w));
    }
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int c = threadIdx.x + i * blockDim.x;
      if (c < nvec) {
        Vec16<T> g, o;
        float af[N], xf[N], gf[N], of[N];
        g.load(gain_s + (size_t)c * N);
        a[i].unpack(af);
        b[i].unpack(xf);
        g.unpack(gf);
        if (resid) {
          rr[i].unpack(of);
        } else {
#pragma unroll
          for (int j = 0; j < N; ++j) of[j] = 0.f;
        }
#pragma unroll
        for (int j = 0; j < N; ++j) of[j] += rs * (af[j] * gf[j] - c1 - (xf[j] - m) * rs * c2);
        o.pack(of);
        o.store(dx + base + (size_t)c * N);
      }
    }
  }
  float* prow = part + (size_t)blockIdx.x * 2 * width;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int c = threadIdx.x + i * blockDim.x;
    if (c < nvec) {
#pragma unroll
      for (int j = 0; j < N; ++j) {
        prow[(size_t)c * N + j] = ag[i][j];
        prow[(size_t)width + (size_t)c * N + j] = ab[i][j];
      }
    }
  }
}

// out[c] += sum over parts of part[p][c]  (second stage of every column sum; fixed order).
// A workgroup owns 64 columns; its four waves each add a quarter of the parts (four independent partial
// sums per lane keep loads in flight), and wave 0 adds the four quarter sums in order.
__device__ __forceinline__ void colsum_finish_block(const float* __restrict__ part, int nparts, int stride, float* out0, float* out1,
                                                    int width, int blk) {
  __shared__ float red[2][4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int c = blk * 64 + lane;
  const int per = (nparts + 3) / 4, p0 = q * per, p1 = min(nparts, p0 + per);
  float a[4] = {0.f, 0.f, 0.f, 0.f}, b[4] = {0.f, 0.f, 0.f, 0.f};
  if (c < width) {
    int p = p0;
    for (; p + 4 <= p1; p += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        a[u] += part[(size_t)(p + u) * stride + c];
        if (out1) b[u] += part[(size_t)(p + u) * stride + width + c];
      }
    }
    for (; p < p1; ++p) {
      a[0] += part[(size_t)p * stride + c];
      if (out1) b[0] += part[(size_t)p * stride + width + c];
    }
  }
  red[0][q][lane] = (a[0] + a[1]) + (a[2] + a[3]);
  red[1][q][lane] = (b[0] + b[1]) + (b[2] + b[3]);
  __syncthreads();
  if (q == 0 && c < width) {
    out0[c] += (red[0][0][lane] + red[0][1][lane]) + (red[0][2][lane] + red[0][3][lane]);
    if (out1) out1[c] += (red[1][0][lane] + red[1][1][lane]) + (red[1][2][lane] + red[1][3][lane]);
  }
}

__global__ void __launch_bounds__(256)
colsum_finish_kernel(const float* __restrict__ part, int nparts, int stride, float* out0, float* out1, int width) {
  colsum_finish_block(part, nparts, stride, out0, out1, width, (int)blockIdx.x);
}

// several finishes in one launch: job j owns workgroups first[j] .. first[j+1]-1; same arithmetic as above
struct ColsumBatchArgs {
  ColsumJob job[kMaxColsumJobs];
  int first[kMaxColsumJobs + 1];
  int n;
};
__global__ void __launch_bounds__(256)
colsum_finish_batch_kernel(ColsumBatchArgs a) {
  const int id = (int)blockIdx.x;
  ColsumJob j = a.job[0];   // constant indices only: the arguments stay in scalar registers
  int first = 0;
#pragma unroll
  for (int q = 1; q < kMaxColsumJobs; ++q)
    if (q < a.n && id >= a.first[q]) {
      j = a.job[q];
      first = a.first[q];
    }
  colsum_finish_block(j.part, j.nparts, j.stride, j.out0, j.out1, j.width, id - first);
}

// ------------------------------------------------------------------------------------------------
// bias + GeLU
// ------------------------------------------------------------------------------------------------
// Standard normal CDF Phi(z) and density phi(z) from one exponential: with x = |z| / sqrt(2),
// erfc(x) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-x^2), t = 1 / (1 + p x) (Abramowitz & Stegun 7.1.26,
// absolute error below 1.5e-7), taken on the side that needs no cancellation.  These kernels are bound by their
// arithmetic, not by memory (41 vector instructions per element before, against 16 bytes moved per 8 elements), so
// the constants are folded (the coefficients carry erfc's factor 0.5, the exponent -log2(e)/2) and the reciprocal is
// the hardware's 1-ulp one instead of a correctly rounded division (ten instructions): its error is a tenth of the
// formula's own.
__device__ __forceinline__ float normal_cdf_pdf(float z, float* pdf) {
  const float e = __builtin_amdgcn_exp2f(z * z * -0.7213475204444817f);   // exp(-z^2 / 2)
  const float t = __builtin_amdgcn_rcpf(fmaf(fabsf(z), 0.3275911f * 0.7071067811865476f, 1.f));
  const float poly = t * (0.127414796f + t * (-0.142248368f + t * (0.7107068705f + t * (-0.7265760135f + t * 0.5307027145f))));
  const float tail = poly * e;   // 0.5 erfc(|z| / sqrt(2))
  *pdf = e * 0.3989422804014327f;
  return z < 0.f ? tail : 1.f - tail;
}
// tanh(u) = 1 - 2 / (1 + exp(2u)) with the hardware's exponential and reciprocal (absolute error ~1e-7; exp
// overflowing to infinity gives exactly 1, underflowing to zero exactly -1)
__device__ __forceinline__ float fast_tanh(float u) {
  return 1.f - 2.f * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(u * 2.8853900817779268f));
}
template <int MODE> __device__ __forceinline__ float gelu_f(float z) {
  if (MODE == PTDP_GELU_TANH) {
    const float c = 0.7978845608028654f;
    return 0.5f * z * (1.f + fast_tanh(c * (z + 0.044715f * z * z * z)));
  }
  float pdf;
  return z * normal_cdf_pdf(z, &pdf);
}
template <int MODE> __device__ __forceinline__ float gelu_grad_f(float z) {
  if (MODE == PTDP_GELU_TANH) {
    const float c = 0.7978845608028654f;
    const float th = fast_tanh(c * (z + 0.044715f * z * z * z));
    return 0.5f * (1.f + th) + 0.5f * z * (1.f - th * th) * c * (1.f + 3.f * 0.044715f * z * z);
  }
  float pdf;
  const float cdf = normal_cdf_pdf(z, &pdf);
  return cdf + z * pdf;
}
template <typename T, int MODE>
__global__ void bias_gelu_fwd_kernel(const T* __restrict__ z, const T* __restrict__ bias, T* __restrict__ g,
                                     size_t total_vec, int nvec_row) {
  constexpr int N = Vec16<T>::N;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total_vec; i += (size_t)gridDim.x * blockDim.x) {
    const int c = (int)(i % nvec_row);
    Vec16<T> a, b;
    float af[N], bf[N];
    a.load(z + i * N);
    b.load(bias + (size_t)c * N);
    a.unpack(af);
    b.unpack(bf);
#pragma unroll
    for (int j = 0; j < N; ++j) af[j] = gelu_f<MODE>(af[j] + bf[j]);
    a.pack(af);
    a.store(g + i * N);
  }
}

// grid (slabs of 64 column groups, row tiles of kColRows); thread owns one 16-byte column group of every fourth row.
template <typename T, int MODE>
__global__ void __launch_bounds__(256)
bias_gelu_bwd_kernel(const T* dg, const T* __restrict__ z, const T* __restrict__ bias, T* dz,
                     float* __restrict__ part, int rows, int width) {
  constexpr int N = Vec16<T>::N;
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const bool valid = c < width / N;
  float bf[N], acc[N];
#pragma unroll
  for (int j = 0; j < N; ++j) acc[j] = 0.f;
  if (valid) {
    Vec16<T> b;
    b.load(bias + (size_t)c * N);
    b.unpack(bf);
    const int r0 = blockIdx.y * kColRows + (threadIdx.x >> 6), r1 = min(rows, (int)(blockIdx.y + 1) * kColRows);
#pragma unroll 8
    for (int r = r0; r < r1; r += kColLanes) {
      const size_t off = (size_t)r * width + (size_t)c * N;
      Vec16<T> a, zz;
      float af[N], zf[N];
      a.load(dg + off);
      zz.load(z + off);
      a.unpack(af);
      zz.unpack(zf);
#pragma unroll
      for (int j = 0; j < N; ++j) {
        af[j] *= gelu_grad_f<MODE>(zf[j] + bf[j]);
        acc[j] += af[j];
      }
      a.pack(af);
      a.store(dz + off);
    }
  }
  colsum_block_store<N>(acc, part, width, c, valid);
}

// ------------------------------------------------------------------------------------------------
// bias + dropout + add
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void bda_fwd_kernel(const T* __restrict__ in, const T* __restrict__ bias, const T* __restrict__ resid,
                               T* __restrict__ out, size_t total_vec, int nvec_row, uint64_t key, uint32_t thr,
                               float scale) {
  constexpr int N = Vec16<T>::N;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total_vec; i += (size_t)gridDim.x * blockDim.x) {
    const int c = (int)(i % nvec_row);
    Vec16<T> a, b, r;
    float af[N], bf[N], rf[N];
    bool keep[N];
    a.load(in + i * N);
    r.load(resid + i * N);
    b.load(bias + (size_t)c * N);
    a.unpack(af);
    b.unpack(bf);
    r.unpack(rf);
    keep_flags<N>(key, (uint64_t)i * N, thr, keep);
#pragma unroll
    for (int j = 0; j < N; ++j) rf[j] += keep[j] ? (af[j] + bf[j]) * scale : 0.f;
    r.pack(rf);
    r.store(out + i * N);
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
bda_bwd_kernel(const T* __restrict__ dout, T* __restrict__ din, float* __restrict__ part, int rows,
               int width, uint64_t key, uint32_t thr, float scale) {
  constexpr int N = Vec16<T>::N;
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const bool valid = c < width / N;
  float acc[N];
#pragma unroll
  for (int j = 0; j < N; ++j) acc[j] = 0.f;
  if (valid) {
    const int r0 = blockIdx.y * kColRows + (threadIdx.x >> 6), r1 = min(rows, (int)(blockIdx.y + 1) * kColRows);
#pragma unroll 8
    for (int r = r0; r < r1; r += kColLanes) {
      const size_t off = (size_t)r * width + (size_t)c * N;
      Vec16<T> a;
      float af[N];
      bool keep[N];
      a.load(dout + off);
      a.unpack(af);
      keep_flags<N>(key, (uint64_t)off, thr, keep);
#pragma unroll
      for (int j = 0; j < N; ++j) {
        af[j] = keep[j] ? af[j] * scale : 0.f;
        acc[j] += af[j];
      }
      a.pack(af);
      a.store(din + off);
    }
  }
  colsum_block_store<N>(acc, part, width, c, valid);
}

// part[blockIdx.y][c] = sum of in[r][c] over the block's kColRows rows (first stage of a bias gradient
// whose producer lives in another kernel, e.g. the QKV bias).
template <typename T>
__global__ void __launch_bounds__(256)
colsum_rows_kernel(const T* __restrict__ in, float* __restrict__ part, int rows, int width) {
  constexpr int N = Vec16<T>::N;
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const bool valid = c < width / N;
  float acc[N];
#pragma unroll
  for (int j = 0; j < N; ++j) acc[j] = 0.f;
  if (valid) {
    const int r0 = blockIdx.y * kColRows + (threadIdx.x >> 6), r1 = min(rows, (int)(blockIdx.y + 1) * kColRows);
#pragma unroll 8
    for (int r = r0; r < r1; r += kColLanes) {
      Vec16<T> a;
      float af[N];
      a.load(in + (size_t)r * width + (size_t)c * N);
      a.unpack(af);
#pragma unroll
      for (int j = 0; j < N; ++j) acc[j] += af[j];
    }
  }
  colsum_block_store<N>(acc, part, width, c, valid);
}

__global__ void dropout_mask_kernel(uint8_t* keep, int64_t n, uint64_t key, uint32_t thr) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const uint64_t r = mix64(key + kGolden * ((uint64_t)i >> 2));
    keep[i] = ((uint32_t)((r >> (16 * (i & 3))) & 0xffffu) >= thr) ? 1 : 0;
  }
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
static inline int ln_threads(int nvec, int* vpt) {
  // smallest register cache that covers the row with at most 512 threads
  int threads = 64;
  while (threads < 512 && threads < nvec) threads <<= 1;
  int v = (nvec + threads - 1) / threads;
  int p = 1;
  while (p < v) p <<= 1;
  *vpt = p;
  return threads;
}

size_t colsum_scratch_bytes(int rows, int width) {
  // one row of `width` floats per tile of kColRows rows (LayerNorm backward passes twice its row width)
  if (rows <= 0 || width <= 0) return 0;
  return (size_t)((rows + kColRows - 1) / kColRows) * (size_t)width * sizeof(float);
}

template <typename T>
static int ln_fwd_t(const void* x, const void* gain, const void* bias, void* u, float* mu, float* rstd, void* x_copy,
                    int rows, int width, float eps, hipStream_t st) {
  constexpr int N = Vec16<T>::N;
  int vpt;
  const int threads = ln_threads(width / N, &vpt);
  if (vpt > 8) return PTDP_E_UNSUPPORTED;
  const double bytes = (double)rows * width * sizeof(T) * (x_copy ? 3 : 2);
  Launch L(PTDP_K_LN_FWD, bytes, st);
#define PTDP_LN_FWD(V)                                                                                        \
  hipLaunchKernelGGL((layernorm_fwd_kernel<T, V>), dim3(rows), dim3(threads), 0, st, (const T*)x, (const T*)gain, \
                     (const T*)bias, (T*)u, mu, rstd, (T*)x_copy, width, eps)
  switch (vpt) {
    case 1: PTDP_LN_FWD(1); break;
    case 2: PTDP_LN_FWD(2); break;
    case 4: PTDP_LN_FWD(4); break;
    default: PTDP_LN_FWD(8); break;
  }
#undef PTDP_LN_FWD
  return L.status();
}

int launch_layernorm_fwd(int dtype, const void* x, const void* gain, const void* bias, void* u, float* mu,
                         float* rstd, void* x_copy, int rows, int width, float eps, hipStream_t st) {
  if (rows == 0) return PTDP_OK;
  return dtype == PTDP_BF16 ? ln_fwd_t<bf16_t>(x, gain, bias, u, mu, rstd, x_copy, rows, width, eps, st)
                            : ln_fwd_t<float>(x, gain, bias, u, mu, rstd, x_copy, rows, width, eps, st);
}

static int colsum_finish(const float* part, int nparts, int stride, float* out0, float* out1, int width,
                         hipStream_t st, ColsumBatch* defer = nullptr) {
  if (defer) {
    if (defer->n >= kMaxColsumJobs) return PTDP_E_INVALID_ARG;
    defer->job[defer->n++] = ColsumJob{part, nparts, stride, width, out0, out1};
    return PTDP_OK;
  }
  Launch L(PTDP_K_COLSUM, (double)nparts * stride * sizeof(float), st);
  hipLaunchKernelGGL(colsum_finish_kernel, dim3((width + 63) / 64), dim3(256), 0, st, part, nparts, stride, out0,
                     out1, width);
  return L.status();
}

int launch_colsum_batch(const ColsumBatch& batch, hipStream_t st) {
  if (batch.n == 0) return PTDP_OK;
  ColsumBatchArgs a;
  a.n = batch.n;
  double bytes = 0.0;
  int at = 0;
  for (int j = 0; j < kMaxColsumJobs; ++j) {
    a.job[j] = batch.job[j < batch.n ? j : 0];   // unused slots repeat job 0 (never selected)
    a.first[j] = at;
    if (j < batch.n) {
      at += (batch.job[j].width + 63) / 64;
      bytes += (double)batch.job[j].nparts * batch.job[j].stride * sizeof(float);
    }
  }
  a.first[kMaxColsumJobs] = at;
  Launch L(PTDP_K_COLSUM, bytes, st);
  hipLaunchKernelGGL(colsum_finish_batch_kernel, dim3(at), dim3(256), 0, st, a);
  return L.status();
}

// rows walked by one block of the backward kernel: at most 256 blocks (one per compute unit of an MI355X)
static inline int ln_bwd_rows_per_block(int rows) { return rows > 256 ? (rows + 255) / 256 : 1; }

size_t layernorm_bwd_scratch_bytes(int rows, int width) {
  if (rows <= 0 || width <= 0) return 0;
  const int rpb = ln_bwd_rows_per_block(rows);
  return (size_t)((rows + rpb - 1) / rpb) * 2 * (size_t)width * sizeof(float);
}

template <typename T>
static int ln_bwd_t(const void* du, const void* x, const void* gain, const float* mu, const float* rstd,
                    const void* resid, void* dx, float* dgain, float* dbias, void* scratch, int rows, int width,
                    hipStream_t st, ColsumBatch* defer) {
  constexpr int N = Vec16<T>::N;
  int vpt;
  const int threads = ln_threads(width / N, &vpt);
  if (vpt > 8) return PTDP_E_UNSUPPORTED;
  vpt = (width / N + threads - 1) / threads;   // exact count: every vector slot costs two column accumulators
  float* part = (float*)scratch;
  const int rpb = ln_bwd_rows_per_block(rows), nblk = (rows + rpb - 1) / rpb;
  {
    const double bytes = (double)rows * width * sizeof(T) * (resid ? 4 : 3);
    Launch L(PTDP_K_LN_BWD, bytes, st);
#define PTDP_LN_BWD(V)                                                                                        \
  hipLaunchKernelGGL((layernorm_bwd_kernel<T, V>), dim3(nblk), dim3(threads), (size_t)width * sizeof(T), st, (const T*)du, (const T*)x, \
                     (const T*)gain, mu, rstd, (const T*)resid, (T*)dx, part, rows, width, rpb)
    switch (vpt) {
      case 1: PTDP_LN_BWD(1); break;
      case 2: PTDP_LN_BWD(2); break;
      case 3: PTDP_LN_BWD(3); break;
      case 4: PTDP_LN_BWD(4); break;
      case 5: PTDP_LN_BWD(5); break;
      case 6: PTDP_LN_BWD(6); break;
      case 7: PTDP_LN_BWD(7); break;
      default: PTDP_LN_BWD(8); break;
    }
#undef PTDP_LN_BWD
    if (L.status() != PTDP_OK) return L.status();
  }
  return colsum_finish(part, nblk, 2 * width, dgain, dbias, width, st, defer);
}

int launch_layernorm_bwd(int dtype, const void* du, const void* x, const void* gain, const float* mu,
                         const float* rstd, const void* resid, void* dx, float* dgain, float* dbias,
                         void* scratch, int rows, int width, hipStream_t st, ColsumBatch* defer) {
  if (rows == 0) return PTDP_OK;
  return dtype == PTDP_BF16
             ? ln_bwd_t<bf16_t>(du, x, gain, mu, rstd, resid, dx, dgain, dbias, scratch, rows, width, st, defer)
             : ln_bwd_t<float>(du, x, gain, mu, rstd, resid, dx, dgain, dbias, scratch, rows, width, st, defer);
}

static inline int stream_grid(size_t total_vec) {
  size_t blocks = (total_vec + 255) / 256;
  const size_t cap = 256 * 32;  // 32 blocks per CU, grid-stride beyond (16: bias+dropout+add 4-5 % slower; 64 and more: the same)
  return (int)(blocks < cap ? (blocks ? blocks : 1) : cap);
}

template <typename T>
static int gelu_fwd_t(int mode, const void* z, const void* bias, void* g, int rows, int width, hipStream_t st) {
  constexpr int N = Vec16<T>::N;
  const size_t total = (size_t)rows * width / N;
  Launch L(PTDP_K_GELU_FWD, (double)rows * width * sizeof(T) * 2, st);
  if (mode == PTDP_GELU_TANH)
    hipLaunchKernelGGL((bias_gelu_fwd_kernel<T, PTDP_GELU_TANH>), dim3(stream_grid(total)), dim3(256), 0, st,
                       (const T*)z, (const T*)bias, (T*)g, total, width / N);
  else
    hipLaunchKernelGGL((bias_gelu_fwd_kernel<T, PTDP_GELU_ERF>), dim3(stream_grid(total)), dim3(256), 0, st,
                       (const T*)z, (const T*)bias, (T*)g, total, width / N);
  return L.status();
}

int launch_bias_gelu_fwd(int dtype, int mode, const void* z, const void* bias, void* g, int rows, int width,
                         hipStream_t st) {
  if (rows == 0) return PTDP_OK;
  return dtype == PTDP_BF16 ? gelu_fwd_t<bf16_t>(mode, z, bias, g, rows, width, st)
                            : gelu_fwd_t<float>(mode, z, bias, g, rows, width, st);
}

template <typename T>
static int gelu_bwd_t(int mode, const void* dg, const void* z, const void* bias, void* dz, float* dbias,
                      void* scratch, int rows, int width, hipStream_t st, ColsumBatch* defer) {
  constexpr int N = Vec16<T>::N;
  const dim3 grid = colsum_grid(width / N, rows);
  float* part = (float*)scratch;
  {
    Launch L(PTDP_K_GELU_BWD, (double)rows * width * sizeof(T) * 3, st);
    if (mode == PTDP_GELU_TANH)
      hipLaunchKernelGGL((bias_gelu_bwd_kernel<T, PTDP_GELU_TANH>), grid, dim3(256), 0, st, (const T*)dg,
                         (const T*)z, (const T*)bias, (T*)dz, part, rows, width);
    else
      hipLaunchKernelGGL((bias_gelu_bwd_kernel<T, PTDP_GELU_ERF>), grid, dim3(256), 0, st, (const T*)dg,
                         (const T*)z, (const T*)bias, (T*)dz, part, rows, width);
    if (L.status() != PTDP_OK) return L.status();
  }
  return colsum_finish(part, grid.y, width, dbias, nullptr, width, st, defer);
}

int launch_bias_gelu_bwd(int dtype, int mode, const void* dg, const void* z, const void* bias, void* dz,
                         float* dbias, void* scratch, int rows, int width, hipStream_t st, ColsumBatch* defer) {
  if (rows == 0) return PTDP_OK;
  return dtype == PTDP_BF16 ? gelu_bwd_t<bf16_t>(mode, dg, z, bias, dz, dbias, scratch, rows, width, st, defer)
                            : gelu_bwd_t<float>(mode, dg, z, bias, dz, dbias, scratch, rows, width, st, defer);
}

template <typename T>
static int bda_fwd_t(const void* in, const void* bias, const void* resid, void* out, int rows, int width, float p,
                     uint64_t key, hipStream_t st) {
  constexpr int N = Vec16<T>::N;
  const size_t total = (size_t)rows * width / N;
  Launch L(PTDP_K_BDA_FWD, (double)rows * width * sizeof(T) * 3, st);
  hipLaunchKernelGGL((bda_fwd_kernel<T>), dim3(stream_grid(total)), dim3(256), 0, st, (const T*)in, (const T*)bias,
                     (const T*)resid, (T*)out, total, width / N, key, p > 0.f ? dropout_threshold(p) : 0u,
                     1.0f / (1.0f - p));
  return L.status();
}

int launch_bda_fwd(int dtype, const void* in, const void* bias, const void* resid, void* out, int rows, int width,
                   float p, uint64_t key, hipStream_t st) {
  if (rows == 0) return PTDP_OK;
  return dtype == PTDP_BF16 ? bda_fwd_t<bf16_t>(in, bias, resid, out, rows, width, p, key, st)
                            : bda_fwd_t<float>(in, bias, resid, out, rows, width, p, key, st);
}

template <typename T>
static int bda_bwd_t(const void* dout, void* din, float* dbias, void* scratch, int rows, int width, float p,
                     uint64_t key, hipStream_t st, ColsumBatch* defer) {
  constexpr int N = Vec16<T>::N;
  const dim3 grid = colsum_grid(width / N, rows);
  float* part = (float*)scratch;
  {
    Launch L(PTDP_K_BDA_BWD, (double)rows * width * sizeof(T) * 2, st);
    hipLaunchKernelGGL((bda_bwd_kernel<T>), grid, dim3(256), 0, st, (const T*)dout, (T*)din, part, rows, width, key,
                       p > 0.f ? dropout_threshold(p) : 0u, 1.0f / (1.0f - p));
    if (L.status() != PTDP_OK) return L.status();
  }
  return colsum_finish(part, grid.y, width, dbias, nullptr, width, st, defer);
}

int launch_bda_bwd(int dtype, const void* dout, void* din, float* dbias, void* scratch, int rows, int width, float p,
                   uint64_t key, hipStream_t st, ColsumBatch* defer) {
  if (rows == 0) return PTDP_OK;
  return dtype == PTDP_BF16 ? bda_bwd_t<bf16_t>(dout, din, dbias, scratch, rows, width, p, key, st, defer)
                            : bda_bwd_t<float>(dout, din, dbias, scratch, rows, width, p, key, st, defer);
}

// Column-sum partials for callers that may not allocate: one array per device, kept until the process
// ends.  In host code `scratch` is only a handle for hipGetSymbolAddress, never a device address: every
// launch below is handed the address looked up once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static int static_scratch(void** out) {
  const int d = device_slot();
  if (d < 0) return PTDP_E_HIP;
  void* ptr = g_scratch_ptr[d].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return PTDP_E_HIP;
    g_scratch_ptr[d].store(ptr, std::memory_order_release);   // racing threads store the same address
  }
  *out = ptr;
  return PTDP_OK;
}

// launch_bda_bwd with the partials in this device's static array (every partial that the finish kernel reads
// is written by the first kernel of the same call, so nothing has to be cleared between calls)
int launch_bda_bwd_static(int dtype, const void* dout, void* din, float* dbias, int rows, int width, float p,
                          uint64_t key, hipStream_t st) {
  if (colsum_scratch_bytes(rows, width) > kStaticScratchBytes) return PTDP_E_TOO_SMALL;
  if (rows == 0) return PTDP_OK;
  void* ptr = nullptr;
  const int rc = static_scratch(&ptr);
  if (rc != PTDP_OK) return rc;
  return launch_bda_bwd(dtype, dout, din, dbias, ptr, rows, width, p, key, st, nullptr);
}

template <typename T>
static int colsum_t(const void* in, float* out, void* scratch, int rows, int width, hipStream_t st, ColsumBatch* defer) {
  constexpr int N = Vec16<T>::N;
  const dim3 grid = colsum_grid(width / N, rows);
  float* part = (float*)scratch;
  {
    Launch L(PTDP_K_COLSUM, (double)rows * width * sizeof(T), st);
    hipLaunchKernelGGL((colsum_rows_kernel<T>), grid, dim3(256), 0, st, (const T*)in, part, rows, width);
    if (L.status() != PTDP_OK) return L.status();
  }
  return colsum_finish(part, grid.y, width, out, nullptr, width, st, defer);
}

int launch_colsum(int dtype, const void* in, float* out, void* scratch, int rows, int width, hipStream_t st,
                  ColsumBatch* defer) {
  if (rows == 0) return PTDP_OK;
  return dtype == PTDP_BF16 ? colsum_t<bf16_t>(in, out, scratch, rows, width, st, defer)
                            : colsum_t<float>(in, out, scratch, rows, width, st, defer);
}

int launch_dropout_mask(uint8_t* keep, int64_t n, float p, uint64_t key, hipStream_t st) {
  if (n == 0) return PTDP_OK;
  Launch L(PTDP_K_OTHER, (double)n, st);
  hipLaunchKernelGGL(dropout_mask_kernel, dim3(stream_grid((size_t)n)), dim3(256), 0, st, keep, n, key,
                     p > 0.f ? dropout_threshold(p) : 0u);
  return L.status();
}

}  // namespace ptdp
