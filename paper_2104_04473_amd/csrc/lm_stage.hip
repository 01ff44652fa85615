// First- and last-stage extras of the GPT model: token + position embedding with hidden dropout (and
// its backward), and the loss over the logit layer's output (softmax cross-entropy, forward and
// backward in one pass over the logits).  The paper counts the embedding tables in eq. (2) and the
// logit layer's GEMMs in its appendix; the GEMMs and the final LayerNorm run through the kernels the
// transformer layers use.  All kernels here are HBM-bound.
#include "common.h"

namespace ptdp {

// ------------------------------------------------------------------------------------------------
// x[i, j, :] = Drop(E_word[token[i, j] - v0] (zero row if outside this shard) + E_pos[i])
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void embed_fwd_kernel(const int32_t* __restrict__ tokens, const T* __restrict__ e_word,
                                 const T* __restrict__ e_pos, T* __restrict__ x, size_t total_vec, int nvec_row, int b,
                                 int v0, int vrows, uint64_t key, uint32_t thr, float scale) {
  constexpr int N = Vec16<T>::N;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total_vec; i += (size_t)gridDim.x * blockDim.x) {
    const size_t row = i / nvec_row;
    const int c = (int)(i % nvec_row);
    const int local = tokens[row] - v0;
    Vec16<T> w, p;
    float wf[N], pf[N];
    bool keep[N];
    p.load(e_pos + ((size_t)(row / b) * nvec_row + c) * N);
    p.unpack(pf);
    if (local >= 0 && local < vrows) {
      w.load(e_word + ((size_t)local * nvec_row + c) * N);
      w.unpack(wf);
    } else {
#pragma unroll
      for (int j = 0; j < N; ++j) wf[j] = 0.f;
    }
    keep_flags<N>(key, (uint64_t)i * N, thr, keep);
#pragma unroll
    for (int j = 0; j < N; ++j) wf[j] = keep[j] ? (wf[j] + pf[j]) * scale : 0.f;
    w.pack(wf);
    w.store(x + i * N);
  }
}

// d = Drop'(dx) written out for the scatter below; d_pos[i, :] += sum_j d[i, j, :] (j in order).
template <typename T>
__global__ void embed_bwd_mask_kernel(const T* __restrict__ dx, T* __restrict__ d, float* __restrict__ d_pos, int s, int b,
                                      int nvec_row, uint64_t key, uint32_t thr, float scale) {
  constexpr int N = Vec16<T>::N;
  const size_t total = (size_t)s * nvec_row;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const size_t pos = i / nvec_row;
    const int c = (int)(i % nvec_row);
    float acc[N];
#pragma unroll
    for (int j = 0; j < N; ++j) acc[j] = 0.f;
    for (int j = 0; j < b; ++j) {
      const size_t v = (pos * b + j) * nvec_row + c;
      Vec16<T> a;
      float af[N];
      bool keep[N];
      a.load(dx + v * N);
      a.unpack(af);
      keep_flags<N>(key, (uint64_t)v * N, thr, keep);
#pragma unroll
      for (int e = 0; e < N; ++e) {
        af[e] = keep[e] ? af[e] * scale : 0.f;
        acc[e] += af[e];
      }
      a.pack(af);
      a.store(d + v * N);
    }
    float* o = d_pos + (pos * nvec_row + c) * N;
#pragma unroll
    for (int e = 0; e < N; ++e) o[e] += acc[e];
  }
}

// d_word[r, :] += sum over the tokens with id v0 + r of d[token, :], in token order.  One workgroup per
// vocabulary row; each wave finds the row's tokens itself (64 ids per ballot, ascending) and owns the
// column slices wave, wave + 4, ...: no atomics, no two waves touch the same element, and rows that no
// token names are left untouched.
template <typename T>
__global__ void __launch_bounds__(256)
embed_bwd_scatter_kernel(const int32_t* __restrict__ tokens, const T* __restrict__ d, float* __restrict__ d_word,
                         int ntok, int nvec_row, int v0) {
  constexpr int N = Vec16<T>::N;
  const int id = v0 + blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  bool any = false;
  for (int t0 = 0; t0 < ntok && !any; t0 += 64) {
    const int t = t0 + lane;
    any = __any(t < ntok && tokens[t] == id);
  }
  if (!any) return;
  for (int c = wave * 64 + lane; c - lane < nvec_row; c += 4 * 64) {
    const bool col_ok = c < nvec_row;
    float acc[N];
#pragma unroll
    for (int j = 0; j < N; ++j) acc[j] = 0.f;
    for (int t0 = 0; t0 < ntok; t0 += 64) {
      const int t = t0 + lane;
      unsigned long long m = __ballot(t < ntok && tokens[t] == id);
      while (m) {
        const int bit = __ffsll((long long)m) - 1;
        m &= m - 1;
        if (col_ok) {
          Vec16<T> a;
          float af[N];
          a.load(d + ((size_t)(t0 + bit) * nvec_row + c) * N);
          a.unpack(af);
#pragma unroll
          for (int j = 0; j < N; ++j) acc[j] += af[j];
        }
      }
    }
    if (col_ok) {
      float* o = d_word + ((size_t)blockIdx.x * nvec_row + c) * N;
#pragma unroll
      for (int j = 0; j < N; ++j) o[j] += acc[j];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Loss over one shard's logits [rows, vrows]: per token m = max, z = sum exp(l - m),
// loss = log z + m - l[target] (target outside the shard: no target term), and in place
// l <- (exp(l - m) / z - [v == target]) * grad_scale.  One workgroup per token; the row is read three
// times, the second and third time from cache.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
xent_kernel(T* __restrict__ logits, const int32_t* __restrict__ targets, float* __restrict__ token_loss, int vrows, int v0,
            float grad_scale) {
  constexpr int N = Vec16<T>::N;
  __shared__ float red[16];
  T* row = logits + (size_t)blockIdx.x * vrows;
  const int nvec = vrows / N;
  float mx = -INFINITY;
  for (int v = threadIdx.x; v < nvec; v += blockDim.x) {
    Vec16<T> a;
    float af[N];
    a.load(row + (size_t)v * N);
    a.unpack(af);
#pragma unroll
    for (int j = 0; j < N; ++j) mx = fmaxf(mx, af[j]);
  }
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float z = 0.f;
  for (int v = threadIdx.x; v < nvec; v += blockDim.x) {
    Vec16<T> a;
    float af[N];
    a.load(row + (size_t)v * N);
    a.unpack(af);
#pragma unroll
    for (int j = 0; j < N; ++j) z += __expf(af[j] - mx);
  }
  z = block_sum(z, red + 4);
  const int local = targets[blockIdx.x] - v0;
  const bool inside = local >= 0 && local < vrows;
  if (threadIdx.x == 0) {
    float picked = 0.f;
    if (inside) {
      if (sizeof(T) == 2) picked = bf16_to_f32(reinterpret_cast<const bf16_t*>(row)[local]);
      else picked = reinterpret_cast<const float*>(row)[local];
    }
    token_loss[blockIdx.x] = __logf(z) + mx - picked;
  }
  __syncthreads();   // the target logit is read before the row is overwritten
  const float rz = grad_scale / z;
  for (int v = threadIdx.x; v < nvec; v += blockDim.x) {
    Vec16<T> a;
    float af[N];
    a.load(row + (size_t)v * N);
    a.unpack(af);
#pragma unroll
    for (int j = 0; j < N; ++j) {
      af[j] = __expf(af[j] - mx) * rz;
      if (inside && v * N + j == local) af[j] -= grad_scale;
    }
    a.pack(af);
    a.store(row + (size_t)v * N);
  }
}

// loss[0] = mean of token_loss[0 .. n), summed in a fixed order by one workgroup
__global__ void __launch_bounds__(256) loss_mean_kernel(const float* __restrict__ token_loss, float* __restrict__ loss, int n) {
  __shared__ float red[16];
  float a = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) a += token_loss[i];
  a = block_sum(a, red);
  if (threadIdx.x == 0) loss[0] = a / (float)n;
}

static inline int grid_for(size_t total) {
  const size_t blocks = (total + 255) / 256, cap = 256 * 16;
  return (int)(blocks < cap ? (blocks ? blocks : 1) : cap);
}

template <typename T>
static int embed_fwd_t(const int32_t* tokens, const void* e_word, const void* e_pos, void* x, int s, int b, int h, int v0,
                       int vrows, float p, uint64_t key, hipStream_t st) {
  constexpr int N = Vec16<T>::N;
  const size_t total = (size_t)s * b * h / N;
  Launch L(PTDP_K_EMBED, (double)s * b * h * sizeof(T) * 2 + (double)s * h * sizeof(T), st);
  hipLaunchKernelGGL((embed_fwd_kernel<T>), dim3(grid_for(total)), dim3(256), 0, st, tokens, (const T*)e_word,
                     (const T*)e_pos, (T*)x, total, h / N, b, v0, vrows, key, p > 0.f ? dropout_threshold(p) : 0u,
                     1.0f / (1.0f - p));
  return L.status();
}

int launch_embed_fwd(int dtype, const int32_t* tokens, const void* e_word, const void* e_pos, void* x, int s, int b, int h,
                     int v0, int vrows, float p, uint64_t key, hipStream_t st) {
  return dtype == PTDP_BF16 ? embed_fwd_t<bf16_t>(tokens, e_word, e_pos, x, s, b, h, v0, vrows, p, key, st)
                            : embed_fwd_t<float>(tokens, e_word, e_pos, x, s, b, h, v0, vrows, p, key, st);
}

template <typename T>
static int embed_bwd_t(const int32_t* tokens, const void* dx, void* dmasked, float* d_e_word, float* d_e_pos, int s, int b,
                       int h, int v0, int vrows, float p, uint64_t key, hipStream_t st) {
  constexpr int N = Vec16<T>::N;
  Launch L(PTDP_K_EMBED, (double)s * b * h * sizeof(T) * 3 + (double)s * h * 8, st);
  hipLaunchKernelGGL((embed_bwd_mask_kernel<T>), dim3(grid_for((size_t)s * h / N)), dim3(256), 0, st, (const T*)dx,
                     (T*)dmasked, d_e_pos, s, b, h / N, key, p > 0.f ? dropout_threshold(p) : 0u, 1.0f / (1.0f - p));
  hipLaunchKernelGGL((embed_bwd_scatter_kernel<T>), dim3(vrows), dim3(256), 0, st, tokens, (const T*)dmasked, d_e_word,
                     s * b, h / N, v0);
  return L.status();
}

int launch_embed_bwd(int dtype, const int32_t* tokens, const void* dx, void* dmasked, float* d_e_word, float* d_e_pos,
                     int s, int b, int h, int v0, int vrows, float p, uint64_t key, hipStream_t st) {
  return dtype == PTDP_BF16 ? embed_bwd_t<bf16_t>(tokens, dx, dmasked, d_e_word, d_e_pos, s, b, h, v0, vrows, p, key, st)
                            : embed_bwd_t<float>(tokens, dx, dmasked, d_e_word, d_e_pos, s, b, h, v0, vrows, p, key, st);
}

int launch_xent(int dtype, void* logits, const int32_t* targets, float* token_loss, float* loss, int rows, int vrows,
                int v0, float grad_scale, hipStream_t st) {
  const size_t esz = dtype == PTDP_BF16 ? 2 : 4;
  Launch L(PTDP_K_XENT, (double)rows * vrows * esz * 2, st);
  if (dtype == PTDP_BF16)
    hipLaunchKernelGGL((xent_kernel<bf16_t>), dim3(rows), dim3(256), 0, st, (bf16_t*)logits, targets, token_loss, vrows, v0,
                       grad_scale);
  else
    hipLaunchKernelGGL((xent_kernel<float>), dim3(rows), dim3(256), 0, st, (float*)logits, targets, token_loss, vrows, v0,
                       grad_scale);
  hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(256), 0, st, (const float*)token_loss, loss, rows);
  return L.status();
}

}  // namespace ptdp
