// fp32 instantiation of the POP prefill path: every step of Sec. 2.1 / Sec. 3.3 with fp32 weights,
// activations and cache entries and fp32 accumulation.  It exists for tight numerical checks on small
// models (max relative error 1e-4 against an fp64 reference instead of the 2e-2 of the bf16 path):
// plain, LDS-tiled FMA kernels, no MFMA, not tuned for speed.
#include <math.h>

#include "pop_device.h"
#include "pop_kernels.h"

namespace pop {
namespace f32 {

namespace impl {

// h[t,:] = row_src[t] < 0 ? table[tokens[t],:] : embeds[row_src[t],:]
__global__ void embed_kernel(const float* __restrict__ table, const int32_t* __restrict__ tokens,
                             const int32_t* __restrict__ row_src, const float* __restrict__ embeds,
                             float* __restrict__ h, int d) {
  const int t = blockIdx.x;
  const int rs = row_src ? row_src[t] : -1;
  const float* src = rs < 0 ? table + (size_t)tokens[t] * d : embeds + (size_t)rs * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)t * d + i] = src[i];
}

// out[t,:] = x[r,:] * rsqrt(mean(x[r,:]^2) + eps) * gamma, r = row_idx ? row_idx[t] : t     (LN of Sec. 2.1)
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gamma,
                                                      float* __restrict__ out, const int32_t* __restrict__ row_idx,
                                                      int d, float eps) {
  __shared__ float red[4];
  const int t = blockIdx.x;
  const float* xr = x + (size_t)(row_idx ? row_idx[t] : t) * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) ss += xr[i] * xr[i];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = (red[0] + red[1]) + (red[2] + red[3]);
  const float rstd = 1.0f / sqrtf(tot / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) out[(size_t)t * d + i] = xr[i] * rstd * gamma[i];
}

__device__ __forceinline__ float glu_act(float g, int act) {
  if (act == 0) return g / (1.f + expf(-g));
  const float u = 0.7978845608028654f * (g + 0.044715f * g * g * g);
  return 0.5f * g * (1.f + tanhf(u));
}

// C = A[M,K] W[N,K]^T, 64x64 output tile per work-group, 16-wide K steps through LDS, 4x4 outputs per
// thread.  EPI: 0 store, 1 out += C, 2 out = act(A Wg^T) * (A Wu^T) with Wg = W rows 0..N-1, Wu = rows N..2N-1.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_kernel(const float* __restrict__ A, int lda, const float* __restrict__ W,
                                                   int ldw, float* __restrict__ out, int ldc, int M, int N, int K,
                                                   int act, float scale /* EPI 1: out += scale * C */) {
  constexpr int BT = 64, BKK = 16;
  __shared__ float sa[BKK][BT + 1], sw[BKK][BT + 1], su[EPI == 2 ? BKK : 1][BT + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
  float acc[4][4], acu[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = acu[i][j] = 0.f;
  for (int k0 = 0; k0 < K; k0 += BKK) {
    // 64 rows x 16 k per tile = 1024 values, 4 per thread: thread -> (row = id / 4 + 0.., k = (id % 4) * 4 ..)
    for (int e = threadIdx.x; e < BT * BKK; e += 256) {
      const int r = e / BKK, kk = e % BKK;
      const int k = k0 + kk;
      sa[kk][r] = (m0 + r < M && k < K) ? A[(size_t)(m0 + r) * lda + k] : 0.f;
      sw[kk][r] = (n0 + r < N && k < K) ? W[(size_t)(n0 + r) * ldw + k] : 0.f;
      if (EPI == 2) su[kk][r] = (n0 + r < N && k < K) ? W[(size_t)(N + n0 + r) * ldw + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BKK; ++kk) {
      float av[4], wv[4], uv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = sa[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        wv[j] = sw[kk][tx * 4 + j];
        uv[j] = EPI == 2 ? su[kk][tx * 4 + j] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] += av[i] * wv[j];
          if (EPI == 2) acu[i][j] += av[i] * uv[j];
        }
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
      float* o = out + (size_t)m * ldc + n;
      if (EPI == 0) *o = acc[i][j];
      else if (EPI == 1) *o += acc[i][j] * scale;
      else *o = glu_act(acc[i][j], act) * acu[i][j];
    }
  }
}

// RoPE (half-split pairs, angle formed in fp64) of the q and k heads of `rows` rows in place, and
// append of k, v to the paged cache at slot[row].  grid (rows, Hq + 2 Hkv), hd/2 threads rounded up to whole
// waves.  With q_gamma / k_gamma every query / key head is RMS-normalised over hd first (per-head QK-norm).
__global__ void rope_write_kernel(float* __restrict__ qkv, int ld, int q_col, int k_col, int v_col, int n_q_heads,
                                  int n_kv_heads, int hd, const int32_t* __restrict__ pos,
                                  const int32_t* __restrict__ slot, double neg2_over_hd_log2theta,
                                  float* __restrict__ k_pool, float* __restrict__ v_pool, int P,
                                  const float* __restrict__ q_gamma, const float* __restrict__ k_gamma, float qk_eps,
                                  KvQuant kvq) {
  __shared__ float red[2];
  const int r = blockIdx.x, head = blockIdx.y;
  const int half = hd >> 1;
  const int i = threadIdx.x;      // whole waves: 64 or 128 threads, the first `half` of them work
  const bool act = i < half;
  const int s = slot[r];
  float* row = qkv + (size_t)r * ld;
  if (head < n_q_heads + n_kv_heads) {
    const bool is_q = head < n_q_heads;
    if (is_q && q_col < 0) return;
    float* x = row + (is_q ? q_col + head * hd : k_col + (head - n_q_heads) * hd);
    float a = act ? x[i] : 0.f, b = act ? x[i + half] : 0.f;
    const float* gamma = is_q ? q_gamma : k_gamma;
    if (gamma) {   // per-head QK-norm before the rotation (uniform over the block)
      const float ss = wave_sum(a * a + b * b);
      if ((i & 63) == 0) red[i >> 6] = ss;
      __syncthreads();
      const float tot = blockDim.x > 64 ? red[0] + red[1] : red[0];
      const float rstd = 1.0f / sqrtf(tot / (float)hd + qk_eps);
      if (act) {
        a *= rstd * gamma[i];
        b *= rstd * gamma[i + half];
      }
    }
    if (!act) return;
    const double ang = (double)pos[r] * exp2((double)i * neg2_over_hd_log2theta);
    double sd, cd;
    sincos(ang, &sd, &cd);
    const float c = (float)cd, sn = (float)sd;
    const float lo = a * c - b * sn, hi = b * c + a * sn;
    x[i] = lo;
    x[i + half] = hi;
    if (!is_q) {
      // 8-bit cache: the fp32 entry holds the value of the e4m3 code the element rounds to
      float* o = k_pool + (((size_t)(s / P) * n_kv_heads + (head - n_q_heads)) * P + (s % P)) * hd;
      o[i] = kvq.fp8 ? e4m3_decode(e4m3_encode(lo * kvq.k_inv)) * kvq.k_scale : lo;
      o[i + half] = kvq.fp8 ? e4m3_decode(e4m3_encode(hi * kvq.k_inv)) * kvq.k_scale : hi;
    }
  } else {
    if (!act) return;
    const int hh = head - n_q_heads - n_kv_heads;
    const float* x = row + v_col + hh * hd;
    float* o = v_pool + (((size_t)(s / P) * n_kv_heads + hh) * P + (s % P)) * hd;
    o[i] = kvq.fp8 ? e4m3_decode(e4m3_encode(x[i] * kvq.v_inv)) * kvq.v_scale : x[i];
    o[i + half] = kvq.fp8 ? e4m3_decode(e4m3_encode(x[i + half] * kvq.v_inv)) * kvq.v_scale : x[i + half];
  }
}

// Attn of Sec. 2.1 for one (row, query head) per work-group against the paged cache of the row's
// sequence: keys lo..pos with lo = max(0, pos - window + 1) (window > 0) or 0, and not below the
// first position the layer holds an entry for (kv_first[sequence], if given).  Scores live in LDS.
__global__ __launch_bounds__(256) void attention_kernel(const float* __restrict__ q, int ldq, int q_col,
                                                        float* __restrict__ out, const int32_t* __restrict__ row_seq,
                                                        const int32_t* __restrict__ row_pos,
                                                        const float* __restrict__ k_pool,
                                                        const float* __restrict__ v_pool,
                                                        const int32_t* __restrict__ block_table, int max_pages, int P,
                                                        int window, const int32_t* __restrict__ kv_first,
                                                        int n_q_heads, int n_kv_heads, int hd, float scale) {
  extern __shared__ float smem[];
  __shared__ float red[4];
  float* qs = smem;        // [hd]
  float* sc = smem + hd;   // [n keys]
  const int r = blockIdx.x, head = blockIdx.y, tid = threadIdx.x;
  const int b = row_seq[r], pos = row_pos[r];
  int lo = window > 0 ? max(0, pos - window + 1) : 0;
  if (kv_first) lo = max(lo, min(kv_first[b], pos));   // the row's own entry always exists
  const int n = pos - lo + 1;
  const int kvh = head / (n_q_heads / n_kv_heads);
  const int32_t* bt = block_table + (size_t)b * max_pages;
  for (int i = tid; i < hd; i += 256) qs[i] = q[(size_t)r * ldq + q_col + head * hd + i];
  __syncthreads();
  float mx = -INFINITY;
  for (int j = tid; j < n; j += 256) {
    const int key = lo + j;
    const float* kp = k_pool + (((size_t)bt[key / P] * n_kv_heads + kvh) * P + (key % P)) * hd;
    float s = 0.f;
    for (int i = 0; i < hd; ++i) s += qs[i] * kp[i];
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int j = tid; j < n; j += 256) {
    const float p = expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  if ((tid & 63) == 0) red[tid >> 6] = sum;
  __syncthreads();
  const float tot = (red[0] + red[1]) + (red[2] + red[3]);
  for (int e = tid; e < hd; e += 256) {
    float acc = 0.f;
    for (int j = 0; j < n; ++j) {
      const int key = lo + j;
      acc += sc[j] * v_pool[(((size_t)bt[key / P] * n_kv_heads + kvh) * P + (key % P)) * hd + e];
    }
    out[(size_t)r * n_q_heads * hd + head * hd + e] = acc / tot;
  }
}

}  // namespace impl

void launch_embed(const float* table, const int32_t* tokens, const int32_t* row_src, const float* embeds, float* h,
                  int T, int d, hipStream_t st) {
  if (T <= 0) return;
  hipLaunchKernelGGL(impl::embed_kernel, dim3(T), dim3(256), 0, st, table, tokens, row_src, embeds, h, d);
}

void launch_rmsnorm(const float* x, const float* gamma, float* out, const int32_t* row_idx, int rows, int d, float eps,
                    hipStream_t st) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(impl::rmsnorm_kernel, dim3(rows), dim3(256), 0, st, x, gamma, out, row_idx, d, eps);
}

void launch_gemm(const float* A, int lda, const float* W, int ldw, float* out, int ldc, int M, int N, int K, int epi,
                 int act, hipStream_t st, float scale) {
  if (M <= 0 || N <= 0) return;
  const dim3 grid((N + 63) / 64, (M + 63) / 64);
  if (epi == EPI_STORE)
    hipLaunchKernelGGL((impl::gemm_kernel<0>), grid, dim3(256), 0, st, A, lda, W, ldw, out, ldc, M, N, K, act, scale);
  else if (epi == EPI_ADD)
    hipLaunchKernelGGL((impl::gemm_kernel<1>), grid, dim3(256), 0, st, A, lda, W, ldw, out, ldc, M, N, K, act, scale);
  else
    hipLaunchKernelGGL((impl::gemm_kernel<2>), grid, dim3(256), 0, st, A, lda, W, ldw, out, ldc, M, N, K, act, scale);
}

void launch_rope_write(float* qkv, int ld, int q_col, int k_col, int v_col, int n_q_heads, int n_kv_heads, int hd,
                       const int32_t* pos, const int32_t* slot, double theta, float* k_pool, float* v_pool, int P,
                       int rows, hipStream_t st, const float* q_gamma, const float* k_gamma, float qk_eps, KvQuant kvq) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(impl::rope_write_kernel, dim3(rows, n_q_heads + 2 * n_kv_heads), dim3((hd / 2 + 63) / 64 * 64), 0, st, qkv, ld,
                     q_col, k_col, v_col, n_q_heads, n_kv_heads, hd, pos, slot, -2.0 / (double)hd * log2(theta), k_pool,
                     v_pool, P, q_gamma, k_gamma, qk_eps, kvq);
}

hipError_t launch_attention(const float* q, int ldq, int q_col, float* out, const int32_t* row_seq,
                            const int32_t* row_pos, const float* k_pool, const float* v_pool,
                            const int32_t* block_table, int max_pages, int P, int window, const int32_t* kv_first, int rows, int n_q_heads,
                            int n_kv_heads, int hd, int max_len, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  const size_t smem = ((size_t)hd + (size_t)max_len) * sizeof(float);
  if (max_len > kMaxContext) return hipErrorInvalidValue;
  hipLaunchKernelGGL(impl::attention_kernel, dim3(rows, n_q_heads), dim3(256), smem, st, q, ldq, q_col, out, row_seq,
                     row_pos, k_pool, v_pool, block_table, max_pages, P, window, kv_first, n_q_heads, n_kv_heads, hd,
                     1.f / sqrtf((float)hd));
  return hipGetLastError();
}

}  // namespace f32
}  // namespace pop
