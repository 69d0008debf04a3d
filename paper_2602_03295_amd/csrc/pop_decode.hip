// Decode-step kernels: one row per sequence through a full layer against the paged KV cache (few-row
// projections, attention over the cache with RoPE and the append of the new entry inside, greedy choice).
// They carry the boundary token of Sec. 3.3 ("Boundary Handling for the Last Input Token": x_N is
// the first decode step with the full model) and pop_decode_step (Sec. 3.2, decode operator).
// With M <= 8 rows every projection streams its weights once: these kernels are HBM-bound.
#include <type_traits>

#include "pop_device.h"
#include "pop_kernels.h"

namespace pop {

namespace decode_impl {

__device__ __forceinline__ float glu_act_f(float g, int act) {
  if (act == 0) return g / (1.f + __expf(-g));
  const float u = 0.7978845608028654f * (g + 0.044715f * g * g * g);
  return 0.5f * g * (1.f + tanhf(u));
}

// acc += sum of the eight bf16 products of w and x, with v_dot2_f32_bf16 (two products and the fp32 sum per
// instruction, operands taken as packed bf16 without conversion): a quarter of the vector instructions of
// converting to fp32 and multiplying, which is what kept the forms with several batch rows below the HBM rate.
__device__ __forceinline__ void fma8(float (&acc), const uint4& w, const uint4& x) {
  typedef __bf16 bf2_t __attribute__((ext_vector_type(2)));
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2_t, w.x), __builtin_bit_cast(bf2_t, x.x), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2_t, w.y), __builtin_bit_cast(bf2_t, x.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2_t, w.z), __builtin_bit_cast(bf2_t, x.z), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2_t, w.w), __builtin_bit_cast(bf2_t, x.w), acc, false);
}

// Each wave owns RW weight rows (for GLU: RW gate rows and the matching RW up rows) and all M batch
// rows; lanes stride over K in 16-byte chunks; fp32 accumulation, wave reduction at the end.
// The K loop is unrolled by U with all weight loads of an unrolled step issued before the first
// multiply: with one row per step a wave has too few bytes in flight to cover HBM latency.
// NORM: the M input rows are fp32 rows xf that are RMS-normalised first (Sec. 2.1, the LN of the layer
// equations): every work-group computes the M normalised bf16 rows into LDS, with the thread layout, the
// summation order and the roundings of rmsnorm_kernel (same bits), which saves the launch of that kernel
// and the round trip of its output.
template <int M, int EPI, int RW, int U, bool NORM>
__global__ __launch_bounds__(256) void gemv_kernel(const bf16_t* __restrict__ x, const float* __restrict__ xf,
                                                   const float* __restrict__ gamma, float eps,
                                                   const bf16_t* __restrict__ W, void* __restrict__ out, int N, int K,
                                                   long long ldo, int act, float scale /* ADD: out += scale * C */,
                                                   int m_valid /* rows that exist (<= M); the others repeat the last */) {
  constexpr int NR = EPI == GEMV_GLU_BF16 ? 2 * RW : RW;  // weight rows streamed per wave
  typedef __attribute__((__vector_size__(16))) unsigned int u32x4_t;
  extern __shared__ __attribute__((aligned(16))) unsigned char gemv_smem[];   // NORM: bf16 [M][K], then float [M][4]
  const bf16_t* xs = reinterpret_cast<const bf16_t*>(gemv_smem);
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n0 = (blockIdx.x * 4 + wave) * RW;
  const bf16_t* wr[NR];
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    int row;
    if (EPI == GEMV_GLU_BF16) row = (r < RW ? 0 : N) + min(n0 + (r % RW), N - 1);
    else row = min(n0 + r, N - 1);
    wr[r] = W + (size_t)row * K;
  }
  int k = lane * 8;
  // NORM: the weights of the first unrolled step are requested before the rows are normalised, so that
  // they travel meanwhile
  u32x4_t wl[U][NR];
  bool preloaded = NORM && k + (U - 1) * 512 < K;
  if (preloaded) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int r = 0; r < NR; ++r)
        wl[u][r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wr[r] + k + u * 512));
  }
  if (NORM) {
    bf16_t* xw = reinterpret_cast<bf16_t*>(gemv_smem);
    float* red = reinterpret_cast<float*>(gemv_smem + (size_t)M * K * 2);
#pragma unroll 1
    for (int m = 0; m < M; ++m) {
      const float* xr = xf + (size_t)m * K;
      float4 v[8];
      float ss = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int i = (j * 256 + threadIdx.x) * 4;
        if (i < K) {
          v[j] = *reinterpret_cast<const float4*>(xr + i);
          ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
        }
      }
      ss = wave_sum(ss);
      if ((threadIdx.x & 63) == 0) red[m * 4 + (threadIdx.x >> 6)] = ss;
      __syncthreads();
      const float total = red[m * 4] + red[m * 4 + 1] + red[m * 4 + 2] + red[m * 4 + 3];
      const float rstd = rsqrtf(total / (float)K + eps);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int i = (j * 256 + threadIdx.x) * 4;
        if (i < K) {
          const float4 gg = *reinterpret_cast<const float4*>(gamma + i);
          uint2 pk;
          pk.x = pack_bf16x2(v[j].x * rstd * gg.x, v[j].y * rstd * gg.y);
          pk.y = pack_bf16x2(v[j].z * rstd * gg.z, v[j].w * rstd * gg.w);
          *reinterpret_cast<uint2*>(xw + (size_t)m * K + i) = pk;
        }
      }
    }
    __syncthreads();
  }
  if (n0 >= N) return;
  auto x_chunk = [&](int m, int k) {
    return NORM ? *reinterpret_cast<const uint4*>(xs + (size_t)m * K + k)
                : *reinterpret_cast<const uint4*>(x + (size_t)min(m, m_valid - 1) * K + k);
  };
  float acc[NR][M];
#pragma unroll
  for (int r = 0; r < NR; ++r)
#pragma unroll
    for (int m = 0; m < M; ++m) acc[r][m] = 0.f;
  for (; k + (U - 1) * 512 < K; k += U * 512) {
    if (!preloaded) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < NR; ++r)
          wl[u][r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wr[r] + k + u * 512));
    }
    preloaded = false;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      uint4 xv[M];
#pragma unroll
      for (int m = 0; m < M; ++m) xv[m] = x_chunk(m, k + u * 512);
#pragma unroll
      for (int r = 0; r < NR; ++r) {
        const uint4 wv = make_uint4(wl[u][r][0], wl[u][r][1], wl[u][r][2], wl[u][r][3]);
#pragma unroll
        for (int m = 0; m < M; ++m) fma8(acc[r][m], wv, xv[m]);
      }
    }
  }
  for (; k < K; k += 512) {
    uint4 xv[M];
#pragma unroll
    for (int m = 0; m < M; ++m) xv[m] = x_chunk(m, k);
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const u32x4_t wt = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(wr[r] + k));
      const uint4 wv = make_uint4(wt[0], wt[1], wt[2], wt[3]);
#pragma unroll
      for (int m = 0; m < M; ++m) fma8(acc[r][m], wv, xv[m]);
    }
  }
#pragma unroll
  for (int r = 0; r < NR; ++r)
#pragma unroll
    for (int m = 0; m < M; ++m) acc[r][m] = wave_sum(acc[r][m]);
  if (lane != 0) return;
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int n = n0 + r;
    if (n >= N) break;
#pragma unroll
    for (int m = 0; m < M; ++m) {
      if (m >= m_valid) break;
      if (EPI == GEMV_GLU_BF16) {
        reinterpret_cast<bf16_t*>(out)[(size_t)m * ldo + n] = f32_to_bf16(glu_act_f(acc[r][m], act) * acc[r + RW][m]);
      } else {
        float* o = reinterpret_cast<float*>(out) + (size_t)m * ldo + n;
        *o = EPI == GEMV_ADD_F32 ? *o + acc[r][m] * scale : acc[r][m];
      }
    }
  }
}

// The input of a projection: bf16 rows x, or (xf != nullptr) fp32 rows to be RMS-normalised with gamma / eps.
struct GemvIn {
  const bf16_t* x;
  const float* xf;
  const float* gamma;
  float eps;
  float scale;   // GEMV_ADD_F32: out += scale * C
  int m_valid = 0;   // 0: all M rows of the instantiation exist; otherwise how many do (bf16 input only)
};

template <int M, int EPI, int RW, int U>
void launch_gemv_cfg(const GemvIn& in, const bf16_t* W, void* out, int N, int K, long long ldo, int act, hipStream_t st) {
  const int blocks = (N + 4 * RW - 1) / (4 * RW);
  if (in.xf)
    hipLaunchKernelGGL((gemv_kernel<M, EPI, RW, U, true>), dim3(blocks), dim3(256), (size_t)M * K * 2 + 16 * M, st,
                       in.x, in.xf, in.gamma, in.eps, W, out, N, K, ldo, act, in.scale, M);
  else
    hipLaunchKernelGGL((gemv_kernel<M, EPI, RW, U, false>), dim3(blocks), dim3(256), 0, st, in.x, in.xf, in.gamma,
                       in.eps, W, out, N, K, ldo, act, in.scale, in.m_valid > 0 ? in.m_valid : M);
}

// Rows per wave and unroll depth: few batch rows leave registers for deep unrolling; a small N gets
// two rows per wave so that the launch still has several waves per SIMD.
template <int M, int EPI>
void launch_gemv_me(const GemvIn& x, const bf16_t* W, void* out, int N, int K, long long ldo, int act, hipStream_t st) {
  if (EPI == GEMV_GLU_BF16) {
    if (M <= 2) launch_gemv_cfg<M, EPI, 2, 4>(x, W, out, N, K, ldo, act, st);
    else launch_gemv_cfg<M, EPI, 2, 1>(x, W, out, N, K, ldo, act, st);
  } else if (M <= 2) {
    if (N <= 8192) launch_gemv_cfg<M, EPI, 2, 4>(x, W, out, N, K, ldo, act, st);
    else launch_gemv_cfg<M, EPI, 4, 4>(x, W, out, N, K, ldo, act, st);
  } else if (M <= 4) {
    launch_gemv_cfg<M, EPI, 4, 2>(x, W, out, N, K, ldo, act, st);
  } else {
    launch_gemv_cfg<M, EPI, 4, 1>(x, W, out, N, K, ldo, act, st);
  }
}

template <int M>
void launch_gemv_m(const GemvIn& x, const bf16_t* W, void* out, int N, int K, long long ldo, int epi, int act,
                   hipStream_t st) {
  switch (epi) {
    case GEMV_STORE_F32: launch_gemv_me<M, GEMV_STORE_F32>(x, W, out, N, K, ldo, act, st); break;
    case GEMV_ADD_F32: launch_gemv_me<M, GEMV_ADD_F32>(x, W, out, N, K, ldo, act, st); break;
    default: launch_gemv_me<M, GEMV_GLU_BF16>(x, W, out, N, K, ldo, act, st);
  }
}

// rows m0 .. m0 + mm - 1 of the input
GemvIn rows_from(const GemvIn& in, int m0, int K) {
  GemvIn r = in;
  if (r.xf) r.xf += (size_t)m0 * K;
  else r.x += (size_t)m0 * K;
  return r;
}

void launch_gemv_in(const GemvIn& in, const bf16_t* W, void* out, int M, int N, int K, int64_t ldo, int epilogue,
                    int act, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  // rows are processed in groups of at most 8 (weights are re-streamed per group)
  const size_t osz = epilogue == GEMV_GLU_BF16 ? 2 : 4;
  for (int m0 = 0; m0 < M; m0 += 8) {
    const int mm = M - m0 < 8 ? M - m0 : 8;
    const GemvIn xs = rows_from(in, m0, K);
    void* os = reinterpret_cast<char*>(out) + (size_t)m0 * ldo * osz;
    if (mm == 1) launch_gemv_m<1>(xs, W, os, N, K, ldo, epilogue, act, st);
    else if (mm == 2) launch_gemv_m<2>(xs, W, os, N, K, ldo, epilogue, act, st);
    else if (mm <= 4) {
      // 3 rows: 2 + 1 (exact sizes; padding to 4 would cost registers in the 2-row form's deep unrolling)
      if (mm == 3) { launch_gemv_m<2>(xs, W, os, N, K, ldo, epilogue, act, st);
                     launch_gemv_m<1>(rows_from(xs, 2, K), W, reinterpret_cast<char*>(os) + 2 * ldo * osz, N, K, ldo, epilogue, act, st); }
      else launch_gemv_m<4>(xs, W, os, N, K, ldo, epilogue, act, st);
    } else if (mm == 8 || !xs.xf) {
      // 5..7 rows of bf16 input run the 8-row form with the missing rows repeating the last one (never stored):
      // the weights are streamed once
      GemvIn x8 = xs;
      x8.m_valid = mm;
      launch_gemv_m<8>(x8, W, os, N, K, ldo, epilogue, act, st);
    } else {  // 5..7 fp32 rows to be normalised: 4 + remainder
      launch_gemv_m<4>(xs, W, os, N, K, ldo, epilogue, act, st);
      launch_gemv_in(rows_from(xs, 4, K), W, reinterpret_cast<char*>(os) + 4 * ldo * osz, mm - 4, N, K, ldo, epilogue, act, st);
    }
  }
}

}  // namespace decode_impl
using namespace decode_impl;

void launch_gemv(const bf16_t* x, const bf16_t* W, void* out, int M, int N, int K, int64_t ldo, int epilogue,
                 int act, hipStream_t st, float scale) {
  launch_gemv_in(GemvIn{x, nullptr, nullptr, 0.f, scale, 0}, W, out, M, N, K, ldo, epilogue, act, st);
}

bool gemv_norm_supported(int M, int K) {
  return M >= 1 && M <= 4 && K % 8 == 0 && K <= 8192 && (size_t)M * K * 2 + 16 * M <= 48 * 1024;
}

void launch_gemv_norm(const float* xf, const float* gamma, float eps, const bf16_t* W, void* out, int M, int N, int K,
                      int64_t ldo, int epilogue, int act, hipStream_t st) {
  launch_gemv_in(GemvIn{nullptr, xf, gamma, eps, 1.f, 0}, W, out, M, N, K, ldo, epilogue, act, st);
}

// ------------------------------------------------------------------------------------- RoPE + append
namespace decode_impl {
__global__ __launch_bounds__(128) void rope_append_kernel(const float* __restrict__ qkv, int ld,
                                                          bf16_t* __restrict__ q_out, int n_q_heads,
                                                          int n_kv_heads, int hd, const int32_t* __restrict__ pos,
                                                          const int32_t* __restrict__ slot,
                                                          double neg2_over_hd_log2theta, bf16_t* __restrict__ k_pool,
                                                          bf16_t* __restrict__ v_pool, int P,
                                                          const float* __restrict__ q_gamma,
                                                          const float* __restrict__ k_gamma, float qk_eps,
                                                          int n_parts, size_t part_stride, KvQuant kvq) {
  __shared__ float red[2];
  const int b = blockIdx.x, head = blockIdx.y;
  const int half = hd >> 1;
  const int i = threadIdx.x;
  const float* row = qkv + (size_t)b * ld + (size_t)head * hd;
  const int s = slot[b];
  // per-head QK-norm (uniform over the block): RMS over the head's hd values, before the rotation
  const float* gamma = head < n_q_heads ? q_gamma : (head < n_q_heads + n_kv_heads ? k_gamma : nullptr);
  float x = i < half ? row[i] : 0.f, y = i < half ? row[i + half] : 0.f;
  for (int p = 1; p < n_parts; ++p)
    if (i < half) {
      x += row[p * part_stride + i];
      y += row[p * part_stride + i + half];
    }
  if (gamma) {
    const float ss = wave_sum(x * x + y * y);
    if ((i & 63) == 0) red[i >> 6] = ss;
    __syncthreads();
    const float rstd = 1.0f / sqrtf((red[0] + red[1]) / (float)hd + qk_eps);
    if (i < half) {
      x *= rstd * gamma[i];
      y *= rstd * gamma[i + half];
    }
  }
  if (i >= half) return;
  if (head < n_q_heads + n_kv_heads) {
    const double ang = (double)pos[b] * exp2((double)i * neg2_over_hd_log2theta);
    double sd, cd;
    sincos(ang, &sd, &cd);
    const float c = (float)cd, sn = (float)sd;
    const float rlo = x * c - y * sn, rhi = y * c + x * sn;
    const bf16_t lo = f32_to_bf16(rlo), hi = f32_to_bf16(rhi);
    if (head < n_q_heads) {
      bf16_t* o = q_out + ((size_t)b * n_q_heads + head) * hd;
      o[i] = lo;
      o[i + half] = hi;
    } else {
      const int hh = head - n_q_heads;
      const size_t eoff = (((size_t)(s / P) * n_kv_heads + hh) * P + (s % P)) * hd;
      if (kvq.fp8) {     // one-byte e4m3 codes
        unsigned char* o = reinterpret_cast<unsigned char*>(k_pool) + eoff;
        o[i] = (unsigned char)e4m3_encode(rlo * kvq.k_inv);
        o[i + half] = (unsigned char)e4m3_encode(rhi * kvq.k_inv);
      } else {
        bf16_t* o = k_pool + eoff;
        o[i] = lo;
        o[i + half] = hi;
      }
    }
  } else {
    const int hh = head - n_q_heads - n_kv_heads;
    const size_t eoff = (((size_t)(s / P) * n_kv_heads + hh) * P + (s % P)) * hd;
    if (kvq.fp8) {
      unsigned char* o = reinterpret_cast<unsigned char*>(v_pool) + eoff;
      o[i] = (unsigned char)e4m3_encode(x * kvq.v_inv);
      o[i + half] = (unsigned char)e4m3_encode(y * kvq.v_inv);
    } else {
      bf16_t* o = v_pool + eoff;
      o[i] = f32_to_bf16(x);
      o[i + half] = f32_to_bf16(y);
    }
  }
}
}  // namespace decode_impl
using namespace decode_impl;

void launch_rope_append(const float* qkv, int ld, bf16_t* q_out, int n_q_heads, int n_kv_heads, int hd,
                        const int32_t* pos, const int32_t* slot, double theta, bf16_t* k_pool, bf16_t* v_pool,
                        int page_size, int B, hipStream_t st, const float* q_gamma, const float* k_gamma,
                        float qk_eps, int n_parts, size_t part_stride, KvQuant kvq) {
  if (B <= 0) return;
  hipLaunchKernelGGL(rope_append_kernel, dim3(B, n_q_heads + 2 * n_kv_heads), dim3(128), 0, st, qkv, ld, q_out,
                     n_q_heads, n_kv_heads, hd, pos, slot, -2.0 / (double)hd * log2(theta), k_pool, v_pool,
                     page_size, q_gamma, k_gamma, qk_eps, n_parts, part_stride, kvq);
}

// ------------------------------------------------------------------------------------- decode attention
namespace decode_impl {

constexpr int KCH = kDecodeKeysPerSplit;  // keys per work-group (one split)
constexpr int GMAX = 8;   // query heads per KV head

// grid (n_splits, Hkv, B), 256 threads.  Split s of sequence b covers keys lo + s*KCH .. +KCH-1,
// lo = first visible key (window start, or the first position the layer holds an entry for).  Writes the unnormalised partial output, its max and its sum.
// GT: compile-time bound of the number of query heads per KV head (registers and loops are sized by it).
// FUSED: RoPE + append inside this kernel (a.qkv_raw given); a template parameter because the preparation's registers
// would otherwise halve the occupancy of the plain form as well.
template <int HD, int GT, bool FUSED>
__global__ __launch_bounds__(256) void attn_decode_split_kernel(AttnDecodeArgs a, float scale) {
  constexpr int LPK = HD / 8;        // lanes per key (16-byte chunk each)
  constexpr int KPI = 256 / LPK;     // keys per block iteration
  __shared__ float sc[GT][KCH];
  __shared__ float red[4][GT][HD];  // one partial per wave
  __shared__ float stat[GT][2];

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int P = a.page_size, lgP = __ffs(P) - 1;   // page sizes are powers of two
  const int qpos = a.pos[b];
  int lo = a.window > 0 ? max(0, qpos - a.window + 1) : 0;
  if (a.kv_first) lo = max(lo, min(a.kv_first[b], qpos));   // the query token's own entry always exists
  const int k_first = lo + split * KCH;
  const int n_keys = min(KCH, qpos + 1 - k_first);  // <= 0: this split is empty
  const int tid = threadIdx.x;
  const bool fp8 = a.kvq.fp8 != 0;      // uniform: the pools hold one-byte e4m3 codes
  const int li = tid % LPK, kslot = tid / LPK;
  const int32_t* bt = a.block_table + (size_t)b * a.max_pages;
  float* part = a.part + (((size_t)b * a.n_q_heads + (size_t)kvh * G) * a.n_splits + split) * (HD + 2);
  const size_t part_head_stride = (size_t)a.n_splits * (HD + 2);

  if (n_keys <= 0) {
    for (int i = tid; i < G * (HD + 2); i += 256) {
      const int g = i / (HD + 2), e = i % (HD + 2);
      part[g * part_head_stride + e] = e == HD ? -INFINITY : 0.f;
    }
    return;
  }

  // this thread's K and V chunks of the split are requested up front (one memory round trip), before the query
  // rows are prepared (in the fused mode the slot of the query position is read too, and replaced further down)
  constexpr int NIT = KCH / KPI;
  uint4 kw[NIT], vw[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int kk = kslot + it * KPI;
    kw[it] = make_uint4(0, 0, 0, 0);
    vw[it] = make_uint4(0, 0, 0, 0);
    if (kk < n_keys) {
      const int key = k_first + kk;
      const int page = bt[key >> lgP];
      const size_t off = (((size_t)page * a.n_kv_heads + kvh) * P + (key & (P - 1))) * HD + li * 8;
      if (fp8) {   // 8 one-byte codes per chunk
        const uint2 k8 = *reinterpret_cast<const uint2*>(reinterpret_cast<const unsigned char*>(a.k_pool) + off);
        const uint2 v8 = *reinterpret_cast<const uint2*>(reinterpret_cast<const unsigned char*>(a.v_pool) + off);
        kw[it].x = k8.x; kw[it].y = k8.y;
        vw[it].x = v8.x; vw[it].y = v8.y;
      } else {
        kw[it] = *reinterpret_cast<const uint4*>(a.k_pool + off);
        vw[it] = *reinterpret_cast<const uint4*>(a.v_pool + off);
      }
    }
  }
  // ---- RoPE + append inside this kernel: head rows from the projection's fp32 output
  constexpr bool fused = FUSED;
  constexpr int HALF = HD / 2;
  const bool hi_half = li * 8 >= HALF;          // this thread's 8 dims are the second members of their pairs
  float rc[8], rs[8];                           // (cos, sin) of those pairs
  if constexpr (fused) {
    const float4* csp = reinterpret_cast<const float4*>(a.cs + (size_t)b * HALF + (li * 8) % HALF);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float4 t = csp[e];
      rc[2 * e] = t.x; rs[2 * e] = t.y; rc[2 * e + 1] = t.z; rs[2 * e + 1] = t.w;
    }
  }
  // This thread's 8 values of the head that starts at column `col` of the raw row: parts added, optionally
  // RMS-normalised over the head (its LPK lanes are an aligned group), optionally rotated.  x = own dims, y = the
  // other members of their pairs; first members become x c - y s, second members x c + y s.
  auto head8 = [&](int col, const float* gamma, bool rotate, float* out8) {
    const float* row = a.qkv_raw + (size_t)b * a.ld + col;
    float x[8], y[8];
    {
      const float4 x0 = *reinterpret_cast<const float4*>(row + li * 8), x1 = *reinterpret_cast<const float4*>(row + li * 8 + 4);
      const float4 y0 = *reinterpret_cast<const float4*>(row + ((li * 8) ^ HALF)), y1 = *reinterpret_cast<const float4*>(row + ((li * 8) ^ HALF) + 4);
      x[0] = x0.x; x[1] = x0.y; x[2] = x0.z; x[3] = x0.w; x[4] = x1.x; x[5] = x1.y; x[6] = x1.z; x[7] = x1.w;
      y[0] = y0.x; y[1] = y0.y; y[2] = y0.z; y[3] = y0.w; y[4] = y1.x; y[5] = y1.y; y[6] = y1.z; y[7] = y1.w;
    }
    for (int p = 1; p < a.n_parts; ++p) {
      const float* rp = row + (size_t)p * a.part_stride;
#pragma unroll
      for (int e = 0; e < 8; ++e) { x[e] += rp[li * 8 + e]; y[e] += rp[((li * 8) ^ HALF) + e]; }
    }
    if (gamma) {
      float s2 = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s2 += x[e] * x[e];
      s2 = group_sum<(LPK < 16 ? LPK : 16)>(s2);
      if (LPK > 16) s2 += __shfl_xor(s2, 16, 64);
      const float rstd = 1.0f / sqrtf(s2 / (float)HD + a.qk_eps);
#pragma unroll
      for (int e = 0; e < 8; ++e) { x[e] *= rstd * gamma[li * 8 + e]; y[e] *= rstd * gamma[((li * 8) ^ HALF) + e]; }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e)
      out8[e] = !rotate ? x[e] : (hi_half ? x[e] * rc[e] + y[e] * rs[e] : x[e] * rc[e] - y[e] * rs[e]);
  };

  // ---- scores
  float qv[GT][8];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    if (g < G) {
      if constexpr (fused) {
        head8((kvh * G + g) * HD, a.q_gamma, true, qv[g]);
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[g][e] = bf16_to_f32(f32_to_bf16(qv[g][e]));   // q enters the scores as bf16
      } else {
        const uint4 w = *reinterpret_cast<const uint4*>(a.q + ((size_t)b * a.n_q_heads + kvh * G + g) * HD + li * 8);
        qv[g][0] = bf16lo(w.x); qv[g][1] = bf16hi(w.x); qv[g][2] = bf16lo(w.y); qv[g][3] = bf16hi(w.y);
        qv[g][4] = bf16lo(w.z); qv[g][5] = bf16hi(w.z); qv[g][6] = bf16lo(w.w); qv[g][7] = bf16hi(w.w);
      }
    }
  }
  // The query position's own entry, if its key falls into this split: formed here (every group of lanes computes
  // the same values; the group whose key it is stores them and keeps them in place of a load).
  const int kk_new = qpos - k_first;
  const bool has_new = fused && kk_new >= 0 && kk_new < n_keys;
  uint4 k_new = make_uint4(0, 0, 0, 0), v_new = make_uint4(0, 0, 0, 0);
  if (has_new) {
    float k8[8], v8[8];
    head8((a.n_q_heads + kvh) * HD, a.k_gamma, true, k8);
    head8((a.n_q_heads + a.n_kv_heads + kvh) * HD, nullptr, false, v8);
    if (fp8) {
      k_new.x = e4m3_pack4(k8[0] * a.kvq.k_inv, k8[1] * a.kvq.k_inv, k8[2] * a.kvq.k_inv, k8[3] * a.kvq.k_inv);
      k_new.y = e4m3_pack4(k8[4] * a.kvq.k_inv, k8[5] * a.kvq.k_inv, k8[6] * a.kvq.k_inv, k8[7] * a.kvq.k_inv);
      v_new.x = e4m3_pack4(v8[0] * a.kvq.v_inv, v8[1] * a.kvq.v_inv, v8[2] * a.kvq.v_inv, v8[3] * a.kvq.v_inv);
      v_new.y = e4m3_pack4(v8[4] * a.kvq.v_inv, v8[5] * a.kvq.v_inv, v8[6] * a.kvq.v_inv, v8[7] * a.kvq.v_inv);
    } else {
      k_new = make_uint4(pack_bf16x2(k8[0], k8[1]), pack_bf16x2(k8[2], k8[3]), pack_bf16x2(k8[4], k8[5]), pack_bf16x2(k8[6], k8[7]));
      v_new = make_uint4(pack_bf16x2(v8[0], v8[1]), pack_bf16x2(v8[2], v8[3]), pack_bf16x2(v8[4], v8[5]), pack_bf16x2(v8[6], v8[7]));
    }
  }
  if (has_new) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if (kslot + it * KPI != kk_new) continue;
      // the new entry: stored (the pools are written in this mode) and kept in place of what was loaded
      kw[it] = k_new;
      vw[it] = v_new;
      const int page = bt[qpos >> lgP];
      const size_t off = (((size_t)page * a.n_kv_heads + kvh) * P + (qpos & (P - 1))) * HD + li * 8;
      if (fp8) {
        *reinterpret_cast<uint2*>(reinterpret_cast<unsigned char*>(const_cast<bf16_t*>(a.k_pool)) + off) = make_uint2(k_new.x, k_new.y);
        *reinterpret_cast<uint2*>(reinterpret_cast<unsigned char*>(const_cast<bf16_t*>(a.v_pool)) + off) = make_uint2(v_new.x, v_new.y);
      } else {
        *reinterpret_cast<uint4*>(const_cast<bf16_t*>(a.k_pool) + off) = k_new;
        *reinterpret_cast<uint4*>(const_cast<bf16_t*>(a.v_pool) + off) = v_new;
      }
    }
  }
  // the 8 values of a chunk as floats: bf16 entries, or e4m3 codes times the tensor's scale
  auto unpack8 = [&](const uint4& w, float* f, float scale8) {
    if (fp8) {
      e4m3_decode4_hw(w.x, f);
      e4m3_decode4_hw(w.y, f + 4);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] *= scale8;
    } else {
      f[0] = bf16lo(w.x); f[1] = bf16hi(w.x); f[2] = bf16lo(w.y); f[3] = bf16hi(w.y);
      f[4] = bf16lo(w.z); f[5] = bf16hi(w.z); f[6] = bf16lo(w.w); f[7] = bf16hi(w.w);
    }
  };
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int kk = kslot + it * KPI;
    float s[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g) s[g] = 0.f;
    {
      float kf[8];
      unpack8(kw[it], kf, a.kvq.k_scale);
#pragma unroll
      for (int g = 0; g < GT; ++g)
        if (g < G) {
#pragma unroll
          for (int e = 0; e < 8; ++e) s[g] += qv[g][e] * kf[e];
        }
    }
#pragma unroll
    for (int g = 0; g < GT; ++g)
      if (g < G) {
        // the LPK lanes of a key are an aligned group inside a row of 16 lanes (two rows at head_dim 256)
        s[g] = group_sum<(LPK < 16 ? LPK : 16)>(s[g]);
        if (LPK > 16) s[g] += __shfl_xor(s[g], 16, 64);
        if (li == 0) sc[g][kk] = kk < n_keys ? s[g] * scale : -INFINITY;
      }
  }
  __syncthreads();
  // ---- per-head max and exp-sum (wave w handles heads w, w+4)
  {
    const int w = tid >> 6, lane = tid & 63;
    for (int g = w; g < G; g += 4) {
      float mx = -INFINITY;
      for (int i = lane; i < KCH; i += 64) mx = fmaxf(mx, sc[g][i]);
      mx = wave_max_rows(mx);
      float sum = 0.f;
      for (int i = lane; i < KCH; i += 64) {
        const float pv = __expf(sc[g][i] - mx);
        sc[g][i] = pv;
        sum += pv;
      }
      sum = wave_sum_rows(sum);
      if (lane == 0) { stat[g][0] = mx; stat[g][1] = sum; }
    }
  }
  __syncthreads();
  // ---- partial O = P V : thread owns 8 head-dim values, strides over keys
  float acc[GT][8];
#pragma unroll
  for (int g = 0; g < GT; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int kk = kslot + it * KPI;
    if (kk >= n_keys) continue;
    float vf[8];
    unpack8(vw[it], vf, a.kvq.v_scale);
#pragma unroll
    for (int g = 0; g < GT; ++g)
      if (g < G) {
        const float pv = sc[g][kk];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] += pv * vf[e];
      }
  }
  // Lanes li, li + LPK, ... of a wave hold partial sums of the same head-dim slice.  They are added by a
  // butterfly that halves the number of values a lane carries at every step (a lane sends the half its partner
  // keeps), so the GT * 8 values cost GT * 8 * (1 - LPK / 64) exchanges instead of GT * 8 per step; at the end
  // the lanes of the different rows hold different values, and all of them write.  Then the 4 waves are added.
  {
    constexpr int NV = GT * 8;
    float v[NV];
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) v[g * 8 + e] = acc[g][e];
    const int lane = tid & 63;
    int first = 0;   // index (g * 8 + e) of this lane's v[0]
    auto fold = [&](auto n_c, int o) {
      constexpr int H = decltype(n_c)::value / 2;
      const bool upper = (lane & o) != 0;
#pragma unroll
      for (int i = 0; i < H; ++i) {
        const float send = upper ? v[i] : v[i + H];
        const float keep = upper ? v[i + H] : v[i];
        v[i] = keep + __shfl_xor(send, o, 64);
      }
      if (upper) first += H;
    };
    constexpr int N1 = NV, N2 = LPK <= 32 ? N1 / 2 : N1, N3 = LPK <= 16 ? N2 / 2 : N2, N4 = LPK <= 8 ? N3 / 2 : N3;
    if constexpr (LPK <= 32) fold(std::integral_constant<int, N1>{}, 32);
    if constexpr (LPK <= 16) fold(std::integral_constant<int, N2>{}, 16);
    if constexpr (LPK <= 8) fold(std::integral_constant<int, N3>{}, 8);
    static_assert(N4 >= 1, "a lane keeps at least one value");
#pragma unroll
    for (int i = 0; i < N4; ++i) {
      const int idx = first + i, g = idx >> 3, e = idx & 7;
      if (g < G) red[tid >> 6][g][li * 8 + e] = v[i];
    }
  }
  __syncthreads();
  for (int i = tid; i < G * HD; i += 256) {
    const int g = i / HD, e = i % HD;
    part[g * part_head_stride + e] = (red[0][g][e] + red[1][g][e]) + (red[2][g][e] + red[3][g][e]);
  }
  if (tid < G) {
    part[tid * part_head_stride + HD] = stat[tid][0];
    part[tid * part_head_stride + HD + 1] = stat[tid][1];
  }
}

// grid (B * Hq), 256 threads: thread (grp, i) sums head-dim element i over the splits s = grp, grp + NG, ..
// (NG = 256 / hd groups), the groups are then added in index order: a fixed summation order.
__global__ __launch_bounds__(256) void attn_decode_combine_kernel(const float* __restrict__ part,
                                                                  bf16_t* __restrict__ out, int n_splits, int hd) {
  __shared__ float red_m[4];
  __shared__ float red_num[4][256];
  __shared__ float red_den[4];
  const size_t bh = blockIdx.x;
  const int tid = threadIdx.x;
  const int stride = hd + 2;
  const float* p = part + bh * n_splits * stride;
  float mx = -INFINITY;
  for (int s = tid; s < n_splits; s += 256) mx = fmaxf(mx, p[s * stride + hd]);
  mx = wave_max(mx);
  if ((tid & 63) == 0) red_m[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
  const int ng = 256 / hd, grp = tid / hd, i = tid % hd;
  float num = 0.f, den = 0.f;
#pragma unroll 4
  for (int s = grp; s < n_splits; s += ng) {
    const float m = p[s * stride + hd];
    const float w = m == -INFINITY ? 0.f : __expf(m - mx);
    num += w * p[s * stride + i];
    den += w * p[s * stride + hd + 1];
  }
  red_num[grp][i] = num;
  if (i == 0) red_den[grp] = den;
  __syncthreads();
  if (tid < hd) {
    float n = red_num[0][tid], d = red_den[0];
    for (int g = 1; g < ng; ++g) { n += red_num[g][tid]; d += red_den[g]; }
    out[bh * hd + tid] = f32_to_bf16(d > 0.f ? n / d : 0.f);
  }
}

template <int HD>
void launch_decode_hd(const AttnDecodeArgs& a, hipStream_t st) {
  const float scale = 1.f / sqrtf((float)HD);
  const dim3 grid(a.n_splits, a.n_kv_heads, a.B);
  const int G = a.n_q_heads / a.n_kv_heads;
  auto go = [&](auto fused_c) {
    constexpr bool F = decltype(fused_c)::value;
    if (G <= 1) hipLaunchKernelGGL((attn_decode_split_kernel<HD, 1, F>), grid, dim3(256), 0, st, a, scale);
    else if (G <= 2) hipLaunchKernelGGL((attn_decode_split_kernel<HD, 2, F>), grid, dim3(256), 0, st, a, scale);
    else if (G <= 4) hipLaunchKernelGGL((attn_decode_split_kernel<HD, 4, F>), grid, dim3(256), 0, st, a, scale);
    else hipLaunchKernelGGL((attn_decode_split_kernel<HD, GMAX, F>), grid, dim3(256), 0, st, a, scale);
  };
  if (a.qkv_raw) go(std::true_type{});
  else go(std::false_type{});
  hipLaunchKernelGGL(attn_decode_combine_kernel, dim3(a.B * a.n_q_heads), dim3(256), 0, st, a.part, a.out,
                     a.n_splits, HD);
}
}  // namespace decode_impl
using namespace decode_impl;

// ------------------------------------------------------------------------------------- greedy choice
namespace decode_impl {
// tok[b] = (step > 0 and tok[b] == eos and eos >= 0) ? eos : argmax_v logits[b, v]  (lowest index on ties),
// and out[b * out_stride + step] = tok[b].  One work-group of 1024 threads per sequence.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits, int vocab,
                                                      int32_t* __restrict__ tok, int32_t* __restrict__ out,
                                                      int out_stride, int step, int eos) {
  __shared__ float bv[16];
  __shared__ int bi[16];
  const int b = blockIdx.x, tid = threadIdx.x;
  const float* row = logits + (size_t)b * vocab;
  float best = -INFINITY;
  int idx = 0x7fffffff;
  // A thread sees its elements in ascending order, so the first maximum it meets is the one it keeps.  With a
  // 16-byte aligned row it takes four consecutive logits per load and has four loads in flight (one block per
  // sequence reads half a megabyte: the latency of dependent scalar loads was 39 us at a vocabulary of 128256).
  if ((vocab & 3) == 0 && (reinterpret_cast<uintptr_t>(row) & 15) == 0) {
    const float4* row4 = reinterpret_cast<const float4*>(row);
    const int n4 = vocab >> 2;
    for (int v0 = tid; v0 < n4; v0 += 4 * 1024) {
      float4 x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int v = v0 + u * 1024;
        x[u] = v < n4 ? row4[v] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int v = (v0 + u * 1024) * 4;
        if (x[u].x > best) { best = x[u].x; idx = v; }
        if (x[u].y > best) { best = x[u].y; idx = v + 1; }
        if (x[u].z > best) { best = x[u].z; idx = v + 2; }
        if (x[u].w > best) { best = x[u].w; idx = v + 3; }
      }
    }
  } else {
    for (int v = tid; v < vocab; v += 1024) {
      const float x = row[v];
      if (x > best) { best = x; idx = v; }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(idx, o, 64);
    if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
  }
  if ((tid & 63) == 0) { bv[tid >> 6] = best; bi[tid >> 6] = idx; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 16; ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
    if (idx == 0x7fffffff) idx = 0;   // a row without any finite maximum
    if (step > 0 && eos >= 0 && tok[b] == eos) idx = eos;
    tok[b] = idx;
    out[(size_t)b * out_stride + step] = idx;
  }
}
}  // namespace decode_impl

void launch_argmax(const float* logits, int vocab, int32_t* tok, int32_t* out, int out_stride, int step, int eos,
                   int B, hipStream_t st) {
  if (B <= 0) return;
  hipLaunchKernelGGL(decode_impl::argmax_kernel, dim3(B), dim3(1024), 0, st, logits, vocab, tok, out, out_stride, step,
                     eos);
}

void launch_attention_decode(const AttnDecodeArgs& a, hipStream_t st) {
  if (a.B <= 0) return;
  switch (a.hd) {
    case 64: launch_decode_hd<64>(a, st); break;
    case 128: launch_decode_hd<128>(a, st); break;
    case 256: launch_decode_hd<256>(a, st); break;
  }
}

}  // namespace pop
