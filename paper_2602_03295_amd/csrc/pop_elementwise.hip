// Bandwidth-bound steps of the POP prefill path for gfx950: embedding gather, RMSNorm (the LN of
// Sec. 2.1), the RoPE angle table, and RoPE + KV-cache append (Sec. 2.1, K/V generation and cache
// append; the same kernel serves the independent KV projections of Sec. 3.3).
#include <algorithm>
#include "pop_device.h"
#include "pop_kernels.h"

namespace pop {

// ------------------------------------------------------------------------------------- embed
__global__ __launch_bounds__(256) void embed_kernel(const bf16_t* __restrict__ table,
                                                    const int32_t* __restrict__ tokens,
                                                    const int32_t* __restrict__ row_src,
                                                    const bf16_t* __restrict__ embeds,
                                                    float* __restrict__ h, int d) {
  const int t = blockIdx.x;
  const int src = row_src ? row_src[t] : -1;
  const bf16_t* row = src < 0 ? table + (size_t)tokens[t] * d : embeds + (size_t)src * d;
  float* dst = h + (size_t)t * d;
  for (int i = threadIdx.x * 8; i < d; i += 256 * 8) {
    const uint4 v = *reinterpret_cast<const uint4*>(row + i);
    float4 a = make_float4(bf16lo(v.x), bf16hi(v.x), bf16lo(v.y), bf16hi(v.y));
    float4 b = make_float4(bf16lo(v.z), bf16hi(v.z), bf16lo(v.w), bf16hi(v.w));
    *reinterpret_cast<float4*>(dst + i) = a;
    *reinterpret_cast<float4*>(dst + i + 4) = b;
  }
}

void launch_embed(const bf16_t* table, const int32_t* tokens, const int32_t* row_src,
                  const bf16_t* embeds, float* h, int T, int d, hipStream_t st) {
  if (T <= 0) return;
  hipLaunchKernelGGL(embed_kernel, dim3(T), dim3(256), 0, st, table, tokens, row_src, embeds, h, d);
}

__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ src,
                                                          const int32_t* __restrict__ idx,
                                                          float* __restrict__ dst, int d) {
  const float* s = src + (size_t)idx[blockIdx.x] * d;
  float* o = dst + (size_t)blockIdx.x * d;
  for (int i = threadIdx.x * 4; i < d; i += 256 * 4)
    *reinterpret_cast<float4*>(o + i) = *reinterpret_cast<const float4*>(s + i);
}

void launch_gather_rows(const float* src, const int32_t* idx, float* dst, int rows, int d, hipStream_t st) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(rows), dim3(256), 0, st, src, idx, dst, d);
}

__global__ __launch_bounds__(256) void scatter_rows_kernel(const float* __restrict__ src,
                                                           const int32_t* __restrict__ idx,
                                                           float* __restrict__ dst, int d) {
  const float* s = src + (size_t)blockIdx.x * d;
  float* o = dst + (size_t)idx[blockIdx.x] * d;
  for (int i = threadIdx.x * 4; i < d; i += 256 * 4)
    *reinterpret_cast<float4*>(o + i) = *reinterpret_cast<const float4*>(s + i);
}

void launch_scatter_rows(const float* src, const int32_t* idx, float* dst, int rows, int d, hipStream_t st) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(scatter_rows_kernel, dim3(rows), dim3(256), 0, st, src, idx, dst, d);
}

// ------------------------------------------------------------------------------------- RMSNorm
// One 256-thread block per row; the row stays in registers between the statistics and the scaling
// (up to 8 float4 per thread, d <= 8192), so x is read from HBM once.
constexpr int kNormMaxV = 8;

__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ add1,
                                                      const float* __restrict__ add2, GammaList gammas,
                                                      int n_out, bf16_t* __restrict__ out, size_t out_stride,
                                                      const int32_t* __restrict__ row_idx, int d, float eps) {
  __shared__ float red[4];
  const int t = blockIdx.x;
  const size_t src_row = row_idx ? (size_t)row_idx[t] : (size_t)t;
  float* xr = x + src_row * d;
  float4 v[kNormMaxV];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < kNormMaxV; ++j) {
    const int i = (j * 256 + threadIdx.x) * 4;
    if (i < d) {
      float4 a = *reinterpret_cast<const float4*>(xr + i);
      if (add1) {
        const float4 b = *reinterpret_cast<const float4*>(add1 + src_row * d + i);
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
        if (add2) {
          const float4 c = *reinterpret_cast<const float4*>(add2 + src_row * d + i);
          a.x += c.x; a.y += c.y; a.z += c.z; a.w += c.w;
        }
        *reinterpret_cast<float4*>(xr + i) = a;
      }
      v[j] = a;
      ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
    }
  }
  const float total = block_sum_256(ss, red);
  const float rstd = rsqrtf(total / (float)d + eps);
  for (int o = 0; o < n_out; ++o) {
    const float* g = gammas.g[o];
    bf16_t* orow = out + (size_t)o * out_stride + (size_t)t * d;
#pragma unroll
    for (int j = 0; j < kNormMaxV; ++j) {
      const int i = (j * 256 + threadIdx.x) * 4;
      if (i < d) {
        const float4 gg = *reinterpret_cast<const float4*>(g + i);
        uint2 p;
        p.x = pack_bf16x2(v[j].x * rstd * gg.x, v[j].y * rstd * gg.y);
        p.y = pack_bf16x2(v[j].z * rstd * gg.z, v[j].w * rstd * gg.w);
        *reinterpret_cast<uint2*>(orow + i) = p;
      }
    }
  }
}

void launch_rmsnorm(float* x, const float* add1, const float* add2, const float* gamma, bf16_t* out,
                    const int32_t* row_idx, int rows, int d, float eps, hipStream_t st) {
  if (rows <= 0) return;
  GammaList gl{};
  gl.g[0] = gamma;
  hipLaunchKernelGGL(rmsnorm_kernel, dim3(rows), dim3(256), 0, st, x, add1, add2, gl, 1, out, (size_t)0,
                     row_idx, d, eps);
}

// Same thread layout, summation order and roundings as rmsnorm_kernel; the parts are added in the order of
// splitk_reduce_kernel (parts first, then the old value).
__global__ __launch_bounds__(256) void add_parts_rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ parts,
                                                                int S, size_t part_stride,
                                                                const float* __restrict__ gamma,
                                                                bf16_t* __restrict__ out, int d, float eps,
                                                                float scale) {
  __shared__ float red[4];
  const size_t row = blockIdx.x;
  float* xr = x + row * d;
  float4 v[kNormMaxV];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < kNormMaxV; ++j) {
    const int i = (j * 256 + threadIdx.x) * 4;
    if (i < d) {
      const float* p0 = parts + row * d + i;
      // all parts are requested before the first addition (S <= 8; few blocks run, so latency is what counts)
      float4 q[8];
#pragma unroll
      for (int s = 0; s < 8; ++s)
        if (s < S) q[s] = *reinterpret_cast<const float4*>(p0 + (size_t)s * part_stride);
      const float4 old = *reinterpret_cast<const float4*>(xr + i);
      float4 acc = q[0];
#pragma unroll
      for (int s = 1; s < 8; ++s)
        if (s < S) { acc.x += q[s].x; acc.y += q[s].y; acc.z += q[s].z; acc.w += q[s].w; }
      acc.x = acc.x * scale + old.x; acc.y = acc.y * scale + old.y;
      acc.z = acc.z * scale + old.z; acc.w = acc.w * scale + old.w;
      *reinterpret_cast<float4*>(xr + i) = acc;
      v[j] = acc;
      ss += acc.x * acc.x + acc.y * acc.y + acc.z * acc.z + acc.w * acc.w;
    }
  }
  const float total = block_sum_256(ss, red);
  const float rstd = rsqrtf(total / (float)d + eps);
  bf16_t* orow = out + row * d;
#pragma unroll
  for (int j = 0; j < kNormMaxV; ++j) {
    const int i = (j * 256 + threadIdx.x) * 4;
    if (i < d) {
      const float4 gg = *reinterpret_cast<const float4*>(gamma + i);
      uint2 p;
      p.x = pack_bf16x2(v[j].x * rstd * gg.x, v[j].y * rstd * gg.y);
      p.y = pack_bf16x2(v[j].z * rstd * gg.z, v[j].w * rstd * gg.w);
      *reinterpret_cast<uint2*>(orow + i) = p;
    }
  }
}

void launch_add_parts_rmsnorm(float* x, const float* parts, int S, size_t part_stride, const float* gamma, bf16_t* out,
                              int rows, int d, float eps, hipStream_t st, float scale) {
  if (rows <= 0 || S < 1 || S > 8) return;
  hipLaunchKernelGGL(add_parts_rmsnorm_kernel, dim3(rows), dim3(256), 0, st, x, parts, S, part_stride, gamma, out, d,
                     eps, scale);
}

void launch_rmsnorm_multi(const float* x, GammaList gammas, int n_out, bf16_t* out, size_t out_stride,
                          int rows, int d, float eps, hipStream_t st, const int32_t* row_idx) {
  if (rows <= 0 || n_out <= 0) return;
  hipLaunchKernelGGL(rmsnorm_kernel, dim3(rows), dim3(256), 0, st, const_cast<float*>(x),
                     (const float*)nullptr, (const float*)nullptr, gammas, n_out, out, out_stride,
                     row_idx, d, eps);
}

// ------------------------------------------------------------------------------------- RoPE table
__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t* __restrict__ pos,
                                                         float2* __restrict__ cs, int T, int half,
                                                         double neg2_over_hd_log2theta) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= T * half) return;
  const int t = i / half, f = i - t * half;
  const double inv_freq = exp2((double)f * neg2_over_hd_log2theta);
  const double ang = (double)pos[t] * inv_freq;
  double s, c;
  sincos(ang, &s, &c);
  cs[i] = make_float2((float)c, (float)s);
}

void launch_rope_table(const int32_t* pos, float2* cs, int T, int hd, double theta, hipStream_t st) {
  if (T <= 0) return;
  const int half = hd / 2;
  const int n = T * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, pos, cs, T, half,
                     -2.0 / (double)hd * log2(theta));
}

// ------------------------------------------------------------------------------------- RoPE + cache append
// grid = (tiles of 64 positions, blocks of 1 to 4 q/k heads followed by one block per v head).
//   q head: rotate in place.   k head: rotate in place + store to the K pool.
//   With q_gamma / k_gamma the head is first RMS-normalised over its hd values (per-head QK-norm); the
//   threads that share a head row are neighbouring lanes and add their sums of squares by shuffles.
//   v head: store to the V pool (+ transposed fp16 copy vT[h][i][col], zero beyond the sequence end).
__global__ __launch_bounds__(256) void rope_write_kernel(RopeWriteArgs a, int heads_per_block) {
  __shared__ uint16_t tr[256 * 66];  // [hd][64 + 2] transposed V tile
  const int tile = blockIdx.x;
  const int b = a.tile_seq[tile];
  const int p0 = a.tile_start[tile];
  const int seq0 = a.cu_seqlens[b];
  const int len = a.cu_seqlens[b + 1] - seq0;
  const int hd = a.hd, half = hd >> 1;
  const int nq = a.q_col >= 0 ? a.n_q_heads : 0;
  const int P = a.page_size;
  const int n_rot = nq + a.n_kv_heads;                               // heads that are rotated
  const int n_rot_blocks = (n_rot + heads_per_block - 1) / heads_per_block;

  if ((int)blockIdx.y < n_rot_blocks) {
    // ---- rotate (q or k): a block takes heads_per_block heads of its 64 positions, so that a thread's
    //      cos/sin values (as many bytes as a head's data) are read once for all of them
    const int head0 = blockIdx.y * heads_per_block;
    const int head1 = min(head0 + heads_per_block, n_rot);
    const int groups = half >> 3;  // 8 pairs per work item; 64 * groups is a multiple of 256 for hd >= 64
    for (int it = threadIdx.x; it < 64 * groups; it += 256) {
      const int p = it / groups, g = it - p * groups;
      const bool valid = p0 + p < len;
      const size_t t = (size_t)seq0 + p0 + (valid ? p : 0);
      float2 cs[8];
      {
        const float2* csp = a.cs + t * half + g * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) cs[e] = csp[e];
      }
      const int s = (a.k_pool && valid) ? a.slot[t] : 0;
      for (int head = head0; head < head1; ++head) {
        const bool is_k = head >= nq;
        const int hh = is_k ? head - nq : head;
        const int col = (is_k ? a.k_col : a.q_col) + hh * hd;
        const float* gamma = is_k ? a.k_gamma : a.q_gamma;
        bf16_t* row = a.qkv + t * a.ld + col;
        const uint4 lo = valid ? *reinterpret_cast<const uint4*>(row + g * 8) : make_uint4(0, 0, 0, 0);
        const uint4 hi = valid ? *reinterpret_cast<const uint4*>(row + half + g * 8) : make_uint4(0, 0, 0, 0);
        const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
        float xs[8], ys[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          xs[2 * e] = a.fp16_input ? f16lo(lw[e]) : bf16lo(lw[e]);
          xs[2 * e + 1] = a.fp16_input ? f16hi(lw[e]) : bf16hi(lw[e]);
          ys[2 * e] = a.fp16_input ? f16lo(hw[e]) : bf16lo(hw[e]);
          ys[2 * e + 1] = a.fp16_input ? f16hi(hw[e]) : bf16hi(hw[e]);
        }
        if (gamma) {   // uniform over the block
          float ss = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) ss += xs[e] * xs[e] + ys[e] * ys[e];
          for (int o = groups >> 1; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
          const float rstd = 1.0f / sqrtf(ss / (float)hd + a.qk_eps);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            xs[e] *= rstd * gamma[g * 8 + e];
            ys[e] *= rstd * gamma[half + g * 8 + e];
          }
        }
        if (!valid) continue;
        uint32_t ol[4], oh[4], fl[4], fh[4];
        float rl[8], rh[8];     // rotated low / high halves
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float2 c0 = cs[2 * e], c1 = cs[2 * e + 1];
          const float x0 = xs[2 * e], x1 = xs[2 * e + 1];
          const float y0 = ys[2 * e], y1 = ys[2 * e + 1];
          rl[2 * e] = x0 * c0.x - y0 * c0.y; rl[2 * e + 1] = x1 * c1.x - y1 * c1.y;
          rh[2 * e] = y0 * c0.x + x0 * c0.y; rh[2 * e + 1] = y1 * c1.x + x1 * c1.y;
        }
        const bool q8 = is_k && a.kvq.fp8;     // an 8-bit cache: the key is what its code stands for
        uint2 cl = make_uint2(0, 0), ch = make_uint2(0, 0);
        if (q8) {
          cl.x = e4m3_pack4(rl[0] * a.kvq.k_inv, rl[1] * a.kvq.k_inv, rl[2] * a.kvq.k_inv, rl[3] * a.kvq.k_inv);
          cl.y = e4m3_pack4(rl[4] * a.kvq.k_inv, rl[5] * a.kvq.k_inv, rl[6] * a.kvq.k_inv, rl[7] * a.kvq.k_inv);
          ch.x = e4m3_pack4(rh[0] * a.kvq.k_inv, rh[1] * a.kvq.k_inv, rh[2] * a.kvq.k_inv, rh[3] * a.kvq.k_inv);
          ch.y = e4m3_pack4(rh[4] * a.kvq.k_inv, rh[5] * a.kvq.k_inv, rh[6] * a.kvq.k_inv, rh[7] * a.kvq.k_inv);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            rl[e] = e4m3_decode(((e < 4 ? cl.x : cl.y) >> (8 * (e & 3))) & 0xffu) * a.kvq.k_scale;
            rh[e] = e4m3_decode(((e < 4 ? ch.x : ch.y) >> (8 * (e & 3))) & 0xffu) * a.kvq.k_scale;
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ol[e] = pack_bf16x2(rl[2 * e], rl[2 * e + 1]);
          oh[e] = pack_bf16x2(rh[2 * e], rh[2 * e + 1]);
          fl[e] = pack_f16x2(rl[2 * e], rl[2 * e + 1]);
          fh[e] = pack_f16x2(rh[2 * e], rh[2 * e + 1]);
        }
        const uint4 vlo = make_uint4(ol[0], ol[1], ol[2], ol[3]);
        const uint4 vhi = make_uint4(oh[0], oh[1], oh[2], oh[3]);
        // in place: fp16 when the attention kernel is the consumer (three more mantissa bits than bf16
        // for the score contraction), bf16 otherwise; the cache entry is bf16 or an e4m3 code
        if (!a.cache_only) {
          *reinterpret_cast<uint4*>(row + g * 8) = a.fp16_inplace ? make_uint4(fl[0], fl[1], fl[2], fl[3]) : vlo;
          *reinterpret_cast<uint4*>(row + half + g * 8) = a.fp16_inplace ? make_uint4(fh[0], fh[1], fh[2], fh[3]) : vhi;
        }
        if (is_k && a.k_pool) {
          const size_t eoff = (((size_t)(s / P) * a.n_kv_heads + hh) * P + (s % P)) * hd;
          if (a.kvq.fp8) {
            unsigned char* dst = reinterpret_cast<unsigned char*>(a.k_pool) + eoff;
            *reinterpret_cast<uint2*>(dst + g * 8) = cl;
            *reinterpret_cast<uint2*>(dst + half + g * 8) = ch;
          } else {
            bf16_t* dst = a.k_pool + eoff;
            *reinterpret_cast<uint4*>(dst + g * 8) = vlo;
            *reinterpret_cast<uint4*>(dst + half + g * 8) = vhi;
          }
        }
      }
    }
    return;
  }
  // ---- v head
  const int hh = blockIdx.y - n_rot_blocks;
  const int col = a.v_col + hh * hd;
  const int groups = hd >> 3;
  for (int it = threadIdx.x; it < 64 * groups; it += 256) {
    const int p = it / groups, g = it - p * groups;
    uint4 v = make_uint4(0, 0, 0, 0);
    bool v_is_f16 = a.fp16_input != 0;     // format of the 8 values in v (fp16 or bf16)
    if (p0 + p < len) {
      const size_t t = (size_t)seq0 + p0 + p;
      v = *reinterpret_cast<const uint4*>(a.qkv + t * a.ld + col + g * 8);
      if (a.kvq.fp8) {
        // 8-bit cache: store the codes; what the attention kernel reads (vT) are the values they stand for
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        float f[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          f[2 * e] = (a.fp16_input ? f16lo(w[e]) : bf16lo(w[e])) * a.kvq.v_inv;
          f[2 * e + 1] = (a.fp16_input ? f16hi(w[e]) : bf16hi(w[e])) * a.kvq.v_inv;
        }
        uint2 c;
        c.x = e4m3_pack4(f[0], f[1], f[2], f[3]);
        c.y = e4m3_pack4(f[4], f[5], f[6], f[7]);
        if (a.v_pool) {
          const int s = a.slot[t];
          unsigned char* dst = reinterpret_cast<unsigned char*>(a.v_pool) +
                               (((size_t)(s / P) * a.n_kv_heads + hh) * P + (s % P)) * hd;
          *reinterpret_cast<uint2*>(dst + g * 8) = c;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = e4m3_decode(((e < 4 ? c.x : c.y) >> (8 * (e & 3))) & 0xffu) * a.kvq.v_scale;
        v = make_uint4(pack_f16x2(f[0], f[1]), pack_f16x2(f[2], f[3]), pack_f16x2(f[4], f[5]), pack_f16x2(f[6], f[7]));
        v_is_f16 = true;
      } else if (a.v_pool) {
        const int s = a.slot[t];
        bf16_t* dst = a.v_pool + (((size_t)(s / P) * a.n_kv_heads + hh) * P + (s % P)) * hd;
        uint4 vb = v;   // the cache entry is bf16
        if (a.fp16_input) {
          vb.x = pack_bf16x2(f16lo(v.x), f16hi(v.x)); vb.y = pack_bf16x2(f16lo(v.y), f16hi(v.y));
          vb.z = pack_bf16x2(f16lo(v.z), f16hi(v.z)); vb.w = pack_bf16x2(f16lo(v.w), f16hi(v.w));
        }
        *reinterpret_cast<uint4*>(dst + g * 8) = vb;
      }
    }
    if (a.vT) {
      // the transposed copy is fp16 (bf16 -> fp16 is exact inside fp16's range; saturates outside)
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        tr[(g * 8 + 2 * e) * 66 + p] = v_is_f16 ? (uint16_t)(w[e] & 0xffff) : f32_to_f16_sat(bf16lo(w[e]));
        tr[(g * 8 + 2 * e + 1) * 66 + p] = v_is_f16 ? (uint16_t)(w[e] >> 16) : f32_to_f16_sat(bf16hi(w[e]));
      }
    }
  }
  if (!a.vT) return;
  __syncthreads();
  const size_t colbase = (size_t)a.vt_off[b] + p0;
  for (int it = threadIdx.x; it < hd * 8; it += 256) {
    const int i = it >> 3, c = it & 7;
    const uint16_t* s = tr + i * 66 + c * 8;
    uint4 o;
    o.x = s[0] | ((uint32_t)s[1] << 16);
    o.y = s[2] | ((uint32_t)s[3] << 16);
    o.z = s[4] | ((uint32_t)s[5] << 16);
    o.w = s[6] | ((uint32_t)s[7] << 16);
    *reinterpret_cast<uint4*>(a.vT + ((size_t)hh * hd + i) * a.Tp + colbase + c * 8) = o;
  }
}

void launch_rope_write(const RopeWriteArgs& a, hipStream_t st) {
  if (a.n_tiles <= 0) return;
  const int nq = a.q_col >= 0 ? a.n_q_heads : 0;
  // several heads per block as long as about 512 blocks remain (two per CU): measured at 2048 tokens of the
  // Llama-3.1-8B shape (1280 head tiles): 19.4 us with one head per block, 17.5 us with two, 21.4 us with four
  const int n_rot = nq + a.n_kv_heads;
  const int hpb = std::max(1, std::min(4, (int)((long long)a.n_tiles * n_rot / 512)));
  const int n_rot_blocks = (n_rot + hpb - 1) / hpb;
  hipLaunchKernelGGL(rope_write_kernel, dim3(a.n_tiles, n_rot_blocks + a.n_kv_heads), dim3(256), 0, st, a, hpb);
}

}  // namespace pop
