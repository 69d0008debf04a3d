// Causal grouped-query flash attention for the prompt body (the Attn block of Sec. 2.1 applied to
// all body rows of a kept layer at once), packed variable-length sequences, optional sliding window.
//
// One work-group = one or two tiles of 128 query rows of one query head (a late tile paired with an
// early one, which balances the causal triangle); 4 waves x 32 rows.  Keys/values stream through
// LDS in tiles of 64, staged with buffer_load ... lds and double buffered.
//
// Inside this kernel Q, K, V and P are fp16 (the RoPE/append kernel hands over fp16 copies; the cache
// itself stays bf16): with random-like V the softmax average shrinks signal and rounding noise alike, so
// the relative error of the output equals that of the individual probabilities, and bf16's 8-bit
// mantissa in q, k and P was the largest error source of a whole layer.  P <= 1 and saturating
// conversions keep fp16's range safe.
//
// MFMA arrangement (v_mfma_f32_32x32x16_f16, D = A * B with A rows / B columns spread over lanes):
//   S^T = K * Q^T   : A = K tile rows (keys), B = Q rows.  A lane then owns ONE query row (lane & 31)
//                     and 16 keys per 32-key block, so the softmax row reductions are in-lane plus a
//                     single exchange with lane ^ 32.
//   O^T = V^T * P^T : A = rows of the pre-transposed V (head-dim index), B = P^T.  The S^T
//                     accumulator registers 8G..8G+7 of a block are exactly the B operand of the
//                     G-th 16-key step, because the keys are fed to the first MFMA in the permuted
//                     order key(i) below; no cross-lane data movement is needed for P.
// Softmax is computed in fp32 with exp2 and running max / sum (online softmax); P is rounded to fp16
// for the second MFMA, O accumulates in fp32.
#include "pop_device.h"
#include "pop_kernels.h"

namespace pop {

namespace attn_impl {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
constexpr int BQ = 128;   // query rows per work-group
constexpr int BKV = 64;   // keys per LDS stage

// MFMA row i (0..31) of the S^T block is fed key row key_of_row(i) of the 32-key block, chosen so
// that accumulator registers 8G..8G+7 of lane-half h hold keys 16G + 8h + (0..7).
__device__ __forceinline__ int key_of_row(int i) {
  const int a = i >> 3, hb = (i >> 2) & 1, r = i & 3;
  return 16 * (a >> 1) + 8 * hb + 4 * (a & 1) + r;
}
// LDS swizzle of the K tile.  gfx950 serves a ds_read_b128 sixteen lanes (256 B = all 64 banks) per
// cycle, and the sixteen lanes of a phase read the sixteen rows of an aligned group (key_of_row
// permutes inside such a group).  Rows of >= 256 B each fill whole bank lines, so the sixteen rows need
// sixteen different chunk positions: key = row & 15.  128-byte rows (head_dim 64) share a bank line in
// pairs: key = (row >> 1) & 7 (the row's parity already selects the half line).
template <int ROW_BYTES>
__device__ __forceinline__ int k_swz(int row) {
  return ROW_BYTES >= 256 ? (row & 15) : ((row >> 1) & 7);
}

template <int HD>
__global__ __launch_bounds__(256) void attn_prefill_kernel(AttnPrefillArgs a, float scale_log2) {
#if defined(__HIP_DEVICE_COMPILE__)  // the buffer-resource builtins exist in the device pass only
  constexpr int KS = HD / 16;            // MFMA steps over the head dim for S
  constexpr int OB = HD / 32;            // 32-row blocks of O^T
  constexpr int K_ROW_BYTES = HD * 2;
  constexpr int K_CPR = HD / 8;          // 16-byte chunks per K row
  constexpr int K_RPL = 64 / K_CPR;      // K rows per wave-load
  constexpr int K_BYTES = BKV * K_ROW_BYTES;
  constexpr int V_BYTES = HD * BKV * 2;  // V^T tile: HD rows of 64 keys (128 B)
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int K_LOADS = K_BYTES / 1024 / 4, V_LOADS = V_BYTES / 1024 / 4;  // per wave

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tile = blockIdx.x;
  const int head = blockIdx.y;
  const int kvh = head / (a.n_q_heads / a.n_kv_heads);
  const int b = a.tile_seq[tile];
  const int seq0 = a.cu_seqlens[b];
  const int len = a.cu_seqlens[b + 1] - seq0;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = lane >> 5;
  // one or two query tiles per work-group (a late and an early tile of the same sequence)
  for (int part = 0; part < 2; ++part) {
  const int q0 = part == 0 ? a.tile_start[tile] : a.tile_start2[tile];
  if (q0 < 0) break;
  if (part == 1) __builtin_amdgcn_s_barrier();  // everyone is done with the first tile's LDS stages
  const int qrow = q0 + wave * 32 + (lane & 31);  // position of this lane's query row
  const bool qvalid = qrow < len;

  // ---- key range of this query tile
  const int q_last = min(q0 + BQ, len) - 1;
  int j_begin = 0;
  if (a.window > 0) j_begin = max(0, q0 - a.window + 1) & ~(BKV - 1);
  const int j_end = q_last + 1;  // exclusive
  const int n_kv = (j_end - j_begin + BKV - 1) / BKV;

  // ---- buffer descriptors
  const __amdgpu_buffer_rsrc_t rK = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(a.qkv), 0, (uint32_t)((long long)a.T * a.ld * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rV = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(a.vT), 0, (uint32_t)((long long)a.n_kv_heads * HD * a.Tp * 2), 0x00020000);

  // staging offsets (K: rows = keys; V^T: rows = head-dim index)
  uint32_t offK[K_LOADS], offV[V_LOADS];
#pragma unroll
  for (int j = 0; j < K_LOADS; ++j) {
    const int row = (j * 4 + wave) * K_RPL + lane / K_CPR;
    const int pchunk = lane % K_CPR;
    const int c = pchunk ^ k_swz<K_ROW_BYTES>(row);
    offK[j] = (uint32_t)((((long long)seq0 + row) * a.ld + a.k_col + kvh * HD + c * 8) * 2);
  }
#pragma unroll
  for (int j = 0; j < V_LOADS; ++j) {
    const int row = (j * 4 + wave) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    offV[j] = (uint32_t)((((long long)kvh * HD + row) * a.Tp + a.vt_off[b] + c * 8) * 2);
  }
  // The key offset goes into the per-lane offset (not the scalar one) so that rows beyond the end of
  // the buffer are range-checked and read as zero.
  auto issue = [&](int it, int stage) {
    const int j0 = j_begin + it * BKV;
    unsigned char* sk = smem + stage * STAGE;
    unsigned char* sv = sk + K_BYTES;
#pragma unroll
    for (int j = 0; j < K_LOADS; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rK, (lds_ptr_t)(sk + (j * 4 + wave) * 1024), 16,
                                               offK[j] + (uint32_t)(j0 * a.ld * 2), 0, 0, 0);
#pragma unroll
    for (int j = 0; j < V_LOADS; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rV, (lds_ptr_t)(sv + (j * 4 + wave) * 1024), 16,
                                               offV[j] + (uint32_t)(j0 * 2), 0, 0, 0);
  };

  // ---- Q fragments (B operand: lane = query row, 8 consecutive head-dim values per step)
  f16x8_t qf[KS];
  {
    const bf16_t* qp = a.qkv + ((long long)seq0 + (qvalid ? qrow : 0)) * a.ld + a.q_col + head * HD + h * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const f16x8_t*>(qp + ks * 16);
  }

  floatx16_t o[OB];
#pragma unroll
  for (int i = 0; i < OB; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // LDS fragment addresses
  const int krow = key_of_row(lane & 31);
  const int k_frag = krow * K_ROW_BYTES;
  const int k_sw = k_swz<K_ROW_BYTES>(krow);  // same for krow + 32 (only bits 0..3 of the row are used)
  const int v_frag = (lane & 31) * 128;
  const int v_sw = ((lane & 31) >> 1) & 7;

  const int wave_last = q0 + wave * 32 + 31;  // last query position this wave owns

  if (n_kv > 0) issue(0, 0);
  for (int it = 0; it < n_kv; ++it) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (it + 1 < n_kv) issue(it + 1, (it + 1) & 1);
    const int j0 = j_begin + it * BKV;
    if (j0 > wave_last) continue;  // tile entirely above this wave's diagonal (uniform per wave)
    if (a.window > 0 && j0 + BKV - 1 < q0 + wave * 32 - a.window + 1) continue;  // entirely outside the window
    const unsigned char* sk = smem + (it & 1) * STAGE;
    const unsigned char* sv = sk + K_BYTES;

    // ---- S^T = K Q^T for 2 blocks of 32 keys
    floatx16_t s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int pc = ((2 * ks + h) ^ k_sw) * 16;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const f16x8_t kf = *reinterpret_cast<const f16x8_t*>(sk + k_frag + kb * 32 * K_ROW_BYTES + pc);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[ks], s[kb], 0, 0, 0);
      }
    }
    // register v of block kb on lane-half h holds key j0 + kb*32 + 16*(v/8) + 8*h + (v%8)
    const bool need_mask = (j0 + BKV - 1 > q0 + wave * 32) || (a.window > 0 && j0 < wave_last - a.window + 1);
    if (need_mask) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = j0 + kb * 32 + 16 * (v >> 3) + 8 * h + (v & 7);
          bool ok = key <= qrow;
          if (a.window > 0) ok = ok && (key > qrow - a.window);
          if (!ok) s[kb][v] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * scale_log2);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);  // m_run = -inf -> 0
    float psum = 0.f;
    f16x8_t pf[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pv = __builtin_amdgcn_exp2f(s[kb][g * 8 + e] * scale_log2 - m_use);
          psum += pv;
          pf[kb][g][e] = static_cast<_Float16>(pv);
        }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {  // the running max moved for some row of this wave
#pragma unroll
      for (int i = 0; i < OB; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] *= alpha;
    }
    // ---- O^T += V^T P^T
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int pc = ((4 * kb + 2 * g + h) ^ v_sw) * 16;
#pragma unroll
        for (int i = 0; i < OB; ++i) {
          const f16x8_t vf = *reinterpret_cast<const f16x8_t*>(sv + v_frag + i * 32 * 128 + pc);
          o[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[kb][g], o[i], 0, 0, 0);
        }
      }
  }

  // ---- normalise and store: lane owns query row qrow, head-dim i*32 + (v/4)*8 + 4h + v%4
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (!qvalid) continue;
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  bf16_t* op = a.out + ((long long)seq0 + qrow) * ((long long)a.n_q_heads * HD) + head * HD;
#pragma unroll
  for (int i = 0; i < OB; ++i)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 pk;
      pk.x = pack_bf16x2(o[i][g * 4 + 0] * inv, o[i][g * 4 + 1] * inv);
      pk.y = pack_bf16x2(o[i][g * 4 + 2] * inv, o[i][g * 4 + 3] * inv);
      *reinterpret_cast<uint2*>(op + i * 32 + g * 8 + h * 4) = pk;
    }
  }  // part
#endif
}

template <int HD>
hipError_t launch_hd(const AttnPrefillArgs& a, hipStream_t st) {
  constexpr int smem = 2 * (BKV * HD * 2 + HD * BKV * 2);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_prefill_kernel<HD>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
  hipLaunchKernelGGL((attn_prefill_kernel<HD>), dim3(a.n_tiles, a.n_q_heads), dim3(256), smem, st, a, scale_log2);
  return hipGetLastError();
}

}  // namespace attn_impl
using namespace attn_impl;

hipError_t launch_attention_prefill(const AttnPrefillArgs& a, hipStream_t st) {
  if (a.n_tiles <= 0) return hipSuccess;
  if ((long long)a.T * a.ld * 2 >= (1LL << 31) || (long long)a.n_kv_heads * a.hd * a.Tp * 2 >= (1LL << 31))
    return hipErrorInvalidValue;
  switch (a.hd) {
    case 64: return launch_hd<64>(a, st);
    case 128: return launch_hd<128>(a, st);
    case 256: return launch_hd<256>(a, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace pop
