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
#include <type_traits>

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
  constexpr int NST = HD <= 128 ? 3 : 2;   // LDS ring: K and V^T tiles are requested NST-1 iterations ahead
  constexpr int DPF = NST - 1;
  constexpr uint32_t kOOB = 0x80000000u;   // pushes a byte offset out of range: the lane stages zeros
  constexpr int K_LOADS = K_BYTES / 1024 / 4, V_LOADS = V_BYTES / 1024 / 4;  // per wave
  constexpr int LPI = K_LOADS + V_LOADS;   // wave-loads per iteration

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
  // Key tile `it` of this query tile goes to ring slot it % NST.  Tiles beyond the key range are
  // requested with every lane out of range (zeros are staged), so that each iteration issues the same
  // number of loads and the vmcnt bookkeeping below stays uniform.
  auto issue_k1 = [&](int j, int it) {
    const int j0 = j_begin + it * BKV;
    unsigned char* sk = smem + (it % NST) * STAGE;
    const uint32_t mask = it < n_kv ? 0u : kOOB;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rK, (lds_ptr_t)(sk + (j * 4 + wave) * 1024), 16,
                                             (offK[j] + (uint32_t)(j0 * a.ld * 2)) | mask, 0, 0, 0);
  };
  auto issue_v1 = [&](int j, int it) {
    const int j0 = j_begin + it * BKV;
    unsigned char* sv = smem + (it % NST) * STAGE + K_BYTES;
    const uint32_t mask = it < n_kv ? 0u : kOOB;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rV, (lds_ptr_t)(sv + (j * 4 + wave) * 1024), 16,
                                             (offV[j] + (uint32_t)(j0 * 2)) | mask, 0, 0, 0);
  };
  auto issue_k = [&](int it) {
#pragma unroll
    for (int j = 0; j < K_LOADS; ++j) issue_k1(j, it);
  };
  auto issue_v = [&](int it) {
#pragma unroll
    for (int j = 0; j < V_LOADS; ++j) issue_v1(j, it);
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

  const int wave_first = q0 + wave * 32;       // first / last query position this wave owns
  const int wave_last = wave_first + 31;

  // The key loop is software pipelined so that the matrix pipe and the vector ALU work at the same
  // time inside one wave: iteration t runs the softmax of key tile t on the vector ALU and, sprinkled
  // between its instructions, the MFMAs of O^T += V^T P^T for tile t-1 and of S^T = K Q^T for tile
  // t+1.  The MFMAs of an iteration are cut into 32 slots, one per exponential.  LDS stage (t+1)&1
  // holds K of tile t+1 and V^T of tile t-1 during iteration t; K of tile t+2 and V^T of tile t are
  // requested at its start into the other stage, whose contents were consumed in iteration t-1.
  constexpr int PVN = 4 * OB;          // MFMAs of one O update, index (kb*2+g)*OB + i
  constexpr int SN = 2 * KS;           // MFMAs of one S tile, index ks*2 + kb
  constexpr int NM = PVN + SN;
  constexpr int DIST = 4;              // fragment reads run this many MFMAs ahead
  constexpr bool UNROLL2 = HD <= 128;  // head_dim 256 has no registers to spare for the unrolled form
  // S^T of tile t lives in sbuf[t & 1] and the packed fp16 P^T of tile t in pbuf[t & 1]; the loop is
  // unrolled by two so that these indices are compile-time constants (no register copies).
  floatx16_t sbuf[2][2];
  uint32_t pbuf[2][2][2][4];
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
  typedef float float2_t __attribute__((ext_vector_type(2)));
  const floatx16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // mask of a diagonal / window-edge tile: register v of block kb on lane-half h holds key
  // j0 + kb*32 + 16*(v/8) + 8*h + (v%8)
  auto mask_tile = [&](floatx16_t(&sv_)[2], int j0) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = j0 + kb * 32 + 16 * (v >> 3) + 8 * h + (v & 7);
        bool ok = key <= qrow;
        if (a.window > 0) ok = ok && (key > qrow - a.window);
        if (!ok) sv_[kb][v] = -INFINITY;
      }
  };
  auto tile_needs_mask = [&](int j0) {
    return (j0 + BKV - 1 > wave_first) || (a.window > 0 && j0 < wave_last - a.window + 1);
  };
  // row maximum of the tile the next iteration works on: this lane's half (mx_part) and the other
  // half of the row (mx_other, lane ^ 32, fetched through the LDS crossbar)
  float mx_part = -INFINITY, mx_other = -INFINITY;

  auto body = [&](int t, auto par_c, auto has_pv_c, auto has_s_c) {
    constexpr int PAR = decltype(par_c)::value;   // t & 1
    constexpr bool HAS_PV = decltype(has_pv_c)::value, HAS_S = decltype(has_s_c)::value;
    floatx16_t(&s_cur)[2] = sbuf[PAR];
    floatx16_t(&s_next)[2] = sbuf[PAR ^ 1];
    uint32_t(&pw)[2][2][4] = pbuf[PAR];
    uint32_t(&pw_prev)[2][2][4] = pbuf[PAR ^ 1];
    // MFMAs of this iteration in issue order: S^T of tile t+1 (slots 0..15), then the O update with
    // tile t-1 (slots 16..31).  Once S^T is complete its row maximum is formed in the later slots, so
    // the next iteration starts its exponentials at once.
    constexpr int NS = HAS_S ? SN : 0, NP = HAS_PV ? PVN : 0, CNT = NS + NP;
    // K of tile t+1 and V^T of tile t-1 were requested DPF iterations ago; the loads of the
    // iterations in between may still be in flight (loads return in order).
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DPF - 1) * LPI) : "memory");
    __builtin_amdgcn_s_barrier();
    const unsigned char* sk = smem + ((t + 1) % NST) * STAGE;
    const unsigned char* sv = smem + ((t + NST - 1) % NST) * STAGE + K_BYTES;
    const int tk = t + 1 + DPF, tv = t - 1 + DPF;   // tiles requested during this iteration

    f16x8_t fr[SN + PVN];
    auto frag_read = [&](int n) {          // n-th MFMA of this iteration
      if (n < NS) {
        const int ks = n / 2, kb = n % 2;
        const int pc = ((2 * ks + h) ^ k_sw) * 16;
        fr[n] = *reinterpret_cast<const f16x8_t*>(sk + k_frag + kb * 32 * K_ROW_BYTES + pc);
      } else {
        const int idx = n - NS;
        const int kb = idx / (2 * OB), g = (idx / OB) % 2, i = idx % OB;
        const int pc = ((4 * kb + 2 * g + h) ^ v_sw) * 16;
        fr[n] = *reinterpret_cast<const f16x8_t*>(sv + v_frag + i * 32 * 128 + pc);
      }
    };
    auto do_mfma = [&](int n) {
      if (n < NS) {
        const int ks = n / 2, kb = n % 2;
        s_next[kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fr[n], qf[ks], ks == 0 ? zero16 : s_next[kb], 0, 0, 0);
      } else {
        const int idx = n - NS;
        const int kb = idx / (2 * OB), g = (idx / OB) % 2, i = idx % OB;
        const uint4 w4 = make_uint4(pw_prev[kb][g][0], pw_prev[kb][g][1], pw_prev[kb][g][2], pw_prev[kb][g][3]);
        o[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fr[n], __builtin_bit_cast(f16x8_t, w4), o[i], 0, 0, 0);
      }
    };
    auto first_of = [](int slot) {   // MFMAs issued before `slot`
      const int s1 = slot < 16 ? slot : 16, s2 = slot < 16 ? 0 : slot - 16;
      return s1 * NS / 16 + s2 * NP / 16;
    };
#pragma unroll
    for (int n = 0; n < DIST && n < CNT; ++n) frag_read(n);

    const float mx = fmaxf(mx_part, mx_other);
    const float m_new = fmaxf(m_run, mx * scale_log2);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);  // m_run = -inf -> 0
    float psum = 0.f;
    // the exponentials are skewed over the slots (argument two slots ahead, exp one slot ahead, sum
    // and packing in the slot itself) so that consecutive vector instructions do not wait on each other
    float xa[32], ea[32];
    xa[0] = s_cur[0][0] * scale_log2 - m_use;
    xa[1] = s_cur[0][1] * scale_log2 - m_use;
    ea[0] = __builtin_amdgcn_exp2f(xa[0]);
    float mxa = -INFINITY, mxb = -INFINITY;   // two chains of the next tile's row maximum
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int slot = 0; slot < 32; ++slot) {
      const int lo = first_of(slot), hi = first_of(slot + 1);
#pragma unroll
      for (int n = lo + DIST; n < hi + DIST; ++n)
        if (n < CNT) frag_read(n);
      if (slot % (32 / LPI) == 0) {   // one global load every few slots
        const int q = slot / (32 / LPI);
        if (q < K_LOADS) issue_k1(q, tk);
        else issue_v1(q - K_LOADS, tv);
      }
      if (slot + 2 < 32) {
        xa[slot + 2] = s_cur[(slot + 2) >> 4][(slot + 2) & 15] * scale_log2 - m_use;
        asm volatile("" : "+v"(xa[slot + 2]));
      }
      if (slot + 1 < 32) {
        ea[slot + 1] = __builtin_amdgcn_exp2f(xa[slot + 1]);
        asm volatile("" : "+v"(ea[slot + 1]));
      }
      {
        const int kb = slot >> 4, v = slot & 15;
        psum += ea[slot];
        if (v & 1) {
          // 0 <= P <= 1: plain round-to-nearest packing, no saturation needed
          const float2_t pp = {ea[slot - 1], ea[slot]};
          pw[kb][v >> 3][(v & 7) >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, half2_t));
          // keep the softmax arithmetic inside its slot (otherwise it is sunk below the loop's
          // last branch, behind all MFMAs, and nothing overlaps)
          asm volatile("" : "+v"(pw[kb][v >> 3][(v & 7) >> 1]), "+v"(psum));
        } else {
          asm volatile("" : "+v"(psum));
        }
      }
      if (HAS_S) {
        if (slot == 18) {
          const int j0n = j_begin + (t + 1) * BKV;
          if (tile_needs_mask(j0n)) mask_tile(s_next, j0n);
        }
        if (slot >= 20 && slot < 28) {   // 4 values per slot, two independent chains
          const int kb = (slot - 20) >> 2, v0 = ((slot - 20) & 3) * 4;
          mxa = fmaxf(fmaxf(mxa, s_next[kb][v0]), s_next[kb][v0 + 1]);
          mxb = fmaxf(fmaxf(mxb, s_next[kb][v0 + 2]), s_next[kb][v0 + 3]);
          asm volatile("" : "+v"(mxa), "+v"(mxb));
        }
        if (slot == 28) {
          mx_part = fmaxf(mxa, mxb);
          mx_other = __shfl_xor(mx_part, 32, 64);
        }
      }
#pragma unroll
      for (int n = lo; n < hi; ++n) do_mfma(n);
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {  // the running max moved for some row of this wave
#pragma unroll
      for (int i = 0; i < OB; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] *= alpha;
    }
    if (!UNROLL2) {   // single-parity form: move the results to where the next iteration expects them
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        if (HAS_S) s_cur[kb] = s_next[kb];
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) pw_prev[kb][g][e] = pw[kb][g][e];
      }
    }
  };
  using std::true_type;
  using std::false_type;

  if (n_kv > 0) {
    // prologue: request K of tiles 0..DPF and V^T of tiles 0..DPF-2, then S of tile 0
    issue_k(0);
#pragma unroll
    for (int i = 1; i <= DPF; ++i) issue_k(i);
#pragma unroll
    for (int i = 0; i <= DPF - 2; ++i) issue_v(i);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(DPF * K_LOADS + (DPF - 1) * V_LOADS) : "memory");
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int pc = ((2 * ks + h) ^ k_sw) * 16;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const f16x8_t kf = *reinterpret_cast<const f16x8_t*>(smem + k_frag + kb * 32 * K_ROW_BYTES + pc);
        sbuf[0][kb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[ks], ks == 0 ? zero16 : sbuf[0][kb], 0, 0, 0);
      }
    }
    if (tile_needs_mask(j_begin)) mask_tile(sbuf[0], j_begin);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx_part = fmaxf(mx_part, sbuf[0][kb][v]);
    mx_other = __shfl_xor(mx_part, 32, 64);
    // O update of the last tile (all remaining loads are masked ones; drain them before the ring is reused)
    auto last_pv = [&](auto par_c) {
      constexpr int PAR = decltype(par_c)::value;
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      const unsigned char* sv = smem + ((n_kv - 1) % NST) * STAGE + K_BYTES;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          const int pc = ((4 * kb + 2 * g + h) ^ v_sw) * 16;
          const uint4 w4 = make_uint4(pbuf[PAR][kb][g][0], pbuf[PAR][kb][g][1], pbuf[PAR][kb][g][2], pbuf[PAR][kb][g][3]);
#pragma unroll
          for (int i = 0; i < OB; ++i) {
            const f16x8_t vf = *reinterpret_cast<const f16x8_t*>(sv + v_frag + i * 32 * 128 + pc);
            o[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, __builtin_bit_cast(f16x8_t, w4), o[i], 0, 0, 0);
          }
        }
    };
    typedef std::integral_constant<int, 0> P0;
    typedef std::integral_constant<int, 1> P1;
    if (n_kv == 1) {
      body(0, P0{}, false_type{}, false_type{});
      if (UNROLL2) last_pv(P0{});
      else last_pv(P1{});
    } else if (!UNROLL2) {
      body(0, P0{}, false_type{}, true_type{});
      for (int t = 1; t < n_kv - 1; ++t) body(t, P0{}, true_type{}, true_type{});
      body(n_kv - 1, P0{}, true_type{}, false_type{});
      last_pv(P1{});
    } else {
      body(0, P0{}, false_type{}, true_type{});
      int t = 1;
      for (; t + 1 < n_kv - 1; t += 2) {
        body(t, P1{}, true_type{}, true_type{});
        body(t + 1, P0{}, true_type{}, true_type{});
      }
      if (t < n_kv - 1) {   // one more middle tile, then the last one has even parity
        body(t, P1{}, true_type{}, true_type{});
        body(t + 1, P0{}, true_type{}, false_type{});
        last_pv(P0{});
      } else {
        body(t, P1{}, true_type{}, false_type{});
        last_pv(P1{});
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
  constexpr int smem = (HD <= 128 ? 3 : 2) * (BKV * HD * 2 + HD * BKV * 2);
  // once per head size; the initialisation of a function-local static is thread-safe
  static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_prefill_kernel<HD>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (attr_err != hipSuccess) return attr_err;
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
