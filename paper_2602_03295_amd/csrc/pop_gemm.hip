// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T with fp32 accumulation and fused epilogues.
// It carries the QKV, O, gate|up (+GLU) and down projections of a kept layer (Sec. 2.1, Attn and
// FFN blocks) and, in batched form, the independent KV projections of all pruned layers (Sec. 3.3).
//
// Design (MI355X):
//   * Both operands have the contraction index contiguous, so a 16-byte chunk is exactly the 8 bf16
//     values one lane feeds to v_mfma_f32_32x32x16_bf16.
//   * Tiles are staged global -> LDS with buffer_load_dwordx4 ... lds (no VGPR round trip); rows
//     beyond M / N are out of range of the buffer descriptor and read as zero, so ragged edges need
//     no branches in the main loop.
//   * LDS rows are 64 bf16 (128 B).  Chunk c of row r is stored at chunk position c ^ (r & 7), which
//     makes the ds_read_b128 operand fetches bank-conflict free.  The permutation is applied on the
//     global side (each lane picks the chunk that belongs at its LDS position).
//   * Two LDS stages; the loads of K-step k+1 are issued right after the barrier that publishes
//     K-step k, so they overlap its MFMA work.
//   * The MFMA is issued with W as the first operand, so a lane ends up with 4 consecutive output
//     columns of one row: epilogues use 8/16-byte accesses.
//   * Work-group ids are remapped so that the groups that run together on one XCD (ids equal mod 8)
//     work on neighbouring M tiles of the same W tile and share it through that XCD's L2.
#include "pop_device.h"
#include "pop_kernels.h"

namespace pop {

namespace gemm_impl {

constexpr int BK = 64;                  // K elements per LDS stage
constexpr uint32_t kOOB = 0x80000000u;  // byte offset beyond any buffer we accept (< 2^31 bytes)

struct GemmParams {
  const bf16_t* A;
  const bf16_t* W;
  void* out;
  int M, N, K;           // N = output columns (for GLU: columns of the result, W has 2N rows)
  int lda, ldw, ldc;     // elements
  int act;
  int tiles_m, tiles_n;  // per batch
  long long strideA, strideC;
  const bf16_t* const* W_list;
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;

__device__ __forceinline__ float glu_act(float g, int act) {
  if (act == 0) return g / (1.f + __expf(-g));
  const float u = 0.7978845608028654f * (g + 0.044715f * g * g * g);
  return 0.5f * g * (1.f + tanhf(u));
}

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(GemmParams p) {
#if defined(__HIP_DEVICE_COMPILE__)  // the buffer-resource builtins exist in the device pass only
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int MB = WTM / 32, NB = WTN / 32;
  constexpr int LA = BM / 8 / NW, LB = BN / 8 / NW;  // wave-loads per stage and wave
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile/wave mismatch");
  static_assert(EPI != EPI_GLU_BF16 || NB % 2 == 0, "GLU needs an even number of column blocks");
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  // ---- which tile (XCD-aware remap of the 1-D grid)
  const int total = p.tiles_m * p.tiles_n;
  const int per_xcd = (total + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= total) return;
  const int tm = logical % p.tiles_m, tn = logical / p.tiles_m;
  const int m0 = tm * BM;
  constexpr int BN_OUT = EPI == EPI_GLU_BF16 ? BN / 2 : BN;
  const int n0 = tn * BN_OUT;  // first output column of the tile

  const int z = blockIdx.z;
  const bf16_t* A = p.A + (long long)z * p.strideA;
  const bf16_t* W = p.W_list ? p.W_list[z] : p.W;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  // ---- buffer descriptors; rows beyond the operand are out of range and load zeros
  const uint32_t a_bytes = (uint32_t)(((long long)(p.M - 1) * p.lda + p.K) * 2);
  const int w_rows = EPI == EPI_GLU_BF16 ? 2 * p.N : p.N;
  const uint32_t w_bytes = (uint32_t)(((long long)(w_rows - 1) * p.ldw + p.K) * 2);
  const __amdgpu_buffer_rsrc_t rA =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(A), 0, a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rW =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(W), 0, w_bytes, 0x00020000);

  // ---- per-lane global offsets of the chunks this lane stages (K offset added per step)
  const int lr = lane >> 3;         // row inside an 8-row group
  const int lc = (lane & 7) ^ lr;   // logical chunk that belongs at this lane's LDS position
  uint32_t offA[LA], offB[LB];
#pragma unroll
  for (int j = 0; j < LA; ++j) {
    const int row = m0 + (j * NW + wave) * 8 + lr;
    offA[j] = row < p.M ? (uint32_t)(((long long)row * p.lda + lc * 8) * 2) : kOOB;
  }
#pragma unroll
  for (int j = 0; j < LB; ++j) {
    const int jn = (j * NW + wave) * 8 + lr;  // row of the LDS B tile
    int wrow;
    bool ok;
    if (EPI == EPI_GLU_BF16) {
      const int w2 = jn / WTN, r = jn % WTN;
      const int up = r >= WTN / 2;
      const int oc = n0 + w2 * (WTN / 2) + (r % (WTN / 2));
      ok = oc < p.N;
      wrow = up * p.N + oc;
    } else {
      wrow = n0 + jn;
      ok = wrow < p.N;
    }
    offB[j] = ok ? (uint32_t)(((long long)wrow * p.ldw + lc * 8) * 2) : kOOB;
  }

  // tail_mask: bit 31 set on lanes whose chunk lies beyond K in the last (partial) K-step, which
  // pushes their offset out of range so they stage zeros.
  auto issue = [&](int kt, int stage, uint32_t tail_mask) {
    const int k0 = kt * BK;
    unsigned char* sa = smem + stage * STAGE;
    unsigned char* sb = sa + A_BYTES;
#pragma unroll
    for (int j = 0; j < LA; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rA, (lds_ptr_t)(sa + (j * NW + wave) * 1024), 16,
                                               offA[j] | tail_mask, k0 * 2, 0, 0);
#pragma unroll
    for (int j = 0; j < LB; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rW, (lds_ptr_t)(sb + (j * NW + wave) * 1024), 16,
                                               offB[j] | tail_mask, k0 * 2, 0, 0);
  };
  const int nk = (p.K + BK - 1) / BK;
  const int nk_full = p.K / BK;  // K-steps that need no tail mask
  const uint32_t last_mask = (nk_full * BK + lc * 8 < p.K) ? 0u : kOOB;

  floatx16_t acc[NB][MB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // LDS read offsets: row (lane & 31) of a 32-row block, chunk (2*ks + lane/32) ^ (row & 7)
  const int frag_row = lane & 31;
  const int frag_hi = lane >> 5;
  const int a_base = (wm * WTM + frag_row) * 128;
  const int b_base = (wn * WTN + frag_row) * 128;

  if (nk_full > 0) issue(0, 0, 0u); else issue(0, 0, last_mask);
  for (int kt = 0; kt < nk; ++kt) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (kt + 1 < nk_full) issue(kt + 1, (kt + 1) & 1, 0u);
    else if (kt + 1 < nk) issue(kt + 1, (kt + 1) & 1, last_mask);
    const unsigned char* sa = smem + (kt & 1) * STAGE;
    const unsigned char* sb = sa + A_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int pc = ((2 * ks + frag_hi) ^ (frag_row & 7)) * 16;
      bf16x8_t af[MB], bfr[NB];
#pragma unroll
      for (int j = 0; j < MB; ++j)
        af[j] = *reinterpret_cast<const bf16x8_t*>(sa + a_base + j * 32 * 128 + pc);
#pragma unroll
      for (int i = 0; i < NB; ++i)
        bfr[i] = *reinterpret_cast<const bf16x8_t*>(sb + b_base + i * 32 * 128 + pc);
#pragma unroll
      for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < MB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[i], af[j], acc[i][j], 0, 0, 0);
    }
  }

  // ---- epilogue.  acc[i][j][v]: row m = .. + j*32 + (lane&31); column block i, columns
  //      (v/4)*8 + (lane>>5)*4 + (v%4) inside it: 4 consecutive columns per (v/4).
  const int m_lane = m0 + wm * WTM + frag_row;
  if (EPI == EPI_GLU_BF16) {
    bf16_t* out = reinterpret_cast<bf16_t*>(p.out) + (long long)z * p.strideC;
#pragma unroll
    for (int i = 0; i < NB / 2; ++i)
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        const int m = m_lane + j * 32;
        if (m >= p.M) continue;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + wn * (WTN / 2) + i * 32 + g * 8 + frag_hi * 4;
          float r[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) r[e] = glu_act(acc[i][j][g * 4 + e], p.act) * acc[i + NB / 2][j][g * 4 + e];
          bf16_t* o = out + (long long)m * p.ldc + n;
          if (n + 3 < p.N) {
            uint2 pk;
            pk.x = pack_bf16x2(r[0], r[1]);
            pk.y = pack_bf16x2(r[2], r[3]);
            *reinterpret_cast<uint2*>(o) = pk;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < p.N) o[e] = f32_to_bf16(r[e]);
          }
        }
      }
  } else {
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        const int m = m_lane + j * 32;
        if (m >= p.M) continue;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + wn * WTN + i * 32 + g * 8 + frag_hi * 4;
          if (n >= p.N) continue;
          const float r0 = acc[i][j][g * 4 + 0], r1 = acc[i][j][g * 4 + 1];
          const float r2 = acc[i][j][g * 4 + 2], r3 = acc[i][j][g * 4 + 3];
          if (EPI == EPI_STORE_BF16) {
            bf16_t* o = reinterpret_cast<bf16_t*>(p.out) + (long long)z * p.strideC + (long long)m * p.ldc + n;
            if (n + 3 < p.N) {
              uint2 pk;
              pk.x = pack_bf16x2(r0, r1);
              pk.y = pack_bf16x2(r2, r3);
              *reinterpret_cast<uint2*>(o) = pk;
            } else {
              const float r[4] = {r0, r1, r2, r3};
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (n + e < p.N) o[e] = f32_to_bf16(r[e]);
            }
          } else {
            float* o = reinterpret_cast<float*>(p.out) + (long long)z * p.strideC + (long long)m * p.ldc + n;
            if (n + 3 < p.N) {
              float4 c = make_float4(r0, r1, r2, r3);
              if (EPI == EPI_ADD_F32) {
                const float4 old = *reinterpret_cast<const float4*>(o);
                c.x += old.x; c.y += old.y; c.z += old.z; c.w += old.w;
              }
              *reinterpret_cast<float4*>(o) = c;
            } else {
              const float r[4] = {r0, r1, r2, r3};
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (n + e < p.N) o[e] = (EPI == EPI_ADD_F32 ? o[e] : 0.f) + r[e];
            }
          }
        }
      }
  }
#endif
}

template <int BM, int BN, int WGM, int WGN, int EPI>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t st) {
  constexpr int BN_OUT = EPI == EPI_GLU_BF16 ? BN / 2 : BN;
  constexpr int smem = 2 * (BM + BN) * BK * 2;
  GemmParams p;
  p.A = g.A; p.W = g.W; p.out = g.out;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.lda = (int)g.lda; p.ldw = (int)g.ldw; p.ldc = (int)g.ldc;
  p.act = g.act;
  p.tiles_m = (g.M + BM - 1) / BM;
  p.tiles_n = (g.N + BN_OUT - 1) / BN_OUT;
  p.strideA = g.strideA; p.strideC = g.strideC;
  p.W_list = g.batch > 1 || g.W_list ? g.W_list : nullptr;
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<BM, BN, WGM, WGN, EPI>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int total = p.tiles_m * p.tiles_n;
  const int grid = ((total + 7) / 8) * 8;
  hipLaunchKernelGGL((gemm_kernel<BM, BN, WGM, WGN, EPI>), dim3(grid, 1, g.batch > 0 ? g.batch : 1),
                     dim3(64 * WGM * WGN), smem, st, p);
  return hipGetLastError();
}

template <int EPI>
hipError_t launch_epi(const GemmArgs& g, hipStream_t st) {
  // Large tiles when there is enough work to fill 256 CUs with them, smaller ones otherwise.
  const long long batch = g.batch > 0 ? g.batch : 1;
  const long long out_cols = EPI == EPI_GLU_BF16 ? 2LL * g.N : g.N;
  const long long big_tiles = ((g.M + 255) / 256) * ((out_cols + 255) / 256) * batch;
  if (big_tiles >= 256) return launch_cfg<256, 256, 2, 2, EPI>(g, st);
  return launch_cfg<128, 128, 2, 2, EPI>(g, st);
}

}  // namespace gemm_impl
using namespace gemm_impl;

hipError_t launch_gemm(const GemmArgs& g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.K <= 0 || g.K % 8 || g.lda % 8 || g.ldw % 8 || g.ldc % 4) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.W) |
       reinterpret_cast<uintptr_t>(g.out)) & 15)
    return hipErrorInvalidValue;
  const long long w_rows = g.epilogue == EPI_GLU_BF16 ? 2LL * g.N : g.N;
  if (((long long)(g.M - 1) * g.lda + g.K) * 2 >= (1LL << 31) || ((w_rows - 1) * g.ldw + g.K) * 2 >= (1LL << 31))
    return hipErrorInvalidValue;
  switch (g.epilogue) {
    case EPI_STORE_BF16: return launch_epi<EPI_STORE_BF16>(g, st);
    case EPI_ADD_F32: return launch_epi<EPI_ADD_F32>(g, st);
    case EPI_GLU_BF16: return launch_epi<EPI_GLU_BF16>(g, st);
    case EPI_STORE_F32: return launch_epi<EPI_STORE_F32>(g, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace pop
