// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T with fp32 accumulation and fused epilogues.
// It carries the QKV, O, gate|up (+GLU) and down projections of a kept layer (Sec. 2.1, Attn and
// FFN blocks) and, in batched form, the independent KV projections of all pruned layers (Sec. 3.3).
//
// Design (MI355X):
//   * Both operands have the contraction index contiguous, so a 16-byte chunk is exactly the 8 bf16
//     values one lane feeds to v_mfma_f32_16x16x32_bf16.  That shape is used rather than 32x32x16:
//     same operand bytes per flop, a quarter of the accumulator registers read and written per
//     instruction, and measurably higher sustained clocks under the power limit.
//   * Tiles are staged global -> LDS with buffer_load_dwordx4 ... lds (no VGPR round trip); rows
//     beyond M / N are out of range of the buffer descriptor and read as zero, so ragged edges need
//     no branches in the main loop.
//   * LDS rows are 64 bf16 (128 B).  Chunk c of row r is stored at chunk position c ^ ((r >> 1) & 7).
//     gfx950's LDS serves a ds_read_b128 sixteen lanes (256 B, 64 banks) per cycle; sixteen
//     consecutive rows are eight 256-byte bank lines, and the key makes the two rows of a line plus
//     the eight lines land on sixteen different 16-byte positions: conflict free (measured:
//     SQ_LDS_BANK_CONFLICT 50 % of SQ_LDS_IDX_ACTIVE with the key r & 7, which collides rows r and
//     r + 8).  The permutation is applied on the global side (each lane picks the chunk that belongs
//     at its LDS position).
//   * STAGES LDS stages (2 for 256x256 tiles, 3 for 256x128): the loads of K-step k+STAGES-1 are
//     issued after the barrier that publishes K-step k, spread over the K-step between groups of
//     four MFMAs, so they overlap MFMA work.  Every K-step each wave also touches a few cache lines
//     several K-steps ahead (a share of the tiles its XCD neighbours will stage), which turns the
//     staging loads into L2 hits.
//   * The main loop is software pipelined by one 32-wide sub-step and rotated so that MFMAs with
//     operands already in registers follow the barrier; when K is a multiple of 64 it contains no
//     vector-ALU instruction besides the MFMAs (they share an issue port).
//   * Tile shape is chosen per problem so that the number of tiles fills 256 CUs evenly; a partly
//     filled last round of 256x256 tiles is computed by a second launch with 128x256 tiles.
//   * The MFMA is issued with W as the first operand, so a lane ends up with 4 consecutive output
//     columns of one row: epilogues use 8/16-byte accesses.
//   * Work-group ids are remapped so that the 32 groups that run together on one XCD (ids equal mod
//     8) work on 8 row tiles x 4 column tiles and share them through that XCD's L2.
#include <algorithm>
#include <cstdlib>
#include <type_traits>
#include <utility>

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
  int tiles_m, tiles_n;  // per batch, of this launch
  int n_tile0;           // first column tile of this launch (a GEMM may be split into two launches)
  long long strideA, strideC, strideW;
  const bf16_t* const* W_list;
  float scale;           // EPI_ADD_F32: out += scale * C
  // KV-cache epilogues
  const KvDest* kv_dest;
  const int32_t* kv_slot;
  int kv_heads, kv_page;
  long long kv_pool_stride;
  KvQuant kvq;
};

// Template values of the KV-cache epilogue (EPI_KV_CACHE of the interface), one per head_dim: the offset between
// the two halves of a head decides which accumulator registers are RoPE partners, so it must be a constant.
constexpr int EPI_KV64 = 1064, EPI_KV128 = 1128, EPI_KV256 = 1256;   // (apart from the interface's values)
constexpr bool epi_is_kv(int e) { return e == EPI_KV64 || e == EPI_KV128 || e == EPI_KV256; }
constexpr int epi_kv_hd(int e) { return e == EPI_KV64 ? 64 : e == EPI_KV128 ? 128 : 256; }

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// SiLU: g * sigmoid(g); tanh-GELU: 0.5 g (1 + tanh(u)) = g * sigmoid(2u), u = sqrt(2/pi) (g + 0.044715 g^3).
// Both are g / (1 + 2^(-g (k0 + k1 g^2))): one v_exp_f32 and one v_rcp_f32, constants chosen per
// activation (SiLU: k0 = log2(e), k1 = 0; GELU: k0 = 2 sqrt(2/pi) log2(e), k1 = 0.044715 k0).
__device__ __forceinline__ float glu_act(float g, float k0, float k1) {
  return g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-g * (k0 + k1 * g * g)));
}

template <typename F, int... I>
__device__ __forceinline__ void for_each_index(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}

// KFULL: K is a multiple of BK.  Then no lane ever needs a tail mask and the main loop carries no
// vector-ALU instruction besides the MFMAs (address arithmetic is loop invariant or scalar): vector
// ALU instructions share the issue port with the MFMAs and every one of them delays the next MFMA.
template <int BM, int BN, int WGM, int WGN, int STAGES, int EPI, bool KFULL>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(GemmParams p) {
#if defined(__HIP_DEVICE_COMPILE__)  // the buffer-resource builtins exist in the device pass only
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int MB = WTM / 16, NB = WTN / 16;   // 16x16 output blocks of a wave tile
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
  // Tiles are numbered in bands of 8 row tiles: inside a band the row tile runs fastest, then the
  // column tile.  The 32 CUs of an XCD then work on 8 row tiles x 4 column tiles at a time whatever M
  // is (each W tile is shared by 8 of them, each A tile by 4), which is what their L2 can hold.
  int tm, tn;
  {
    const int band = logical / (8 * p.tiles_n);
    const int rows = min(8, p.tiles_m - band * 8);     // the last band may be narrower
    const int r = logical - band * 8 * p.tiles_n;
    tn = r / rows;
    tm = band * 8 + r % rows;
  }
  const int m0 = tm * BM;
  constexpr int BN_OUT = EPI == EPI_GLU_BF16 ? BN / 2 : BN;
  const int n0 = (p.n_tile0 + tn) * BN_OUT;  // first output column of the tile

  const int z = blockIdx.z;
  const bf16_t* A = p.A + (long long)z * p.strideA;
  const bf16_t* W = p.W_list ? p.W_list[z] : p.W + (long long)z * p.strideW;

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
  static_assert(NW % 2 == 0, "the swizzle key of a staged row must not depend on the load index");
  const int lr = lane >> 3;         // row inside an 8-row group
  // logical chunk that belongs at this lane's LDS position: key = (tile row >> 1) & 7, and the tile
  // row is (j * NW + wave) * 8 + lr with NW even, so the key is ((wave & 1) << 2) | (lr >> 1)
  const int lc = (lane & 7) ^ (((wave & 1) << 2) | (lr >> 1));
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

  // K-step t is staged by LA + LB wave-loads, spread over the STEPS = BK/32 MFMA sub-steps of the
  // K-step before it (LPS per sub-step).  tail_mask has bit 31 set on lanes whose chunk lies beyond K (or for a K-step beyond
  // the last one): that pushes the offset out of range and the lane stages zeros.
  constexpr int STEPS = BK / 32;
  constexpr int LOADS = LA + LB;
  constexpr int LPS = (LOADS + STEPS - 1) / STEPS;  // loads per slice
  const int nk = (p.K + BK - 1) / BK;
  // KFULL: a K-step beyond the last one re-stages the last one (into a stage nobody reads any more),
  // which keeps the number of loads per iteration uniform without a per-lane mask.
  auto issue_one = [&](int q, int kt, unsigned char* stage_base, uint32_t tail_mask) {
    if (q >= LOADS) return;
    const int k0 = (KFULL ? min(kt, nk - 1) : kt) * BK;
    unsigned char* sa = stage_base;
    unsigned char* sb = sa + A_BYTES;
    if (q < LA)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rA, (lds_ptr_t)(sa + (q * NW + wave) * 1024), 16,
                                               KFULL ? offA[q] : (offA[q] | tail_mask), k0 * 2, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rW, (lds_ptr_t)(sb + ((q - LA) * NW + wave) * 1024), 16,
                                               KFULL ? offB[q - LA] : (offB[q - LA] | tail_mask), k0 * 2, 0, 0);
  };
  auto issue = [&](int kt, int stage, uint32_t tail_mask) {
#pragma unroll
    for (int q = 0; q < LOADS; ++q) issue_one(q, kt, smem + stage * STAGE, tail_mask);
  };
  const int nk_full = p.K / BK;  // K-steps that need no tail mask
  const uint32_t last_mask = (nk_full * BK + lc * 8 < p.K) ? 0u : kOOB;

  // L2 prefetch.  The work-groups that run together on one XCD share their W tile (same tn, eight
  // consecutive tm) and their A tile (same tm, four tn), and all of them walk K in step, so an L2
  // miss of one is a miss of all: every staged line then pays HBM latency, which bounds the loading
  // rate.  Each K-step every wave therefore touches (4-byte DMA load into a scratch line of LDS) a
  // few cache lines PF_DIST K-steps ahead: wave 0 one eighth of the W tile's rows (slice tm % 8),
  // waves 1 and 2 one quarter of the A tile's rows (slice tn % 4).  Together the sharers cover both
  // tiles, and the real loads later hit in L2.
  constexpr int PF_DIST = STAGES + 1;
  unsigned char* pf_scratch = smem + STAGES * STAGE;
  uint32_t pf_off;
  {
    const int l32 = lane & 31;
    if (wave == 0) {
      const int jn = (tm & 7) * (BN / 8) + (lane % (BN / 8));   // row of the LDS B tile
      int wrow; bool ok = lane < BN / 8;
      if (EPI == EPI_GLU_BF16) {
        const int w2 = jn / WTN, r = jn % WTN;
        const int oc = n0 + w2 * (WTN / 2) + (r % (WTN / 2));
        ok = ok && oc < p.N;
        wrow = (r >= WTN / 2 ? p.N : 0) + oc;
      } else {
        wrow = n0 + jn;
        ok = ok && wrow < p.N;
      }
      pf_off = ok ? (uint32_t)((long long)wrow * p.ldw * 2) : kOOB;
    } else if (wave <= 2) {
      const int row = m0 + (tn & 3) * (BM / 4) + (wave - 1) * 32 + l32;
      const bool ok = lane < 32 && (wave - 1) * 32 + l32 < BM / 4 && row < p.M;
      pf_off = ok ? (uint32_t)((long long)row * p.lda * 2) : kOOB;
    } else {
      pf_off = kOOB;
    }
  }
  auto prefetch = [&](int kt) {   // one DMA load per wave; lanes beyond K or beyond the tile are masked
    const uint32_t off = KFULL ? pf_off : ((kt * BK < p.K) ? pf_off : kOOB);
    const int kk = KFULL ? min(kt, nk - 1) : kt;
    if (wave == 0) __builtin_amdgcn_raw_ptr_buffer_load_lds(rW, (lds_ptr_t)pf_scratch, 4, off, kk * BK * 2, 0, 0);
    else __builtin_amdgcn_raw_ptr_buffer_load_lds(rA, (lds_ptr_t)(pf_scratch + 256), 4, off, kk * BK * 2, 0, 0);
  };

  // v_mfma_f32_16x16x32_bf16: D[16 x 16] += A[16 x 32] B[32 x 16].  Lane l supplies row l % 16 of A
  // (here: a W row = output column) and column l % 16 of B (an activation row = output row), 8
  // consecutive k each starting at 8 (l / 16), and receives rows 4 (l / 16) .. +3 of column l % 16.
  // The 16x16 shape is used instead of 32x32x16 for its smaller accumulator traffic per flop.
  floatx4_t acc[NB][MB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

  // LDS read offsets: row (lane & 15) of a 16-row block, chunk (4*ks + lane/16) ^ ((row >> 1) & 7)
  const int frag_row = lane & 15;
  const int frag_hi = lane >> 4;
  const int a_base = (wm * WTM + frag_row) * 128;
  const int b_base = (wn * WTN + frag_row) * 128;

  static_assert(STAGES >= 2 && STAGES <= 8, "2 to 8 LDS stages");
  static_assert(1 + (STAGES - 2) * (LOADS + 1) < 64, "vmcnt is a 6-bit counter");
#pragma unroll
  for (int t = 0; t < STAGES - 1; ++t) {
    // with 4 or more stages the waits below count on every prologue stage having been requested: a stage
    // beyond the last K-step is requested masked (or re-stages the last K-step) and never read
    if (t < nk) issue(t, t, t < nk_full ? 0u : last_mask);
    else if (STAGES >= 4) issue(t, t, kOOB);
  }
  // The K loop is rotated by one (32-wide) sub-step: the MFMAs of the last sub-step of K-step kt-1 are issued
  // after the barrier of K-step kt, from fragments that are already in registers, so the matrix
  // pipe has work while the first fragments of the new stage travel from LDS.  Sub-step s of a
  // K-step uses fragment buffer s & 1 (STEPS is even); the buffer of the "previous last sub-step"
  // starts as zeros, which makes the first iteration's MFMAs add nothing.
  static_assert(STEPS % 2 == 0, "fragment buffer parity must repeat every K-step");
  bf16x8_t af[2][MB], bfr[2][NB];
#pragma unroll
  for (int j = 0; j < MB; ++j)
#pragma unroll
    for (int v = 0; v < 8; ++v) af[1][j][v] = (__bf16)0.f;
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int v = 0; v < 8; ++v) bfr[1][i][v] = (__bf16)0.f;
  constexpr int READS = MB + NB, MFMAS = MB * NB;
  constexpr int G = MB % 2 == 0 ? 2 * NB : NB;      // groups per sub-step: half a W block's MFMAs (64 cycles) each
  constexpr int MPG = MFMAS / G;                    // MFMAs per group
  constexpr int RPG = (READS + G - 1) / G;          // LDS reads per group
  constexpr int LPG = (LPS + G - 1) / G;            // global loads per group
  static_assert(MFMAS % G == 0, "MFMAs must split evenly into groups");
  // One K-step; the stage that holds it and the stage refilled meanwhile are compile-time constants
  // (the loop below is unrolled by STAGES), so LDS addresses are loop-invariant registers + immediates.
  auto kstep = [&](int kt, auto stage_c, auto fill_c) {
    constexpr int stage = decltype(stage_c)::value, fill = decltype(fill_c)::value;
    // Wait until K-step kt has landed.  Loads return in order, so it is enough to bound how many
    // younger ones may still be in flight.  Every iteration issues exactly LOADS staging loads (masked
    // beyond the last K-step) followed by one prefetch load, so behind K-step kt's loads there are:
    // 2 stages: the previous iteration's prefetch; 3 stages: prefetch, LOADS, prefetch.  The first
    // iterations have fewer; waiting for more than necessary there is harmless.
    // The fragment reads of the previous K-step must also have completed before any wave refills
    // the stage they came from (lgkmcnt).
    if (STAGES == 2) {
      if (kt > 0) asm volatile("s_waitcnt vmcnt(1) lgkmcnt(0)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    } else if (STAGES == 3) {
      if (kt >= 2) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(LOADS + 2) : "memory");
      else if (kt == 1) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(LOADS) : "memory");
      else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    } else {
      // General form: from K-step STAGES-1 on, behind K-step kt's loads there are its own iteration's
      // prefetch and STAGES-2 whole iterations (LOADS + 1 each).  K-steps 0 .. STAGES-2 were requested in
      // the prologue, stage by stage; behind K-step kt's loads there are at least the STAGES-2-kt stages
      // requested after it (kt equals `stage` there).
      constexpr int GENERAL = 1 + (STAGES - 2) * (LOADS + 1);
      constexpr int EARLY = stage <= STAGES - 2 ? (STAGES - 2 - stage) * LOADS : 0;
      if (kt >= STAGES - 1) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(GENERAL) : "memory");
      else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(EARLY) : "memory");
    }
    __builtin_amdgcn_s_barrier();
    // K-step to prefetch during this one (branch-free: beyond the end every lane is masked off)
    const int tp = kt + STAGES - 1;
    const uint32_t pmask = KFULL ? 0u : (tp < nk_full ? 0u : (tp < nk ? last_mask : kOOB));
    unsigned char* fill_base = smem + fill * STAGE;
    const unsigned char* sa = smem + stage * STAGE;
    const unsigned char* sb = sa + A_BYTES;
    // Every slot is cut into G groups; a group carries a share of the LDS reads of sub-step `slot`,
    // one slice of the next K-step's global loads, and MPG MFMAs of the sub-step before it.
    // Scheduling barriers pin that order: a wave that issues its global loads in one burst sits in
    // the memory pipeline's issue queue while its MFMAs could run.
    auto load_frag = [&](int ks, int buf, int r) {    // r-th fragment read of sub-step ks
      const int pc = ((4 * ks + frag_hi) ^ ((frag_row >> 1) & 7)) * 16;
      if (r < NB) bfr[buf][r] = *reinterpret_cast<const bf16x8_t*>(sb + b_base + r * 16 * 128 + pc);
      else af[buf][r - NB] = *reinterpret_cast<const bf16x8_t*>(sa + a_base + (r - NB) * 16 * 128 + pc);
    };
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int slot = 0; slot < STEPS; ++slot) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int r = g * RPG; r < (g + 1) * RPG && r < READS; ++r) load_frag(slot, slot & 1, r);
#pragma unroll
        for (int q = g * LPG; q < (g + 1) * LPG && q < LPS; ++q) issue_one(slot * LPS + q, tp, fill_base, pmask);
#pragma unroll
        for (int e = g * MPG; e < (g + 1) * MPG; ++e) {
          // W block by W block, the activation blocks forwards and backwards in turn: from one MFMA to the next
          // only one of the two operands changes (measured 0.3 to 1.2 % faster than restarting at block 0:
          // the clock under this load is set by power, and operand switching is part of it)
          const int i = e / MB, j = (i & 1) ? MB - 1 - e % MB : e % MB;
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[(slot + 1) & 1][i], af[(slot + 1) & 1][j],
                                                              acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    prefetch(kt + PF_DIST);
  };
  {
    typedef std::integral_constant<int, 0> S0;
    typedef std::integral_constant<int, 1> S1;
    typedef std::integral_constant<int, 2> S2;
    int kt = 0;
    if constexpr (STAGES == 2) {
      for (; kt + 1 < nk; kt += 2) {
        kstep(kt, S0{}, S1{});
        kstep(kt + 1, S1{}, S0{});
      }
      if (kt < nk) kstep(kt, S0{}, S1{});
    } else if constexpr (STAGES >= 4) {
      // unrolled by STAGES: instance I handles K-steps congruent to I, in stage I, refilling stage I - 1
      auto one = [&](int base, auto idx) {
        constexpr int I = decltype(idx)::value;
        kstep(base + I, std::integral_constant<int, I>{}, std::integral_constant<int, (I + STAGES - 1) % STAGES>{});
      };
      for (; kt + STAGES - 1 < nk; kt += STAGES)
        for_each_index([&](auto idx) { one(kt, idx); }, std::make_integer_sequence<int, STAGES>{});
      for_each_index([&](auto idx) { if (kt + decltype(idx)::value < nk) one(kt, idx); },
                     std::make_integer_sequence<int, STAGES>{});
    } else {
      for (; kt + 2 < nk; kt += 3) {
        kstep(kt, S0{}, S2{});
        kstep(kt + 1, S1{}, S0{});
        kstep(kt + 2, S2{}, S1{});
      }
      if (kt < nk) kstep(kt, S0{}, S2{});
      if (kt + 1 < nk) kstep(kt + 1, S1{}, S0{});
    }
  }
  // last sub-step of the last K-step
#pragma unroll
  for (int e = 0; e < MFMAS; ++e) {
    const int i = e / MB, j = (i & 1) ? MB - 1 - e % MB : e % MB;
    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[(STEPS - 1) & 1][i], af[(STEPS - 1) & 1][j], acc[i][j], 0, 0, 0);
  }
  // masked staging loads and prefetches of the last iterations still target this group's LDS
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // ---- epilogue.  acc[i][j][v]: row m = .. + j*16 + (lane & 15); column block i, columns
  //      4 (lane >> 4) + v inside it: 4 consecutive columns per lane.
  const int m_lane = m0 + wm * WTM + frag_row;
  if (EPI == EPI_GLU_BF16) {
    const float act_k0 = p.act == 0 ? 1.4426950408889634f : 2.302208198f;
    const float act_k1 = p.act == 0 ? 0.f : 0.1029432396f;
    bf16_t* out = reinterpret_cast<bf16_t*>(p.out) + (long long)z * p.strideC;
    // rows outer, column blocks inner: the stores that complete one 128-byte line of a row follow
    // each other directly
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int i = 0; i < NB / 2; ++i) {
        const int m = m_lane + j * 16;
        if (m >= p.M) continue;
        {
          const int n = n0 + wn * (WTN / 2) + i * 16 + frag_hi * 4;
          float r[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) r[e] = glu_act(acc[i][j][e], act_k0, act_k1) * acc[i + NB / 2][j][e];
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
  } else if (epi_is_kv(EPI)) {
   if constexpr (epi_is_kv(EPI)) {   // (the indices below only exist for these instantiations)
    // Independent KV projections (Sec. 3.3) straight into the paged cache.  The wave tile holds whole heads
    // (WTN is a multiple of the head size): column block i of a head and block i + HB are the two halves of the
    // same rotation pairs, in the same lane and register slot.  K columns are rotated in fp32 on the accumulators
    // and rounded to bf16 once; V columns are rounded and stored.  Rows outer, blocks inner, low half then high
    // half: the 8-byte stores of the four lanes that share a row complete 32 bytes, the blocks a 128-byte line.
    constexpr int HD = epi_kv_hd(EPI), HB = HD / 32, HPW = WTN / HD;   // HB: 16-column blocks in half a head
    static_assert(WTN % HD == 0, "a wave tile must hold whole heads");
    const int Dkv = p.N >> 1;
    const int n_wave = n0 + wn * WTN;                  // first column of the wave tile (wave-uniform)
    if (n_wave < p.N) {
      const bool is_k = n_wave < Dkv;                  // Dkv is a multiple of WTN (checked by the launcher)
      const int head0 = (is_k ? n_wave : n_wave - Dkv) / HD;
      const KvDest dst = p.kv_dest[z];
      const bool fp8 = p.kvq.fp8 != 0;                 // one-byte e4m3 codes instead of bf16 entries
      const long long esz = fp8 ? 1 : 2;
      char* pool = reinterpret_cast<char*>(dst.k_pool) + (is_k ? 0 : p.kv_pool_stride) * esz;
      const float inv = is_k ? p.kvq.k_inv : p.kvq.v_inv;
      const int P = p.kv_page;
#pragma unroll
      for (int j = 0; j < MB; ++j) {
        const int m = m_lane + j * 16;
        if (m >= p.M) continue;
        const int s = p.kv_slot[m];
        char* row = pool + ((((long long)(s / P) * p.kv_heads + head0) * P + (s % P)) * HD + frag_hi * 4) * esz;
        const float4* csr = reinterpret_cast<const float4*>(dst.cs + (long long)m * (HD / 2) + frag_hi * 4);
#pragma unroll
        for (int hw = 0; hw < HPW; ++hw) {
          char* hrow = row + (long long)hw * P * HD * esz;
#pragma unroll
          for (int ib = 0; ib < HB; ++ib) {
            const int lo = hw * 2 * HB + ib, hi = lo + HB;
            float a[4], b[4];
            if (is_k) {
              // (cos, sin) of the four pairs this lane holds: dims ib*16 + frag_hi*4 .. +3
              const float4 c01 = csr[ib * 8], c23 = csr[ib * 8 + 1];
              const float cc[4] = {c01.x, c01.z, c23.x, c23.z}, sn[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                a[e] = acc[lo][j][e] * cc[e] - acc[hi][j][e] * sn[e];
                b[e] = acc[hi][j][e] * cc[e] + acc[lo][j][e] * sn[e];
              }
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e) { a[e] = acc[lo][j][e]; b[e] = acc[hi][j][e]; }
            }
            if (fp8) {
              *reinterpret_cast<uint32_t*>(hrow + ib * 16) = e4m3_pack4(a[0] * inv, a[1] * inv, a[2] * inv, a[3] * inv);
              *reinterpret_cast<uint32_t*>(hrow + HD / 2 + ib * 16) = e4m3_pack4(b[0] * inv, b[1] * inv, b[2] * inv, b[3] * inv);
            } else {
              uint2 pa, pb;
              pa.x = pack_bf16x2(a[0], a[1]); pa.y = pack_bf16x2(a[2], a[3]);
              pb.x = pack_bf16x2(b[0], b[1]); pb.y = pack_bf16x2(b[2], b[3]);
              *reinterpret_cast<uint2*>(hrow + (ib * 16) * 2) = pa;
              *reinterpret_cast<uint2*>(hrow + (HD / 2 + ib * 16) * 2) = pb;
            }
          }
        }
      }
    }
   }
  } else if (EPI == EPI_ADD_F32) {
    // out += C.  The old values are requested sixteen 16x16 blocks at a time, without branches (a lane whose
    // four columns are not all inside reads the first element of the matrix instead), so that the loads
    // of a group are in flight together; a load that sits behind a branch of its own is waited for before the
    // next one is requested (one memory round trip per block; measured: 2 to 7 us per projection at 2048 rows).
    float* outp = reinterpret_cast<float*>(p.out) + (long long)z * p.strideC;
    constexpr int TOT = MB * NB, CH = 16;
#pragma unroll
    for (int c0 = 0; c0 < TOT; c0 += CH) {
      float4 old[CH];
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int e = c0 + c;
        if (e < TOT) {
          const int j = e / NB, i = e % NB;
          const int m = m_lane + j * 16, n = n0 + wn * WTN + i * 16 + frag_hi * 4;
          const bool full = m < p.M && n + 3 < p.N;
          old[c] = *reinterpret_cast<const float4*>(full ? outp + (long long)m * p.ldc + n : outp);
        }
      }
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int e = c0 + c;
        if (e < TOT) {
          const int j = e / NB, i = e % NB;
          const int m = m_lane + j * 16, n = n0 + wn * WTN + i * 16 + frag_hi * 4;
          float* o = outp + (long long)m * p.ldc + n;
          if (m < p.M && n + 3 < p.N) {
            *reinterpret_cast<float4*>(o) = make_float4(acc[i][j][0] * p.scale + old[c].x, acc[i][j][1] * p.scale + old[c].y,
                                                        acc[i][j][2] * p.scale + old[c].z, acc[i][j][3] * p.scale + old[c].w);
          } else if (m < p.M && n < p.N) {   // the last, partial group of four columns
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (n + q < p.N) o[q] += acc[i][j][q] * p.scale;
          }
        }
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int m = m_lane + j * 16;
        if (m >= p.M) continue;
        {
          const int n = n0 + wn * WTN + i * 16 + frag_hi * 4;
          if (n >= p.N) continue;
          const float r0 = acc[i][j][0], r1 = acc[i][j][1];
          const float r2 = acc[i][j][2], r3 = acc[i][j][3];
          if (EPI == EPI_STORE_BF16 || EPI == EPI_STORE_F16) {
            bf16_t* o = reinterpret_cast<bf16_t*>(p.out) + (long long)z * p.strideC + (long long)m * p.ldc + n;
            if (n + 3 < p.N) {
              uint2 pk;
              pk.x = EPI == EPI_STORE_F16 ? pack_f16x2(r0, r1) : pack_bf16x2(r0, r1);
              pk.y = EPI == EPI_STORE_F16 ? pack_f16x2(r2, r3) : pack_bf16x2(r2, r3);
              *reinterpret_cast<uint2*>(o) = pk;
            } else {
              const float r[4] = {r0, r1, r2, r3};
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (n + e < p.N) o[e] = EPI == EPI_STORE_F16 ? f32_to_f16_sat(r[e]) : f32_to_bf16(r[e]);
            }
          } else {   // EPI_STORE_F32
            float* o = reinterpret_cast<float*>(p.out) + (long long)z * p.strideC + (long long)m * p.ldc + n;
            if (n + 3 < p.N) {
              *reinterpret_cast<float4*>(o) = make_float4(r0, r1, r2, r3);
            } else {
              const float r[4] = {r0, r1, r2, r3};
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (n + e < p.N) o[e] = r[e];
            }
          }
        }
      }
  }
#endif
}

template <int BM, int BN, int WGM, int WGN, int STAGES, int EPI>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t st, int n_tile0 = 0, int n_tiles = -1) {
  constexpr int BN_OUT = EPI == EPI_GLU_BF16 ? BN / 2 : BN;
  constexpr int smem = STAGES * (BM + BN) * BK * 2 + 1024;  // stages + prefetch scratch
  static_assert(smem <= 160 * 1024, "LDS budget of a gfx950 CU");
  GemmParams p;
  p.A = g.A; p.W = g.W; p.out = g.out;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.lda = (int)g.lda; p.ldw = (int)g.ldw; p.ldc = (int)g.ldc;
  p.act = g.act;
  p.scale = residual_scale(g);
  p.kv_dest = g.kv_dest; p.kv_slot = g.kv_slot; p.kv_heads = g.kv_heads; p.kv_page = g.kv_page_size;
  p.kv_pool_stride = g.kv_pool_stride;
  p.kvq = g.kvq;
  p.tiles_m = (g.M + BM - 1) / BM;
  p.tiles_n = n_tiles >= 0 ? n_tiles : (g.N + BN_OUT - 1) / BN_OUT;
  p.n_tile0 = n_tile0;
  if (p.tiles_n <= 0) return hipSuccess;
  p.strideA = g.strideA; p.strideC = g.strideC; p.strideW = g.W_list ? 0 : g.strideW;
  p.W_list = g.batch > 1 || g.W_list ? g.W_list : nullptr;
  // once per instantiation; the initialisation of a function-local static is thread-safe
  static const hipError_t attr_err = [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<BM, BN, WGM, WGN, STAGES, EPI, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<BM, BN, WGM, WGN, STAGES, EPI, false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  }();
  if (attr_err != hipSuccess) return attr_err;
  const int total = p.tiles_m * p.tiles_n;
  const int grid = ((total + 7) / 8) * 8;
  const dim3 grid3(grid, 1, g.batch > 0 ? g.batch : 1), block3(64 * WGM * WGN);
  if (g.K % BK == 0)
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WGM, WGN, STAGES, EPI, true>), grid3, block3, smem, st, p);
  else
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WGM, WGN, STAGES, EPI, false>), grid3, block3, smem, st, p);
  return hipGetLastError();
}

// Tile choice: minimise the estimated time on the critical path,
//     rounds * K-steps * max(latency floor of a K-step, work-groups per CU * compute time of a K-step),
//     rounds = ceil(tiles / (256 CUs * work-groups per CU)).
// The compute time of a K-step is tile area * a relative cost per flop measured on MI355X at the
// Llama-3.1-8B projection shapes (256x256 tiles move the fewest operand bytes per flop and are the
// fastest per flop; smaller tiles only win when they fill the chip better).  The floor is what a
// K-step takes when the work-group only waits for its loads (0.55 us with 2 stages, about half with
// 3): with few rows (short prompts) a projection is weight streaming, every configuration runs at
// its floor, and the small tiles win because more work-groups, several per CU, have loads in flight.
struct TileCfg { int id, bm, bn; double rel; int occ; double floor_us; };
constexpr TileCfg kTileCfgs[] = {
    {1, 256, 256, 1.00, 1, 0.55}, {5, 256, 192, 1.08, 1, 0.55}, {3, 256, 128, 1.25, 1, 0.30},
    {4, 128, 128, 1.40, 2, 0.55}, {7, 128, 64, 1.75, 2, 0.30},  {8, 64, 128, 1.67, 2, 0.30},
    {6, 64, 64, 2.09, 3, 0.27},   {9, 64, 64, 2.09, 1, 0.22},   // 9: six stages, one work-group per CU
};

// Estimated time (us) of configuration c for M rows, `cols` W rows, K, `batch` problems.
inline double tile_cost_us(const TileCfg& c, long long M, long long cols, long long K, long long batch) {
  const long long tiles = ((M + c.bm - 1) / c.bm) * ((cols + c.bn - 1) / c.bn) * batch;
  const double kstep_us = (double)c.bm * c.bn * c.rel * (1.54 / 65536.0);   // 256x256: 1.54 us
  const long long rounds = (tiles + 256LL * c.occ - 1) / (256LL * c.occ);
  const long long share = std::min<long long>(c.occ, (tiles + 255) / 256);
  return (double)rounds * (double)((K + BK - 1) / BK) * std::max(c.floor_us, (double)share * kstep_us);
}

template <int EPI>
hipError_t launch_epi(const GemmArgs& g, hipStream_t st) {
  const long long batch = g.batch > 0 ? g.batch : 1;
  const long long cols = EPI == EPI_GLU_BF16 ? 2LL * g.N : g.N;  // W rows consumed
  auto cost = [&](const TileCfg& c) { return tile_cost_us(c, g.M, cols, g.K, batch); };
  // Building with -DPOP_FORCE_GEMM_TILE=1..9 forces one configuration (tile-shape experiments, never the
  // product build): the choice is a compile-time constant and nothing in the environment can change it.
#ifdef POP_FORCE_GEMM_TILE
  constexpr int forced = POP_FORCE_GEMM_TILE;
#else
  constexpr int forced = 0;
#endif
  int pick = forced;
  if (pick < 1 || pick > 9 || (pick == 5 && EPI == EPI_GLU_BF16)) {
    double best = 1e300;
    for (const TileCfg& c : kTileCfgs) {      // ordered by area: ties go to the larger tile
      if (c.id == 5 && EPI == EPI_GLU_BF16) continue;
      const double t = cost(c);
      if (t < best) { best = t; pick = c.id; }
    }
  }
  switch (pick) {
    case 2: return launch_cfg<256, 256, 2, 4, 2, EPI>(g, st);
    case 3: return launch_cfg<256, 128, 2, 2, 3, EPI>(g, st);
    case 4: return launch_cfg<128, 128, 2, 2, 2, EPI>(g, st);
    case 6: return launch_cfg<64, 64, 2, 2, 3, EPI>(g, st);
    case 7: return launch_cfg<128, 64, 2, 2, 3, EPI>(g, st);
    case 8: return launch_cfg<64, 128, 2, 2, 3, EPI>(g, st);
    case 9: return launch_cfg<64, 64, 2, 2, 6, EPI>(g, st);
    case 5:
      if constexpr (EPI != EPI_GLU_BF16) return launch_cfg<256, 192, 2, 2, 2, EPI>(g, st);
      [[fallthrough]];
    default: break;
  }
  // 256x256 tiles.  If they leave the last round of 256 work-groups partly empty, the column tiles
  // of that last round are computed by a second launch with 128x256 tiles (twice as many, half as
  // long): at M = 2048 the gate|up projection has 896 tiles = 3.5 rounds, i.e. 3 rounds of 256x256
  // plus one round of 128x256 instead of four rounds.
  const int tiles_m = (g.M + 255) / 256;
  const int tiles_n = (int)((cols + 255) / 256);
  const long long total = (long long)tiles_m * tiles_n * batch;
  const long long rem = total % 256;
  if (forced == 0 && batch == 1 && total > 256 && rem > 0 && rem <= 128 && g.M > 128) {
    const int tail_cols = (int)((rem + tiles_m - 1) / tiles_m);   // column tiles moved to the second launch
    const int head_cols = tiles_n - tail_cols;
    // only worth it when the second launch fills the chip better than the partial round did
    if (head_cols > 0 && (long long)tail_cols * ((g.M + 127) / 128) <= 256) {
      hipError_t e = launch_cfg<256, 256, 2, 2, 2, EPI>(g, st, 0, head_cols);
      if (e != hipSuccess) return e;
      return launch_cfg<128, 256, 2, 2, 2, EPI>(g, st, head_cols, tail_cols);
    }
  }
  return launch_cfg<256, 256, 2, 2, 2, EPI>(g, st);
}

}  // namespace gemm_impl
using namespace gemm_impl;

// ------------------------------------------------------------------------------------- split K
namespace gemm_impl {
// out = epilogue(parts[0] + parts[1] + ... + parts[S-1]), parts fp32 [S][M][N] dense, added in index order
// (deterministic).  One thread per 4 consecutive columns.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ parts, int S, long long part_stride,
                                                            int M, int N, void* __restrict__ out, long long ldc,
                                                            float scale /* EPI_ADD_F32: out += scale * sum */) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const int n4 = N >> 2;
  if (idx >= (long long)M * n4) return;
  const int m = (int)(idx / n4), n = (int)(idx % n4) * 4;
  const float* p0 = parts + (long long)m * N + n;
  float4 acc = *reinterpret_cast<const float4*>(p0);
  for (int s = 1; s < S; ++s) {
    const float4 v = *reinterpret_cast<const float4*>(p0 + (long long)s * part_stride);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  if (EPI == EPI_STORE_BF16 || EPI == EPI_STORE_F16) {
    uint2 pk;
    pk.x = EPI == EPI_STORE_F16 ? pack_f16x2(acc.x, acc.y) : pack_bf16x2(acc.x, acc.y);
    pk.y = EPI == EPI_STORE_F16 ? pack_f16x2(acc.z, acc.w) : pack_bf16x2(acc.z, acc.w);
    *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(out) + (long long)m * ldc + n) = pk;
  } else {
    float* o = reinterpret_cast<float*>(out) + (long long)m * ldc + n;
    if (EPI == EPI_ADD_F32) {
      const float4 old = *reinterpret_cast<const float4*>(o);
      acc.x = acc.x * scale + old.x; acc.y = acc.y * scale + old.y;
      acc.z = acc.z * scale + old.z; acc.w = acc.w * scale + old.w;
    }
    *reinterpret_cast<float4*>(o) = acc;
  }
}

// Number of K parts for this problem (1 = do not split).  Measured inside the model, where every layer's
// weights come from HBM for the first time: with 256 rows the down projection (K = 14336, 256 work-groups
// of 224 K-steps each) takes 75 us unsplit and 51 us in 8 parts; at K = 4096 (QKV, O) a split gains
// nothing (the second kernel costs what the shorter loop saves), and from 1024 rows on the projections
// are compute bound.  Hence: split only long K with few rows, as far as the scratch allows, and any K when
// the rows fit one 64-row tile and the launch would leave CUs idle.
inline int choose_split(const GemmArgs& g) {
  if (!g.splitk_ws || g.batch > 1 || g.W_list || g.epilogue == EPI_GLU_BF16 || g.epilogue == EPI_KV_CACHE) return 1;
  if (g.N % 4 || g.K % BK || (reinterpret_cast<uintptr_t>(g.splitk_ws) & 15)) return 1;
  if (g.M > 512 && g.force_split <= 1) return 1;
  // Building with -DPOP_FORCE_SPLITK=S forces S parts where the problem allows it (experiments only).
#ifdef POP_FORCE_SPLITK
  constexpr int forced = POP_FORCE_SPLITK;
#else
  constexpr int forced = 0;
#endif
  auto fits = [&](int S) {
    return g.K % (S * BK) == 0 && g.K / (S * BK) >= 8 && (size_t)S * g.M * g.N * 4 <= g.splitk_ws_bytes;
  };
  if (forced == 1) return 1;
  if (forced > 1) return fits(forced) ? forced : 1;
  if (g.force_split > 1 && g.force_split <= 8 && fits(g.force_split)) return g.force_split;
  if (g.M > 256) return 1;
  if (g.K >= 8192) {
    for (int S = 8; S >= 2; S /= 2)
      if (fits(S)) return S;
    return 1;
  }
  // A handful of rows (decode steps, boundary rows) and a short K: the unsplit launch has one row of 64-wide
  // tiles, fewer work-groups than CUs (96 for the Llama QKV projection); split until there are about 256.
  // Measured on batch-8 decode steps at the Llama-3.1-8B shape: 5.29 -> 4.93 ms per step.
  if (g.M > 64) return 1;
  const long long tiles = (g.N + 63) / 64;
  if (tiles >= 256) return 1;
  for (int S = 2; S <= 8; S *= 2)
    if (tiles * S >= 256 || S == 8) return fits(S) ? S : (S > 2 && fits(S / 2) ? S / 2 : 1);
  return 1;
}
}  // namespace gemm_impl

hipError_t launch_gemm(const GemmArgs& g, hipStream_t st) {
  if (g.split_used) *g.split_used = 1;
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.K <= 0 || g.K % 8 || g.lda % 8 || g.ldw % 8 || g.ldc % 4) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.W) |
       (g.epilogue == EPI_KV_CACHE ? 0 : reinterpret_cast<uintptr_t>(g.out))) & 15)
    return hipErrorInvalidValue;
  const long long w_rows = g.epilogue == EPI_GLU_BF16 ? 2LL * g.N : g.N;
  if (((long long)(g.M - 1) * g.lda + g.K) * 2 >= (1LL << 31) || ((w_rows - 1) * g.ldw + g.K) * 2 >= (1LL << 31))
    return hipErrorInvalidValue;
  if (const int S = choose_split(g); S > 1) {
    GemmArgs part = g;
    part.K = g.K / S;
    part.batch = S;
    part.strideA = part.K;                 // part b starts b * K/S elements into every row of A and W
    part.strideW = part.K;
    part.W_list = nullptr;
    part.out = g.splitk_ws;
    part.ldc = g.N;
    part.strideC = (int64_t)g.M * g.N;
    part.epilogue = EPI_STORE_F32;
    part.splitk_ws = nullptr;
    part.partials_only = false;
    part.split_used = nullptr;
    part.scaled = false;
    if (hipError_t e = launch_epi<EPI_STORE_F32>(part, st); e != hipSuccess) return e;
    if (g.partials_only && g.split_used && S <= 8) {   // (the callers' second kernels take up to 8 parts)
      *g.split_used = S;
      return hipGetLastError();
    }
    const long long items = (long long)g.M * (g.N / 4);
    const dim3 grid((unsigned)((items + 255) / 256));
    switch (g.epilogue) {
      case EPI_STORE_BF16:
        hipLaunchKernelGGL(splitk_reduce_kernel<EPI_STORE_BF16>, grid, dim3(256), 0, st, g.splitk_ws, S, part.strideC, g.M, g.N, g.out, (long long)g.ldc, residual_scale(g)); break;
      case EPI_STORE_F16:
        hipLaunchKernelGGL(splitk_reduce_kernel<EPI_STORE_F16>, grid, dim3(256), 0, st, g.splitk_ws, S, part.strideC, g.M, g.N, g.out, (long long)g.ldc, residual_scale(g)); break;
      case EPI_ADD_F32:
        hipLaunchKernelGGL(splitk_reduce_kernel<EPI_ADD_F32>, grid, dim3(256), 0, st, g.splitk_ws, S, part.strideC, g.M, g.N, g.out, (long long)g.ldc, residual_scale(g)); break;
      default:
        hipLaunchKernelGGL(splitk_reduce_kernel<EPI_STORE_F32>, grid, dim3(256), 0, st, g.splitk_ws, S, part.strideC, g.M, g.N, g.out, (long long)g.ldc, residual_scale(g)); break;
    }
    return hipGetLastError();
  }
  switch (g.epilogue) {
    case EPI_STORE_BF16: return launch_epi<EPI_STORE_BF16>(g, st);
    case EPI_ADD_F32: return launch_epi<EPI_ADD_F32>(g, st);
    case EPI_GLU_BF16: return launch_epi<EPI_GLU_BF16>(g, st);
    case EPI_STORE_F32: return launch_epi<EPI_STORE_F32>(g, st);
    case EPI_STORE_F16: return launch_epi<EPI_STORE_F16>(g, st);
    case EPI_KV_CACHE:
      // 256-column tiles whose wave tiles hold whole heads: 2 x 2 waves of 128 x 128 for head sizes 64 and 128,
      // 4 x 1 waves of 64 x 256 for head size 256
      if (!gemm_kv_cache_supported(g.kv_heads, g.kv_hd) || g.N != 2 * g.kv_heads * g.kv_hd || !g.kv_dest ||
          !g.kv_slot || g.kv_page_size < 1)
        return hipErrorInvalidValue;
      if (g.kv_hd == 64) return launch_cfg<256, 256, 2, 2, 2, EPI_KV64>(g, st);
      if (g.kv_hd == 128) return launch_cfg<256, 256, 2, 2, 2, EPI_KV128>(g, st);
      return launch_cfg<256, 256, 4, 1, 2, EPI_KV256>(g, st);
  }
  return hipErrorInvalidValue;
}

bool gemm_kv_cache_supported(int n_kv_heads, int hd) {
  if (hd != 64 && hd != 128 && hd != 256) return false;
  const int wtn = hd == 256 ? 256 : 128;            // columns of a wave tile in the configurations above
  return n_kv_heads > 0 && ((long long)n_kv_heads * hd) % wtn == 0;
}

}  // namespace pop
