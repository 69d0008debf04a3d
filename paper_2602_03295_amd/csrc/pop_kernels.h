// Internal launch interface of the gfx950 kernels behind the POP C ABI.
// Every function enqueues on `st` and returns; pointers are device pointers unless said otherwise.
// Shapes are validated by the callers in pop_api.cpp; launchers only assert what the kernel's
// indexing relies on.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pop {

typedef uint16_t bf16_t;  // raw bf16 bits in memory

// Host side: stores `msg` as the calling thread's last error (the text pop_last_error() returns) and returns
// `status` unchanged.  For the source files of the C ABI other than pop_api.cpp, which owns the record.
int record_error(int status, const char* msg);

// How cache entries are stored: bf16 values, or (fp8) one-byte e4m3 codes of x * inv_scale that read back as
// code value * scale.  Every kernel that appends to the cache or reads it takes one of these.
struct KvQuant {
  int fp8;
  float k_scale, v_scale, k_inv, v_inv;
};

// ---------------------------------------------------------------------------------------------
// Elementwise / bandwidth-bound steps (pop_elementwise.hip)
// ---------------------------------------------------------------------------------------------
// h[t,:] = row_src[t] < 0 ? table[tokens[t],:] : embeds[row_src[t],:]      (fp32 residual stream)
void launch_embed(const bf16_t* table, const int32_t* tokens, const int32_t* row_src,
                  const bf16_t* embeds, float* h, int T, int d, hipStream_t st);

// out[t,:] = bf16( x[t,:] * rsqrt(mean(x[t,:]^2) + eps) * gamma )   -- LN(.) of Sec. 2.1
// If row_idx != nullptr the source row of output row t is row_idx[t] (gather).
// If add1/add2 != nullptr they are first added into x (x is updated in place): this is how the
// partial sums of a split-K projection reach the residual stream.
void launch_rmsnorm(float* x, const float* add1, const float* add2, const float* gamma,
                    bf16_t* out, const int32_t* row_idx, int rows, int d, float eps, hipStream_t st);

// Same statistics, several scales: out[j][t,:] = bf16(x[t,:] * rstd[t] * gammas[j]), j < n_out <= 8.
// Used by the K/V-only path of Sec. 3.3, where all pruned layers see the same hidden state.
struct GammaList {
  const float* g[8];
};
void launch_rmsnorm_multi(const float* x, GammaList gammas, int n_out, bf16_t* out, size_t out_stride,
                          int rows, int d, float eps, hipStream_t st, const int32_t* row_idx = nullptr);
// x[r] += parts[0][r] + parts[1][r] + ... + parts[S-1][r] (fp32 [rows, d] each, part_stride elements apart, added
// in index order), then out[r] = bf16(RMSNorm(x[r]; gamma, eps)): the second kernel of a split projection with a
// residual epilogue and the normalisation that follows it (Sec. 2.1), in one launch.  d % 4 == 0, d <= 8192,
// 1 <= S <= 8.
void launch_add_parts_rmsnorm(float* x, const float* parts, int S, size_t part_stride, const float* gamma, bf16_t* out,
                              int rows, int d, float eps, hipStream_t st, float scale = 1.f);
// (scale: the sum of the parts is multiplied by it before it is added to x)

// cs[t, i] = (cos, sin)(pos[t] * theta^(-2 i / hd)), i < hd/2, angle formed in fp64.
void launch_rope_table(const int32_t* pos, float2* cs, int T, int hd, double theta, hipStream_t st);

// Prefill RoPE + cache append for one layer.  Work is organised in tiles of 64 consecutive
// positions of one sequence: tile i covers positions tile_start[i] .. +63 of sequence tile_seq[i].
struct RopeWriteArgs {
  bf16_t* qkv;            // [T, ld] rows q | k | v ; q and k are rotated in place
  int fp16_input;         // 1: qkv holds fp16 (EPI_STORE_F16 output), 0: bf16
  int ld;                 // row stride in elements
  int q_col, k_col, v_col;  // first column of q / k / v inside a row (q_col < 0: no q heads)
  int n_q_heads, n_kv_heads, hd;
  const float2* cs;       // [T, hd/2]
  const float* q_gamma;   // nullptr or [hd]: every query head is RMS-normalised over hd with this scale before RoPE
  const float* k_gamma;   // the same for the key heads (per-head QK-norm)
  float qk_eps;
  const int32_t* slot;    // [T] cache slot of each packed token
  bf16_t* k_pool;         // this layer's K pool [page][Hkv][P][hd]
  bf16_t* v_pool;
  int page_size;
  int fp16_inplace;       // 1: rotated q and k are written back as fp16 (consumer = attention kernel)
  int cache_only;         // 1: rotated k goes to the cache only, qkv is left as it is (K/V-only projection)
  bf16_t* vT;             // nullptr or [Hkv][hd][Tp]: transposed fp16 copy of V for the attention kernel
  int Tp;
  const int32_t* cu_seqlens;  // [B+1]
  const int32_t* vt_off;      // [B] first column of each sequence in vT (multiple of 64)
  const int32_t* tile_seq;    // [n_tiles]
  const int32_t* tile_start;  // [n_tiles]
  int n_tiles;
  // 8-bit cache: the pools take e4m3 codes, and what the attention kernel reads (the in-place fp16 k and vT) are
  // the values those codes stand for, since every attention reads the stored entries
  KvQuant kvq;
};
void launch_rope_write(const RopeWriteArgs& a, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// bf16 MFMA GEMM (pop_gemm.hip):  C = A[M,K] * W[N,K]^T, fp32 accumulate
// ---------------------------------------------------------------------------------------------
enum GemmEpilogue {
  EPI_STORE_BF16 = 0,  // out bf16 [M, ldc]
  EPI_ADD_F32 = 1,     // out fp32 [M, ldc]: out += C           (residual update)
  EPI_GLU_BF16 = 2,    // W is [2N, K] (gate rows then up rows); out bf16 [M, ldc] = act(gate) * up
  EPI_STORE_F32 = 3,   // out fp32 [M, ldc] = C
  EPI_STORE_F16 = 4,   // out fp16 [M, ldc] = C (saturating), for outputs that stay inside the library
  // The independent KV projections of Sec. 3.3 written straight into the paged cache: W is [2 Dkv, K] (a layer's
  // W^K rows, then its W^V rows, N = 2 Dkv); columns < Dkv are rotated (RoPE on the fp32 accumulators, the two
  // halves of a head are registers of the same lane) and stored as bf16 at the row's slot of the K pool, the
  // others at the same slot of the V pool.  Nothing else is written (out, ldc, strideC are ignored).
  EPI_KV_CACHE = 5
};
// Per batch entry (= pruned layer) of an EPI_KV_CACHE launch: where its entries go and which RoPE table it uses.
struct KvDest {
  bf16_t* k_pool;      // the layer's K pool [page][Hkv][P][hd]; its V pool follows kv_pool_stride elements later
  const float2* cs;    // [M, hd/2] (cos, sin) of every row's position with the layer's RoPE base
};
struct GemmArgs {
  const bf16_t* A;   // [M, lda]
  const bf16_t* W;   // [N, ldw]   (EPI_GLU: [2N, ldw])
  void* out;
  int M, N, K;
  int64_t lda, ldw, ldc;
  int epilogue;
  int act;           // EPI_GLU only: 0 SiLU, 1 tanh-GELU
  // batched form (the K/V-only path): batch b uses A + b*strideA, W_list[b], out + b*strideC elems
  int batch;                 // 1 = plain
  int64_t strideA, strideC;  // in elements
  const bf16_t* const* W_list;  // DEVICE array of `batch` weight pointers, or nullptr for plain
  int64_t strideW;           // without W_list: batch b uses W + b*strideW elements
  // Optional scratch for a deterministic split of K (few rows, long K: the projections of short prompts):
  // the K range is cut into S parts that run as S times as many work-groups, each part writes its fp32
  // partial product here, and a second kernel adds the parts in a fixed order and applies the epilogue.
  float* splitk_ws;          // DEVICE, 16-byte aligned, or nullptr (never split)
  size_t splitk_ws_bytes;
  // With partials_only a split launch stops after the partial products (fp32 [S][M][N] dense in splitk_ws) and
  // leaves adding them and the epilogue to the caller; *split_used receives S (1: not split, or more than 8
  // parts: epilogue applied as usual).
  bool partials_only;
  int* split_used;
  // > 1: split K into exactly this many parts whatever the automatic rule says (the caller has measured that it
  // pays: a long-K projection whose 256 x 256 tiles would fill only a fraction of the chip), if the scratch and K
  // allow it; otherwise the automatic rule applies.
  int force_split;
  // EPI_ADD_F32 with `scaled`: out += scale * C (the virtual gate of Sec. 3.1 on a residual branch); otherwise
  // out += C.  A caller that adds partial products itself (partials_only) applies the scale there.
  bool scaled;
  float scale;
  // EPI_KV_CACHE only
  const KvDest* kv_dest;     // DEVICE [batch]
  const int32_t* kv_slot;    // DEVICE [M] cache slot of every row
  int kv_heads, kv_hd, kv_page_size;
  int64_t kv_pool_stride;    // elements from a layer's K pool to its V pool
  KvQuant kvq;               // bf16 entries or e4m3 codes
};
// Whether launch_gemm can run EPI_KV_CACHE for this shape (otherwise the caller projects to a scratch matrix
// and appends with launch_rope_write): head_dim 64 / 128 / 256 and whole heads per wave tile.
bool gemm_kv_cache_supported(int n_kv_heads, int hd);
inline float residual_scale(const GemmArgs& g) { return g.scaled ? g.scale : 1.f; }
// Returns hipSuccess or the launch error.  Requirements: K % 8 == 0, lda/ldw % 8 == 0,
// A/W 16-byte aligned, ldc % 4 == 0, and every operand below 2^31 bytes.
hipError_t launch_gemm(const GemmArgs& g, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// Causal GQA flash attention over packed variable-length sequences (pop_attention.hip)
// ---------------------------------------------------------------------------------------------
struct AttnPrefillArgs {
  const bf16_t* qkv;  // rotated q and k inside [T, ld], as fp16 (written by launch_rope_write with fp16_inplace)
  int ld, q_col, k_col;
  const bf16_t* vT;   // [Hkv][hd][Tp] fp16
  int Tp;
  bf16_t* out;        // [T, Hq*hd] bf16
  int T, n_q_heads, n_kv_heads, hd;
  int window;         // 0 = global
  const int32_t* cu_seqlens;
  const int32_t* vt_off;
  const int32_t* tile_seq;    // work list: sequence, first position of a 128-row query tile, and
  const int32_t* tile_start;  // first position of a second tile of the same sequence (or -1)
  const int32_t* tile_start2;
  int n_tiles;
};
hipError_t launch_attention_prefill(const AttnPrefillArgs& a, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// Decode-step kernels for the boundary rows (pop_decode.hip); rows = sequences, M <= 8 per launch
// ---------------------------------------------------------------------------------------------
enum GemvEpilogue { GEMV_STORE_F32 = 0, GEMV_ADD_F32 = 1, GEMV_GLU_BF16 = 2 };
// out[m, n] (op)= sum_k x[m,k] * W[n,k], x bf16 [M, K] (M <= 8), W bf16 [N, K] ([2N, K] for GLU).
void launch_gemv(const bf16_t* x, const bf16_t* W, void* out, int M, int N, int K, int64_t ldo,
                 int epilogue, int act, hipStream_t st, float scale = 1.f);   // GEMV_ADD_F32: out += scale * C
// The same with the RMSNorm of the input fused in (Sec. 2.1): xf fp32 [M, K] is normalised with gamma / eps
// inside the kernel (bit-identical to launch_rmsnorm followed by launch_gemv).  Only where
// gemv_norm_supported(M, K): M <= 4 rows whose normalised copies fit 48 KB of LDS.
bool gemv_norm_supported(int M, int K);
void launch_gemv_norm(const float* xf, const float* gamma, float eps, const bf16_t* W, void* out, int M, int N, int K,
                      int64_t ldo, int epilogue, int act, hipStream_t st);
// (n_parts > 1: qkv is given as that many fp32 partial products, part_stride elements apart, which are added in
// index order first: the second kernel of a QKV projection whose K range was split)

// Keys per split of the decode attention: small enough that a 2K-token context already gives every
// CU a work-group (len / 64 splits x KV heads x sequences).
constexpr int kDecodeKeysPerSplit = 64;

// Attention of one query row per sequence over its paged cache entries 0..len-1 (len = pos + 1),
// split over the key range; `part` holds the per-split partial results.
// RoPE of one new token per sequence + cache append: qkv fp32 [B, ld] -> q bf16 [B, Hq*hd] rotated,
// k (rotated) and v stored at slot[b].
void launch_rope_append(const float* qkv, int ld, bf16_t* q_out, int n_q_heads, int n_kv_heads, int hd,
                        const int32_t* pos, const int32_t* slot, double theta, bf16_t* k_pool,
                        bf16_t* v_pool, int page_size, int B, hipStream_t st, const float* q_gamma = nullptr,
                        const float* k_gamma = nullptr, float qk_eps = 0.f, int n_parts = 1, size_t part_stride = 0,
                        KvQuant kvq = KvQuant{0, 1.f, 1.f, 1.f, 1.f});

struct AttnDecodeArgs {
  const bf16_t* q;        // [B, Hq*hd] rotated query rows (launch_rope_append), unused when qkv_raw is given
  const bf16_t* k_pool;   // this layer's pools; with qkv_raw the query position's entry is written by the kernel
  const bf16_t* v_pool;
  const int32_t* block_table;  // [B, max_pages]
  int max_pages, page_size;
  const int32_t* pos;   // [B] position of the query token (attends 0..pos)
  const int32_t* kv_first;  // [B] first position that has an entry in this layer's cache, or nullptr (= 0):
                            // a layer pruned without KV projections holds nothing for the prompt body
  int window;
  int B, n_q_heads, n_kv_heads, hd;
  int n_splits;         // splits of kDecodeKeysPerSplit keys that cover the longest visible key range
  int max_len;          // upper bound of pos+1 over the batch
  float* part;          // [B, Hq, n_splits, hd + 2]
  bf16_t* out;          // [B, Hq*hd]
  KvQuant kvq;          // bf16 entries or e4m3 codes in the pools
  // qkv_raw != nullptr: RoPE + append happen inside this kernel.  The query token's q, k, v rows come as the QKV
  // projection left them, every work-group rotates the query heads it needs, and the work-group whose keys include
  // the query position also forms that position's cache entry (per-head key norm, rotation, rounding to the cache's
  // type), stores it and uses it from registers.  One launch less; pays with few sequences (each of the
  // n_splits x Hkv x B work-groups repeats the preparation of its query heads).
  const float* qkv_raw;     // fp32 [n_parts][B, ld], rows q | k | v; the parts (a split projection) are added
  int ld, n_parts;
  size_t part_stride;       // elements between parts
  const float2* cs;         // [B, hd/2] (cos, sin) of each sequence's query position (launch_rope_table)
  const float* q_gamma;     // per-head QK-norm scales [hd], or nullptr
  const float* k_gamma;
  float qk_eps;
};
void launch_attention_decode(const AttnDecodeArgs& a, hipStream_t st);

// ---------------------------------------------------------------------------------------------
// fp32 instantiation of every step (pop_f32.hip): fp32 weights, activations and cache entries
// ---------------------------------------------------------------------------------------------
namespace f32 {
constexpr int kMaxContext = 15000;  // scores of one query row are held in LDS
enum { EPI_STORE = 0, EPI_ADD = 1, EPI_GLU = 2 };
void launch_embed(const float* table, const int32_t* tokens, const int32_t* row_src, const float* embeds, float* h,
                  int T, int d, hipStream_t st);
// out[t,:] = LN(x[row_idx ? row_idx[t] : t, :])
void launch_rmsnorm(const float* x, const float* gamma, float* out, const int32_t* row_idx, int rows, int d, float eps,
                    hipStream_t st);
// out (op)= A[M,K] W[N,K]^T ; EPI_GLU: W is [2N,K] (gate rows, then up rows)
void launch_gemm(const float* A, int lda, const float* W, int ldw, float* out, int ldc, int M, int N, int K, int epi,
                 int act, hipStream_t st, float scale = 1.f);   // EPI_ADD: out += scale * C
// rotate q (unless q_col < 0) and k of `rows` rows in place, append k, v at slot[row]
void launch_rope_write(float* qkv, int ld, int q_col, int k_col, int v_col, int n_q_heads, int n_kv_heads, int hd,
                       const int32_t* pos, const int32_t* slot, double theta, float* k_pool, float* v_pool, int P,
                       int rows, hipStream_t st, const float* q_gamma = nullptr, const float* k_gamma = nullptr,
                       float qk_eps = 0.f, KvQuant kvq = KvQuant{0, 1.f, 1.f, 1.f, 1.f});
// (kvq.fp8: the fp32 entries stored are the values of the e4m3 codes, i.e. decode(encode(x * inv)) * scale)
// out[r, :] = Attn of row r (sequence row_seq[r], position row_pos[r]) over its cache entries
// kv_first: per sequence, first position that has a cache entry in this layer (nullptr = 0)
hipError_t launch_attention(const float* q, int ldq, int q_col, float* out, const int32_t* row_seq,
                            const int32_t* row_pos, const float* k_pool, const float* v_pool,
                            const int32_t* block_table, int max_pages, int P, int window, const int32_t* kv_first,
                            int rows, int n_q_heads, int n_kv_heads, int hd, int max_len, hipStream_t st);
}  // namespace f32

// Greedy choice of the next token of every sequence from fp32 logits [B, vocab]: tok[b] (device, in/out)
// becomes the index of the largest logit (lowest index on ties), or stays `eos` once it was `eos`
// (step > 0, eos >= 0); the choice is also stored at out[b * out_stride + step].
void launch_argmax(const float* logits, int vocab, int32_t* tok, int32_t* out, int out_stride, int step, int eos,
                   int B, hipStream_t st);

// gather fp32 rows: dst[i,:] = src[idx[i],:]
void launch_gather_rows(const float* src, const int32_t* idx, float* dst, int rows, int d, hipStream_t st);
// dst[idx[r], :] = src[r, :] (fp32 rows of width d; idx must not repeat)
void launch_scatter_rows(const float* src, const int32_t* idx, float* dst, int rows, int d, hipStream_t st);

}  // namespace pop
