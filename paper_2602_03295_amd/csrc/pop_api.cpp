// Host side of the POP prefill library: argument validation, paged-cache slot mapping, workspace
// carving and the per-layer launch schedule (kept layers / KV-only layers / boundary rows) behind
// the C ABI of pop.h.  Everything here is decided before the first launch, so every error path can
// be exercised without a GPU.
#include "../../include/pop.h"
#include "../../include/pop_ops.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "pop_kernels.h"

using pop::bf16_t;

// ----------------------------------------------------------------------------------------- errors
namespace {
thread_local std::string g_last_error;

pop_status fail(pop_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return st;
}
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#define POP_HIP(expr)                                                                              \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return fail(POP_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));    \
  } while (0)

pop_status check_config(const pop_config* c) {
  if (!c) return fail(POP_EINVAL, "config is NULL");
  if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1 ||
      c->d_ffn < 1 || c->vocab < 1)
    return fail(POP_EINVAL, "config has a non-positive size");
  if (c->n_q_heads % c->n_kv_heads) return fail(POP_EINVAL, "n_q_heads %d is not a multiple of n_kv_heads %d",
                                                 c->n_q_heads, c->n_kv_heads);
  if (c->n_q_heads / c->n_kv_heads > 8) return fail(POP_ESHAPE, "more than 8 query heads per KV head");
  if (c->dtype != POP_DTYPE_BF16 && c->dtype != POP_DTYPE_F32) return fail(POP_EINVAL, "unknown dtype %d", c->dtype);
  if (c->act != POP_ACT_SILU && c->act != POP_ACT_GELU_TANH) return fail(POP_EINVAL, "unknown activation %d", c->act);
  if (c->head_dim != 64 && c->head_dim != 128 && c->head_dim != 256)
    return fail(POP_ESHAPE, "head_dim %d is not one of 64, 128, 256", c->head_dim);
  if (c->d_model % 8 || c->d_ffn % 8) return fail(POP_ESHAPE, "d_model and d_ffn must be multiples of 8");
  if (c->d_model > 8192) return fail(POP_ESHAPE, "d_model above 8192");
  if (c->page_size < 1 || c->page_size > 256 || (c->page_size & (c->page_size - 1)))
    return fail(POP_ESHAPE, "page_size %d is not a power of two in 1..256", c->page_size);
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return fail(POP_EINVAL, "bad rms_eps / rope_theta");
  if (c->sliding_window < 0 || c->global_every < 0) return fail(POP_EINVAL, "negative sliding_window / global_every");
  if (c->sliding_window > 0 && c->global_every > 0 && !(c->rope_theta_local > 0.f))
    return fail(POP_EINVAL, "bad rope_theta_local");
  if (c->kv_dtype != POP_KV_BF16 && c->kv_dtype != POP_KV_FP8_E4M3) return fail(POP_EINVAL, "unknown kv_dtype %d", c->kv_dtype);
  if (c->kv_dtype == POP_KV_FP8_E4M3 &&
      !(c->k_scale > 0.f && c->v_scale > 0.f && std::isfinite(c->k_scale) && std::isfinite(c->v_scale)))
    return fail(POP_EINVAL, "k_scale / v_scale of an 8-bit cache must be finite and positive");
  return POP_OK;
}

// Bytes of one cache element: the fp32 checking path keeps fp32 entries (holding the rounded values when the
// cache is 8-bit), the bf16 path bf16 entries or one-byte e4m3 codes.
size_t cache_elem_bytes(const pop_config& c) {
  if (c.dtype == POP_DTYPE_F32) return sizeof(float);
  return c.kv_dtype == POP_KV_FP8_E4M3 ? 1 : sizeof(bf16_t);
}
// How the kernels store and read cache entries.
pop::KvQuant kv_quant(const pop_config& c) {
  pop::KvQuant q{};
  q.fp8 = c.kv_dtype == POP_KV_FP8_E4M3;
  q.k_scale = q.fp8 ? c.k_scale : 1.f;
  q.v_scale = q.fp8 ? c.v_scale : 1.f;
  q.k_inv = 1.f / q.k_scale;
  q.v_inv = 1.f / q.v_scale;
  return q;
}

bool layer_is_global(const pop_config& c, int l /*1-based*/) {
  return c.global_every == 0 || c.sliding_window == 0 || l % c.global_every == 0;
}
}  // namespace

namespace pop {
int record_error(int status, const char* msg) {
  g_last_error = msg ? msg : "";
  return status;
}
}  // namespace pop

struct TimedSpan {
  int kind;
  hipEvent_t start, stop;
};

struct pop_model {
  pop_config cfg;
  pop_weights w;
  std::vector<pop_layer_weights> layers;
  int Dq, Dkv, Dqkv;
  // optional per-step timing (pop_timing_enable)
  bool timing = false;
  std::vector<TimedSpan> spans;      // recorded since the last read
  std::vector<hipEvent_t> free_events;
  hipEvent_t take_event() {
    if (!free_events.empty()) {
      hipEvent_t e = free_events.back();
      free_events.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};

namespace {
// Records an event pair around the launches issued during its lifetime (only while timing is on).
struct StepTimer {
  pop_model* m;
  hipStream_t st;
  hipEvent_t stop = nullptr;
  StepTimer(pop_model* model, hipStream_t stream, int kind) : m(model), st(stream) {
    if (!m->timing) return;
    hipEvent_t start = m->take_event();
    stop = m->take_event();
    if (!start || !stop) { stop = nullptr; return; }
    (void)hipEventRecord(start, st);
    m->spans.push_back(TimedSpan{kind, start, stop});
  }
  ~StepTimer() {
    if (stop) (void)hipEventRecord(stop, st);
  }
};
}  // namespace

struct pop_cache {
  pop_config cfg;
  bf16_t* pool;                      // fp32 configs: the same bytes viewed as float (see k_pool_f32)
  size_t bytes;
  int n_pages, max_seqs, max_pages;
  int n_seqs;                        // live sequences
  std::vector<int32_t> seq_lens;     // [max_seqs]
  std::vector<int32_t> block_table;  // [max_seqs][max_pages]
  // First position that has an entry, per layer and sequence: 0 unless the layer was pruned without
  // KV projections in the prefill, in which case nothing exists below the first full-depth token.
  std::vector<int32_t> kv_first;     // [n_layers][max_seqs]
  bool any_kv_first = false;
  // Two pinned host buffers that the calls' metadata is copied to the device from, in turn (allocated at the
  // first call that needs them).  A copy from pageable memory may still be reading its source after
  // hipMemcpyAsync returns; these buffers outlive the call, and an event per buffer says when it is free again.
  void* stage_host[2] = {nullptr, nullptr};
  size_t stage_bytes[2] = {0, 0};
  hipEvent_t stage_done[2] = {nullptr, nullptr};
  unsigned stage_turn = 0;
  size_t layer_stride() const {      // elements between the K pools of consecutive layers
    return 2 * pool_stride();
  }
  size_t pool_stride() const {
    return (size_t)n_pages * cfg.n_kv_heads * cfg.page_size * cfg.head_dim;
  }
  // (typed as bf16_t* for the kernels' argument lists; with an 8-bit cache the address is that of one-byte codes)
  size_t esz() const { return cache_elem_bytes(cfg); }
  bf16_t* k_pool(int l0) const {
    return reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(pool) + (size_t)l0 * layer_stride() * esz());
  }
  bf16_t* v_pool(int l0) const {
    return reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(k_pool(l0)) + pool_stride() * esz());
  }
  float* k_pool_f32(int l0) const { return reinterpret_cast<float*>(pool) + (size_t)l0 * layer_stride(); }
  float* v_pool_f32(int l0) const { return k_pool_f32(l0) + pool_stride(); }
};

// ----------------------------------------------------------------------------------------- workspace
namespace {

constexpr int kKvChunk = 8;  // pruned layers projected per batched GEMM

// Parts into which the down projection (K = d_ffn) of T prompt rows splits its K range.  With 256 x 256 tiles
// the projection has ceil(T / 256) * ceil(d / 256) tiles; when that is half the chip or less, and K is long, as
// many work-groups again per part run the tiles' K ranges side by side (measured at 2048 rows of the Llama-3.1-8B
// shape: 128 tiles, 2 parts).  The parts are added in index order by the kernel that normalises the result for the
// next layer, or by the split's own second kernel.  1 = no split (few rows use the automatic rule of the GEMM).
int down_split_parts(int T, int d, int f) {
#ifdef POP_NO_DOWN_SPLIT      // (experiments only: a build without it, for A/B timing)
  return 1;
#endif
  if (T <= 512 || f < 8192) return 1;
  const long long tiles = (long long)((T + 255) / 256) * ((d + 255) / 256);
  int S = 1;
  while (S < 8 && tiles * S * 2 <= 256 && f % (S * 2 * 64) == 0 && f / (S * 2 * 64) >= 8) S *= 2;
  return S;
}

struct Workspace {
  // int32 meta (one upload per call)
  size_t meta_bytes;
  size_t o_tokens, o_row_src, o_pos, o_slot, o_cu, o_vt_off, o_t64_seq, o_t64_start, o_ta_seq, o_ta_start, o_ta_start2,
      o_bnd_row, o_bnd_pos, o_bnd_slot, o_bt, o_kv_first, o_wl_full, o_wl_tail, o_kvd_full, o_kvd_tail, o_tr_row, o_tr_pos, o_tr_slot,
      o_tr_cu, o_tr_t64_seq, o_tr_t64_start;
  // device buffers
  size_t o_h, o_a, o_qkv, o_attn, o_u, o_vT, o_cs_g, o_cs_l, o_cs_tail, o_a_multi, o_kv_out;
  size_t o_dcs_g, o_dcs_l;   // (cos, sin) of the decode-style rows' positions, [B][hd/2] per RoPE base
  size_t o_xb, o_ab, o_qkvb, o_qb, o_attnb, o_ub, o_part, o_splitk;
  size_t splitk_bytes;
  size_t total;
  int Tp_max, nt64_max, nta_max, n_splits_max;
};

Workspace carve(const pop_config& c, int T, int B, int maxp) {
  Workspace w{};
  const size_t d = c.d_model, hd = c.head_dim;
  const size_t Dq = (size_t)c.n_q_heads * hd, Dkv = (size_t)c.n_kv_heads * hd, Dqkv = Dq + 2 * Dkv;
  const size_t f = c.d_ffn;
  w.Tp_max = (int)round_up((size_t)T + 63 * (size_t)B, 64);
  w.nt64_max = T / 64 + B;
  w.nta_max = T / 128 + B;
  const long long max_len = (long long)maxp * c.page_size;
  w.n_splits_max = (int)std::max<long long>(1, (max_len + pop::kDecodeKeysPerSplit - 1) / pop::kDecodeKeysPerSplit);
  size_t o = 0;
  auto take = [&](size_t bytes) {
    const size_t at = o;
    o += round_up(bytes, 256);
    return at;
  };
  w.o_tokens = take(4 * (size_t)T);
  w.o_row_src = take(4 * (size_t)T);
  w.o_pos = take(4 * (size_t)T);
  w.o_slot = take(4 * (size_t)T);
  w.o_cu = take(4 * ((size_t)B + 1));
  w.o_vt_off = take(4 * (size_t)B);
  w.o_t64_seq = take(4 * (size_t)w.nt64_max);
  w.o_t64_start = take(4 * (size_t)w.nt64_max);
  w.o_ta_seq = take(4 * (size_t)w.nta_max);
  w.o_ta_start = take(4 * (size_t)w.nta_max);
  w.o_ta_start2 = take(4 * (size_t)w.nta_max);
  w.o_bnd_row = take(4 * (size_t)B);
  w.o_bnd_pos = take(4 * (size_t)B);
  w.o_bnd_slot = take(4 * (size_t)B);
  w.o_bt = take(4 * (size_t)B * maxp);
  w.o_kv_first = take(4 * (size_t)c.n_layers * B);
  w.o_wl_full = take(8 * (size_t)c.n_layers);
  w.o_wl_tail = take(8 * (size_t)c.n_layers);
  w.o_kvd_full = take(sizeof(pop::KvDest) * (size_t)c.n_layers);
  w.o_kvd_tail = take(sizeof(pop::KvDest) * (size_t)c.n_layers);
  w.o_tr_row = take(4 * (size_t)T);
  w.o_tr_pos = take(4 * (size_t)T);
  w.o_tr_slot = take(4 * (size_t)T);
  w.o_tr_cu = take(4 * ((size_t)B + 1));
  w.o_tr_t64_seq = take(4 * (size_t)w.nt64_max);
  w.o_tr_t64_start = take(4 * (size_t)w.nt64_max);
  w.meta_bytes = o;
  w.o_h = take(4 * (size_t)T * d);
  w.o_a = take(2 * (size_t)T * d);
  w.o_qkv = take(2 * (size_t)T * Dqkv);
  w.o_attn = take(2 * (size_t)T * Dq);
  w.o_u = take(2 * (size_t)T * f);
  w.o_vT = take(2 * Dkv * (size_t)w.Tp_max);
  w.o_cs_g = take(8 * (size_t)T * (hd / 2));
  w.o_cs_l = take(8 * (size_t)T * (hd / 2));
  w.o_cs_tail = c.sliding_window > 0 ? take(8 * (size_t)T * (hd / 2)) : o;
  w.o_dcs_g = take(8 * (size_t)B * (hd / 2));
  w.o_dcs_l = take(8 * (size_t)B * (hd / 2));
  const size_t rc = std::min(kKvChunk, c.n_layers);
  w.o_a_multi = take(2 * rc * (size_t)T * d);
  w.o_kv_out = take(2 * rc * (size_t)T * 2 * Dkv);
  w.o_xb = take(4 * (size_t)B * d);
  w.o_ab = take(2 * (size_t)B * std::max(d, Dq));
  w.o_qkvb = take(4 * (size_t)B * Dqkv);
  w.o_qb = take(2 * (size_t)B * Dq);
  w.o_attnb = take(2 * (size_t)B * Dq);
  w.o_ub = take(2 * (size_t)B * f);
  w.o_part = take(4 * (size_t)B * c.n_q_heads * w.n_splits_max * (hd + 2));
  // fp32 partial products of a projection whose K range is split (short prompts only)
  // (all packed rows of a short batch; otherwise the boundary rows, which are projected on their own)
  const size_t split_rows = T <= 512 ? (size_t)T : (B <= 512 ? (size_t)B : 0);
  w.splitk_bytes = 8 * 4 * split_rows * std::max(Dqkv, d);
  // (or the parts of the down projection of a long prompt)
  if (const int S = down_split_parts(T, (int)d, (int)f); S > 1)
    w.splitk_bytes = std::max(w.splitk_bytes, 4 * (size_t)S * (size_t)T * d);
  w.o_splitk = take(w.splitk_bytes);
  w.total = o;
  return w;
}

// Copies `bytes` of host metadata to the device on the stream, through one of the cache's pinned buffers.
pop_status upload_meta(pop_cache* c, void* dev_dst, const void* src, size_t bytes, hipStream_t st) {
  if (bytes == 0) return POP_OK;
  const unsigned k = c->stage_turn++ & 1;
  if (c->stage_done[k]) POP_HIP(hipEventSynchronize(c->stage_done[k]));   // the buffer's previous copy has been read
  if (c->stage_bytes[k] < bytes) {
    if (c->stage_host[k]) (void)hipHostFree(c->stage_host[k]);
    c->stage_host[k] = nullptr;
    c->stage_bytes[k] = 0;
    const size_t want = round_up(bytes, (size_t)1 << 16);
    if (hipHostMalloc(&c->stage_host[k], want, hipHostMallocDefault) == hipSuccess) c->stage_bytes[k] = want;
    else { c->stage_host[k] = nullptr; (void)hipGetLastError(); }
  }
  if (c->stage_host[k] && !c->stage_done[k] &&
      hipEventCreateWithFlags(&c->stage_done[k], hipEventDisableTiming) != hipSuccess) {
    c->stage_done[k] = nullptr;
    (void)hipGetLastError();
  }
  if (!c->stage_host[k] || !c->stage_done[k]) {
    // no pinned memory to be had: copy from the caller's buffer and wait until it has been read
    POP_HIP(hipMemcpyAsync(dev_dst, src, bytes, hipMemcpyHostToDevice, st));
    POP_HIP(hipStreamSynchronize(st));
    return POP_OK;
  }
  std::memcpy(c->stage_host[k], src, bytes);
  POP_HIP(hipMemcpyAsync(dev_dst, c->stage_host[k], bytes, hipMemcpyHostToDevice, st));
  POP_HIP(hipEventRecord(c->stage_done[k], st));
  return POP_OK;
}

template <typename T>
T* at(void* base, size_t off) {
  return reinterpret_cast<T*>(reinterpret_cast<char*>(base) + off);
}

// Slot mapping and its validation (shared by pop_slot_map and pop_prefill).
pop_status slot_map_impl(const int32_t* cu, int n_seqs, const int32_t* bt, int maxp, int P, int n_pages,
                         int32_t* slots, int extra_positions /* room checked beyond each length */) {
  if (!cu || !bt) return fail(POP_EINVAL, "cu_seqlens / block_table is NULL");
  if (n_seqs < 1) return fail(POP_EINVAL, "n_seqs %d < 1", n_seqs);
  if (maxp < 1 || P < 1 || n_pages < 1) return fail(POP_EINVAL, "bad page geometry");
  if (cu[0] != 0) return fail(POP_EINVAL, "cu_seqlens[0] = %d, expected 0", cu[0]);
  std::vector<uint8_t> used((size_t)n_pages, 0);
  for (int b = 0; b < n_seqs; ++b) {
    const long long len = (long long)cu[b + 1] - cu[b];
    if (len < 1) return fail(POP_EINVAL, "sequence %d has length %lld (cu_seqlens must be strictly increasing)", b, len);
    const long long need = (len + extra_positions + P - 1) / P;
    if (need > maxp) return fail(POP_ENOSPACE, "sequence %d needs %lld pages, the table has %d columns", b, need, maxp);
    for (int pg = 0; pg < maxp; ++pg) {
      const int id = bt[(size_t)b * maxp + pg];
      if (id < 0) {
        if (pg < need) return fail(POP_ENOSPACE, "sequence %d has no page for position %d", b, pg * P);
        continue;
      }
      if (id >= n_pages) return fail(POP_EINVAL, "page id %d of sequence %d is outside [0, %d)", id, b, n_pages);
      if (used[id]) return fail(POP_EINVAL, "page %d is assigned twice", id);
      used[id] = 1;
    }
    if (slots)
      for (long long t = 0; t < len; ++t)
        slots[cu[b] + t] = bt[(size_t)b * maxp + t / P] * P + (int)(t % P);
  }
  return POP_OK;
}

// Work list of the prefill attention kernel.  A work-group processes one or two query tiles of 128
// rows of one sequence: the k-th latest tile (most keys) is paired with the k-th earliest (fewest),
// so every work-group of a sequence sees the same number of key tiles and the causal triangle is
// balanced.  Longer sequences (more work per pair) come first.  Returns the number of entries.
int build_attention_work(const int32_t* cu, int B, int32_t* seq_out, int32_t* start_out, int32_t* start2_out) {
  struct Item { int work, seq, a, b; };
  std::vector<Item> items;
  for (int b = 0; b < B; ++b) {
    const int len = cu[b + 1] - cu[b];
    const int nt = (len + 127) / 128;
    for (int k = 0; k < (nt + 1) / 2; ++k) {
      const int heavy = nt - 1 - k, light = k;
      items.push_back(Item{heavy == light ? heavy + 1 : nt + 1, b, heavy * 128, heavy == light ? -1 : light * 128});
    }
  }
  std::stable_sort(items.begin(), items.end(), [](const Item& x, const Item& y) { return x.work > y.work; });
  int n = 0;
  for (const Item& it : items) {
    seq_out[n] = it.seq;
    start_out[n] = it.a;
    start2_out[n++] = it.b;
  }
  return n;
}

struct LayerCtx {
  const pop_model* m;
  pop_cache* c;
  void* ws;
  const Workspace* w;
  hipStream_t st;
  const int32_t* kv_first = nullptr;  // DEVICE [n_layers][B] or nullptr (every layer holds every position)
  // The norm scale with which the bf16 scratch rows `ab` hold RMSNorm(xb), or nullptr when they do not: a split
  // projection with a residual epilogue normalises its result for the next projection in its second kernel.
  mutable const float* ab_gamma = nullptr;
  const float* gates = nullptr;       // HOST [n_layers] virtual gates of the stage this context runs, or nullptr
  float gate(int l /*1-based*/) const { return gates ? gates[l - 1] : 1.f; }
};

// (cos, sin) tables of the B decode-style rows at positions pos[0..B-1], one per RoPE base in use: what the decode
// attention kernel rotates the query token's q and k with.  Once per pass over the layers.
void decode_rope_tables(const LayerCtx& x, const int32_t* pos, int B) {
  const pop_config& c = x.m->cfg;
  pop::launch_rope_table(pos, at<float2>(x.ws, x.w->o_dcs_g), B, c.head_dim, (double)c.rope_theta, x.st);
  bool any_local = false;
  for (int l = 1; l <= c.n_layers; ++l) any_local = any_local || !layer_is_global(c, l);
  if (any_local)
    pop::launch_rope_table(pos, at<float2>(x.ws, x.w->o_dcs_l), B, c.head_dim, (double)c.rope_theta_local, x.st);
}

// The prefill's pruning, resolved from the arguments (Sec. 2.2: a skip set; Sec. 3.3: applied to the
// body tokens of the prefill only).
struct PrunePlan {
  std::vector<char> pruned;  // [n_layers + 2], 1-based
  bool kv_projection;        // pruned layers store independent KV projections of the body
  bool window_writes;        // pruned sliding-window layers store only what a later token can see
  int n_pruned;
};

// Tail rows of every sequence that a pruned sliding-window layer still has to store (window_kv_writes):
// positions first_b .. len_b - 1 with first_b = max(0, p0 - W + 1), p0 the position of the first token that
// runs the full model on this cache.  Packed like the prompt itself.
struct TailRows {
  std::vector<int32_t> row, pos, slot, cu, t64_seq, t64_start;
  int n = 0;
};

TailRows tail_rows(const pop_config& cfg, const pop_prefill_args* a, const std::vector<int32_t>& slots) {
  TailRows t;
  const int B = a->n_seqs, W = cfg.sliding_window;
  t.cu.push_back(0);
  for (int b = 0; b < B; ++b) {
    const int s0 = a->cu_seqlens[b], len = a->cu_seqlens[b + 1] - s0;
    const int p0 = a->mode == POP_MODE_POP ? len - 1 : len;
    const int first = std::min(len, std::max(0, p0 - W + 1));
    for (int p = first; p < len; ++p) {
      t.row.push_back(s0 + p);
      t.pos.push_back(p);
      t.slot.push_back(slots[(size_t)s0 + p]);
    }
    const int cnt = len - first;
    for (int q0 = 0; q0 < cnt; q0 += 64) {
      t.t64_seq.push_back(b);
      t.t64_start.push_back(q0);
    }
    t.cu.push_back(t.cu.back() + cnt);
  }
  t.n = t.cu.back();
  return t;
}

pop_status make_plan(const pop_config& cfg, const pop_prefill_args* a, PrunePlan* plan) {
  const int L = cfg.n_layers;
  if (a->mode != POP_MODE_POP && a->mode != POP_MODE_BODY_ONLY && a->mode != POP_MODE_NO_BOUNDARY)
    return fail(POP_EINVAL, "unknown mode %d", a->mode);
  if (a->no_kv_projection != 0 && a->no_kv_projection != 1)
    return fail(POP_EINVAL, "no_kv_projection must be 0 or 1, got %d", a->no_kv_projection);
  plan->pruned.assign((size_t)L + 2, 0);
  if (a->window_kv_writes != 0 && a->window_kv_writes != 1)
    return fail(POP_EINVAL, "window_kv_writes must be 0 or 1, got %d", a->window_kv_writes);
  if (a->gates) {
    if (a->mode == POP_MODE_POP)
      return fail(POP_EINVAL, "gates are prefill-stage gates: use POP_MODE_BODY_ONLY (and pop_decode_step_gated for "
                              "the last token) or POP_MODE_NO_BOUNDARY");
    for (int l = 0; l < L; ++l)
      if (!std::isfinite(a->gates[l])) return fail(POP_EINVAL, "gates[%d] is not finite", l);
  }
  plan->kv_projection = a->no_kv_projection == 0;
  plan->window_writes = a->window_kv_writes == 1 && cfg.sliding_window > 0 && cfg.global_every > 0;
  plan->n_pruned = 0;
  if (a->skip_layers) {
    if (a->n_skip < 0 || a->n_skip > L) return fail(POP_EINVAL, "n_skip %d outside [0, %d]", a->n_skip, L);
    for (int i = 0; i < a->n_skip; ++i) {
      const int l = a->skip_layers[i];
      if (l < 1 || l > L) return fail(POP_EINVAL, "skip_layers[%d] = %d outside [1, %d]", i, l, L);
      if (i > 0 && l <= a->skip_layers[i - 1])
        return fail(POP_EINVAL, "skip_layers must be strictly increasing (entry %d)", i);
      plan->pruned[l] = 1;
    }
    plan->n_pruned = a->n_skip;
  } else {
    if (a->n_skip != 0) return fail(POP_EINVAL, "n_skip %d given without skip_layers", a->n_skip);
    if (a->l_keep < 0 || a->l_keep > L) return fail(POP_EINVAL, "l_keep %d outside [0, %d]", a->l_keep, L);
    for (int l = a->l_keep + 1; l <= L; ++l) plan->pruned[l] = 1;
    plan->n_pruned = L - a->l_keep;
  }
  return POP_OK;
}

// Records which positions exist per layer after this prefill and writes the device copy [L][B].
void record_kv_first(pop_cache* c, const pop_prefill_args* a, const PrunePlan& plan, int32_t* meta_out) {
  const int L = c->cfg.n_layers, B = a->n_seqs;
  std::fill(c->kv_first.begin(), c->kv_first.end(), 0);
  c->any_kv_first = !plan.kv_projection && plan.n_pruned > 0;
  for (int l = 1; l <= L; ++l)
    for (int b = 0; b < B; ++b) {
      const int len = a->cu_seqlens[b + 1] - a->cu_seqlens[b];
      const int first = (plan.pruned[l] && !plan.kv_projection) ? len - (a->mode == POP_MODE_POP ? 1 : 0) : 0;
      c->kv_first[(size_t)(l - 1) * c->max_seqs + b] = first;
      meta_out[(size_t)(l - 1) * B + b] = first;
    }
}

// Projection of the B rows of a decode-style layer.  The GEMV kernel streams every weight row once per row
// group and is the fastest form for one or a few rows; from kRowsForGemm rows on the tiled MFMA GEMM with
// its small tiles (and the split of a long K) reads the weights faster than the GEMV kernel's 8-row form
// (measured on decode steps of 8 sequences at the Llama-3.1-8B shape: 4.75 ms per step through the tiled GEMM, 7.6 ms
// through the 8-row GEMV, whose 256 work-groups for 4096 output rows leave a CU with four waves' worth of loads).
constexpr int kRowsForGemm = 5;
constexpr int rows_for_gemm() { return kRowsForGemm; }
constexpr int kFusedAppendRows = 4;   // decode-style rows up to which the attention kernel does RoPE + append itself

// parts_out (optional): the caller can add partial products itself.  If the K range was split, *parts_out receives
// the number of parts (fp32 [parts][B][N] dense at the split scratch of the workspace) and `out` is not written;
// otherwise it receives 1.
pop_status few_rows_projection(const LayerCtx& x, const bf16_t* in, const void* W, void* out, int B, int N, int K,
                               int ldo, int gemv_epi, int act, int* parts_out = nullptr) {
  if (parts_out) *parts_out = 1;
  if (B < rows_for_gemm() || ldo % 4) {   // (the tiled GEMM stores four columns at a time)
    pop::launch_gemv(in, (const bf16_t*)W, out, B, N, K, ldo, gemv_epi, act, x.st);
    return POP_OK;
  }
  pop::GemmArgs g{};
  g.batch = 1;
  g.A = in; g.lda = K; g.W = (const bf16_t*)W; g.ldw = K; g.out = out; g.ldc = ldo;
  g.M = B; g.N = N; g.K = K; g.act = act;
  g.epilogue = gemv_epi == pop::GEMV_STORE_F32 ? pop::EPI_STORE_F32
               : gemv_epi == pop::GEMV_ADD_F32 ? pop::EPI_ADD_F32 : pop::EPI_GLU_BF16;
  g.splitk_ws = x.w->splitk_bytes ? at<float>(x.ws, x.w->o_splitk) : nullptr;
  g.splitk_ws_bytes = x.w->splitk_bytes;
  g.partials_only = parts_out != nullptr;
  g.split_used = parts_out;
  hipError_t e = pop::launch_gemm(g, x.st);
  if (e != hipSuccess) return fail(POP_EHIP, "projection launch failed: %s", hipGetErrorString(e));
  return POP_OK;
}

// The same for fp32 rows that are RMS-normalised first (Sec. 2.1): with a few rows the GEMV kernel normalises
// them itself; otherwise the norm kernel writes bf16 rows to `normed` and the projection reads those.
pop_status normed_few_rows_projection(const LayerCtx& x, float* rows, const float* gamma, bf16_t* normed, const void* W,
                                      void* out, int B, int N, int K, int ldo, int gemv_epi, int act,
                                      int* parts_out = nullptr) {
  if (parts_out) *parts_out = 1;
  const float eps = x.m->cfg.rms_eps;
  if (x.ab_gamma == gamma && gamma != nullptr)   // the previous projection's second kernel left them in `normed`
    return few_rows_projection(x, normed, W, out, B, N, K, ldo, gemv_epi, act, parts_out);
  if (B < rows_for_gemm() && pop::gemv_norm_supported(B, K)) {
    pop::launch_gemv_norm(rows, gamma, eps, (const bf16_t*)W, out, B, N, K, ldo, gemv_epi, act, x.st);
    return POP_OK;
  }
  pop::launch_rmsnorm(rows, nullptr, nullptr, gamma, normed, nullptr, B, K, eps, x.st);
  return few_rows_projection(x, normed, W, out, B, N, K, ldo, gemv_epi, act, parts_out);
}

// xb += in W^T for the B rows of a decode-style layer.  With next_gamma the caller announces the norm scale of the
// projection that follows: when this one runs as a split GEMM its second kernel then also writes
// RMSNorm(xb; next_gamma) to ab (and records that in x.ab_gamma), which saves that projection's norm launch.
pop_status residual_few_rows_projection(const LayerCtx& x, const bf16_t* in, const void* W, int B, int N, int K,
                                        const float* next_gamma, float scale /* the layer's virtual gate */) {
  float* xb = at<float>(x.ws, x.w->o_xb);
  x.ab_gamma = nullptr;
  if (B < rows_for_gemm() || N % 4) {
    pop::launch_gemv(in, (const bf16_t*)W, xb, B, N, K, N, pop::GEMV_ADD_F32, 0, x.st, scale);
    return POP_OK;
  }
  pop::GemmArgs g{};
  g.batch = 1;
  g.A = in; g.lda = K; g.W = (const bf16_t*)W; g.ldw = K; g.out = xb; g.ldc = N;
  g.M = B; g.N = N; g.K = K;
  g.epilogue = pop::EPI_ADD_F32;
  g.scaled = true;
  g.scale = scale;
  g.splitk_ws = x.w->splitk_bytes ? at<float>(x.ws, x.w->o_splitk) : nullptr;
  g.splitk_ws_bytes = x.w->splitk_bytes;
  int S = 1;
  g.partials_only = next_gamma != nullptr && N <= 8192;
  g.split_used = &S;
  hipError_t e = pop::launch_gemm(g, x.st);
  if (e != hipSuccess) return fail(POP_EHIP, "projection launch failed: %s", hipGetErrorString(e));
  if (g.partials_only && S > 1) {
    pop::launch_add_parts_rmsnorm(xb, g.splitk_ws, S, (size_t)B * N, next_gamma, at<bf16_t>(x.ws, x.w->o_ab), B, N,
                                  x.m->cfg.rms_eps, x.st, scale);
    x.ab_gamma = next_gamma;
  }
  return POP_OK;
}

// One decode-style layer for B rows held in xb (fp32 [B, d]); pos/slot are device arrays [B].
// next_gamma: norm scale of the projection that will read xb next (the next layer's input norm, the final norm),
// or nullptr when something else happens to the rows first.
pop_status decode_layer(const LayerCtx& x, int l /*1-based*/, int B, const int32_t* pos, const int32_t* slot,
                        int max_len, const float* next_gamma) {
  const pop_config& c = x.m->cfg;
  const pop_layer_weights& lw = x.m->layers[l - 1];
  const int d = c.d_model, f = c.d_ffn, Dq = x.m->Dq, Dqkv = x.m->Dqkv;
  float* xb = at<float>(x.ws, x.w->o_xb);
  bf16_t* ab = at<bf16_t>(x.ws, x.w->o_ab);
  float* qkvb = at<float>(x.ws, x.w->o_qkvb);
  bf16_t* attnb = at<bf16_t>(x.ws, x.w->o_attnb);
  bf16_t* ub = at<bf16_t>(x.ws, x.w->o_ub);
  const bool glob = layer_is_global(c, l);
  // Up to kFusedAppendRows rows: RoPE and the append of the new entries happen inside the attention kernel (one
  // launch less; decode_rope_tables has run for these positions, the slot is implied by the block table).  With more
  // rows every one of the n_splits x Hkv x B work-groups would repeat the preparation of its query heads, and a
  // separate kernel that does it once per row and head is faster (measured at 8 sequences of 2048 tokens: attention
  // 33.7 us + 4.9 us for the projection's own reduction of its K parts, against 24.5 us + 4.8 us for that kernel,
  // which also adds the parts).
  const bool fused_append = B <= kFusedAppendRows;
  int qkv_parts = 1;
  if (pop_status s = normed_few_rows_projection(x, xb, (const float*)lw.norm_in, ab, lw.wqkv, qkvb, B, Dqkv, d, Dqkv,
                                                pop::GEMV_STORE_F32, 0, fused_append ? nullptr : &qkv_parts))
    return s;
  pop::AttnDecodeArgs ad{};
  if (fused_append) {
    ad.qkv_raw = qkvb;
    ad.ld = Dqkv; ad.n_parts = 1; ad.part_stride = 0;
    ad.cs = at<float2>(x.ws, glob ? x.w->o_dcs_g : x.w->o_dcs_l);
    ad.q_gamma = (const float*)lw.q_norm; ad.k_gamma = (const float*)lw.k_norm; ad.qk_eps = c.rms_eps;
  } else {
    bf16_t* qb = at<bf16_t>(x.ws, x.w->o_qb);
    pop::launch_rope_append(qkv_parts > 1 ? at<float>(x.ws, x.w->o_splitk) : qkvb, Dqkv, qb, c.n_q_heads, c.n_kv_heads,
                            c.head_dim, pos, slot, glob ? (double)c.rope_theta : (double)c.rope_theta_local,
                            x.c->k_pool(l - 1), x.c->v_pool(l - 1), c.page_size, B, x.st, (const float*)lw.q_norm,
                            (const float*)lw.k_norm, c.rms_eps, qkv_parts, (size_t)B * Dqkv, kv_quant(c));
    ad.q = qb;
  }
  ad.k_pool = x.c->k_pool(l - 1);
  ad.v_pool = x.c->v_pool(l - 1);
  ad.block_table = at<int32_t>(x.ws, x.w->o_bt);
  ad.max_pages = x.c->max_pages;
  ad.page_size = c.page_size;
  ad.pos = pos;
  ad.kv_first = x.kv_first ? x.kv_first + (size_t)(l - 1) * B : nullptr;
  ad.window = glob ? 0 : c.sliding_window;
  ad.B = B;
  ad.n_q_heads = c.n_q_heads;
  ad.n_kv_heads = c.n_kv_heads;
  ad.hd = c.head_dim;
  const int span = ad.window > 0 ? std::min(max_len, ad.window) : max_len;
  ad.n_splits = std::max(1, (span + pop::kDecodeKeysPerSplit - 1) / pop::kDecodeKeysPerSplit);
  ad.max_len = max_len;
  ad.part = at<float>(x.ws, x.w->o_part);
  ad.out = attnb;
  ad.kvq = kv_quant(c);
  pop::launch_attention_decode(ad, x.st);
  if (pop_status s = residual_few_rows_projection(x, attnb, lw.wo, B, d, Dq, (const float*)lw.norm_post, x.gate(l))) return s;
  if (pop_status s = normed_few_rows_projection(x, xb, (const float*)lw.norm_post, ab, lw.w_gate_up, ub, B, f, d, f,
                                                pop::GEMV_GLU_BF16, c.act))
    return s;
  if (pop_status s = residual_few_rows_projection(x, ub, lw.w_down, B, d, f, next_gamma, x.gate(l))) return s;
  POP_HIP(hipGetLastError());
  return POP_OK;
}

pop_status lm_head(const LayerCtx& x, int B, float* dev_logits) {
  const pop_config& c = x.m->cfg;
  float* xb = at<float>(x.ws, x.w->o_xb);
  bf16_t* ab = at<bf16_t>(x.ws, x.w->o_ab);
  if (pop_status s = normed_few_rows_projection(x, xb, (const float*)x.m->w.final_norm, ab, x.m->w.lm_head, dev_logits,
                                                B, c.vocab, c.d_model, c.vocab, pop::GEMV_STORE_F32, 0))
    return s;
  POP_HIP(hipGetLastError());
  return POP_OK;
}

// ------------------------------------------------------------------------------- fp32 instantiation
struct WorkspaceF32 {
  size_t meta_bytes;
  size_t o_tokens, o_row_src, o_pos, o_slot, o_row_seq, o_bnd_row, o_bnd_pos, o_bnd_slot, o_bnd_seq, o_bt, o_kv_first, o_tr_row, o_tr_pos,
      o_tr_slot;
  size_t o_h, o_a, o_qkv, o_attn, o_u, o_xb, o_ab, o_qkvb, o_attnb, o_ub;
  size_t total;
};

WorkspaceF32 carve_f32(const pop_config& c, int T, int B, int maxp) {
  WorkspaceF32 w{};
  const size_t d = c.d_model, hd = c.head_dim, f = c.d_ffn;
  const size_t Dq = (size_t)c.n_q_heads * hd, Dkv = (size_t)c.n_kv_heads * hd, Dqkv = Dq + 2 * Dkv;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    const size_t at = o;
    o += round_up(bytes, 256);
    return at;
  };
  w.o_tokens = take(4 * (size_t)T);
  w.o_row_src = take(4 * (size_t)T);
  w.o_pos = take(4 * (size_t)T);
  w.o_slot = take(4 * (size_t)T);
  w.o_row_seq = take(4 * (size_t)T);
  w.o_bnd_row = take(4 * (size_t)B);
  w.o_bnd_pos = take(4 * (size_t)B);
  w.o_bnd_slot = take(4 * (size_t)B);
  w.o_bnd_seq = take(4 * (size_t)B);
  w.o_bt = take(4 * (size_t)B * maxp);
  w.o_kv_first = take(4 * (size_t)c.n_layers * B);
  w.o_tr_row = take(4 * (size_t)T);
  w.o_tr_pos = take(4 * (size_t)T);
  w.o_tr_slot = take(4 * (size_t)T);
  w.meta_bytes = o;
  w.o_h = take(4 * (size_t)T * d);
  w.o_a = take(4 * (size_t)T * d);
  w.o_qkv = take(4 * (size_t)T * Dqkv);
  w.o_attn = take(4 * (size_t)T * Dq);
  w.o_u = take(4 * (size_t)T * f);
  w.o_xb = take(4 * (size_t)B * d);
  w.o_ab = take(4 * (size_t)B * d);
  w.o_qkvb = take(4 * (size_t)B * Dqkv);
  w.o_attnb = take(4 * (size_t)B * Dq);
  w.o_ub = take(4 * (size_t)B * f);
  w.total = o;
  return w;
}

struct CtxF32 {
  const pop_model* m;
  pop_cache* c;
  void* ws;
  const WorkspaceF32* w;
  hipStream_t st;
  const int32_t* kv_first = nullptr;  // DEVICE [n_layers][B] or nullptr
  int B = 0;                          // sequences (row stride of kv_first)
  const float* gates = nullptr;       // HOST [n_layers] virtual gates of the stage this context runs, or nullptr
  float gate(int l /*1-based*/) const { return gates ? gates[l - 1] : 1.f; }
};

// One layer of Sec. 2.1 for `rows` rows of x (fp32 [rows, d], updated in place); a / qkv / attn / u are
// scratch of matching height.  row_seq / pos / slot are device arrays [rows].
pop_status layer_f32(const CtxF32& x, int l /*1-based*/, int rows, float* xh, float* a, float* qkv, float* attn, float* u,
                     const int32_t* row_seq, const int32_t* pos, const int32_t* slot, int max_len) {
  const pop_config& c = x.m->cfg;
  const pop_layer_weights& lw = x.m->layers[l - 1];
  const int d = c.d_model, f = c.d_ffn, hd = c.head_dim, Dq = x.m->Dq, Dkv = x.m->Dkv, Dqkv = x.m->Dqkv;
  const bool glob = layer_is_global(c, l);
  namespace F = pop::f32;
  F::launch_rmsnorm(xh, (const float*)lw.norm_in, a, nullptr, rows, d, c.rms_eps, x.st);
  F::launch_gemm(a, d, (const float*)lw.wqkv, d, qkv, Dqkv, rows, Dqkv, d, F::EPI_STORE, 0, x.st);
  F::launch_rope_write(qkv, Dqkv, 0, Dq, Dq + Dkv, c.n_q_heads, c.n_kv_heads, hd, pos, slot,
                       glob ? (double)c.rope_theta : (double)c.rope_theta_local, x.c->k_pool_f32(l - 1),
                       x.c->v_pool_f32(l - 1), c.page_size, rows, x.st, (const float*)lw.q_norm, (const float*)lw.k_norm,
                       c.rms_eps, kv_quant(c));
  hipError_t e = F::launch_attention(qkv, Dqkv, 0, attn, row_seq, pos, x.c->k_pool_f32(l - 1), x.c->v_pool_f32(l - 1),
                                     at<int32_t>(x.ws, x.w->o_bt), x.c->max_pages, c.page_size,
                                     glob ? 0 : c.sliding_window,
                                     x.kv_first ? x.kv_first + (size_t)(l - 1) * x.B : nullptr, rows, c.n_q_heads,
                                     c.n_kv_heads, hd, max_len, x.st);
  if (e != hipSuccess) return fail(POP_EHIP, "fp32 attention launch failed: %s", hipGetErrorString(e));
  F::launch_gemm(attn, Dq, (const float*)lw.wo, Dq, xh, d, rows, d, Dq, F::EPI_ADD, 0, x.st, x.gate(l));
  F::launch_rmsnorm(xh, (const float*)lw.norm_post, a, nullptr, rows, d, c.rms_eps, x.st);
  F::launch_gemm(a, d, (const float*)lw.w_gate_up, d, u, f, rows, f, d, F::EPI_GLU, c.act, x.st);
  F::launch_gemm(u, f, (const float*)lw.w_down, f, xh, d, rows, d, f, F::EPI_ADD, 0, x.st, x.gate(l));
  POP_HIP(hipGetLastError());
  return POP_OK;
}

pop_status lm_head_f32(const CtxF32& x, int B, float* dev_logits) {
  const pop_config& c = x.m->cfg;
  namespace F = pop::f32;
  float* xb = at<float>(x.ws, x.w->o_xb);
  float* ab = at<float>(x.ws, x.w->o_ab);
  F::launch_rmsnorm(xb, (const float*)x.m->w.final_norm, ab, nullptr, B, c.d_model, c.rms_eps, x.st);
  F::launch_gemm(ab, c.d_model, (const float*)x.m->w.lm_head, c.d_model, dev_logits, c.vocab, B, c.vocab, c.d_model,
                 F::EPI_STORE, 0, x.st);
  POP_HIP(hipGetLastError());
  return POP_OK;
}

// pop_prefill for an fp32 model; arguments are already validated (slots, row_src computed by the caller)
pop_status prefill_f32(pop_model* m, pop_cache* c, const pop_prefill_args* a, const PrunePlan& plan, float* dev_logits,
                       void* ws, size_t workspace_bytes, hipStream_t st, const std::vector<int32_t>& slots,
                       const std::vector<int32_t>& row_src) {
  const pop_config& cfg = m->cfg;
  const int B = a->n_seqs, maxp = c->max_pages, T = a->cu_seqlens[B];
  const WorkspaceF32 w = carve_f32(cfg, T, B, maxp);
  if (workspace_bytes < w.total)
    return fail(POP_ENOSPACE, "workspace has %zu bytes, %zu needed for %d tokens in %d sequences", workspace_bytes,
                w.total, T, B);
  std::vector<unsigned char> meta(w.meta_bytes, 0);
  auto mi = [&](size_t off) { return reinterpret_cast<int32_t*>(meta.data() + off); };
  std::copy(a->tokens, a->tokens + T, mi(w.o_tokens));
  std::copy(row_src.begin(), row_src.end(), mi(w.o_row_src));
  std::copy(slots.begin(), slots.end(), mi(w.o_slot));
  int max_len = 0;
  for (int b = 0; b < B; ++b) {
    const int s0 = a->cu_seqlens[b], len = a->cu_seqlens[b + 1] - s0;
    max_len = std::max(max_len, len);
    for (int t = 0; t < len; ++t) {
      mi(w.o_pos)[s0 + t] = t;
      mi(w.o_row_seq)[s0 + t] = b;
    }
    mi(w.o_bnd_row)[b] = s0 + len - 1;
    mi(w.o_bnd_pos)[b] = len - 1;
    mi(w.o_bnd_slot)[b] = slots[s0 + len - 1];
    mi(w.o_bnd_seq)[b] = b;
    std::copy(a->block_table + (size_t)b * maxp, a->block_table + (size_t)(b + 1) * maxp, mi(w.o_bt) + (size_t)b * maxp);
  }
  if (max_len > pop::f32::kMaxContext)
    return fail(POP_EUNSUPPORTED, "the fp32 path holds one row of scores in LDS: sequences up to %d tokens",
                pop::f32::kMaxContext);
  record_kv_first(c, a, plan, mi(w.o_kv_first));
  TailRows tr;
  if (plan.window_writes) {
    tr = tail_rows(cfg, a, slots);
    std::copy(tr.row.begin(), tr.row.end(), mi(w.o_tr_row));
    std::copy(tr.pos.begin(), tr.pos.end(), mi(w.o_tr_pos));
    std::copy(tr.slot.begin(), tr.slot.end(), mi(w.o_tr_slot));
  }
  if (pop_status us = upload_meta(c, ws, meta.data(), w.meta_bytes, st)) return us;
  c->n_seqs = B;
  std::fill(c->seq_lens.begin(), c->seq_lens.end(), 0);
  std::fill(c->block_table.begin(), c->block_table.end(), -1);
  for (int b = 0; b < B; ++b) {
    c->seq_lens[b] = a->cu_seqlens[b + 1] - a->cu_seqlens[b];
    std::copy(a->block_table + (size_t)b * maxp, a->block_table + (size_t)(b + 1) * maxp,
              c->block_table.begin() + (size_t)b * maxp);
  }
  namespace F = pop::f32;
  const int d = cfg.d_model, hd = cfg.head_dim, Dq = m->Dq, Dkv = m->Dkv;
  float* h = at<float>(ws, w.o_h);
  float* abuf = at<float>(ws, w.o_a);
  float* qkv = at<float>(ws, w.o_qkv);
  float* attn = at<float>(ws, w.o_attn);
  float* u = at<float>(ws, w.o_u);
  const int32_t* d_pos = at<int32_t>(ws, w.o_pos);
  const int32_t* d_slot = at<int32_t>(ws, w.o_slot);
  CtxF32 x{m, c, ws, &w, st};
  x.kv_first = c->any_kv_first ? at<int32_t>(ws, w.o_kv_first) : nullptr;
  x.B = B;
  x.gates = a->gates;
  F::launch_embed((const float*)m->w.embed, at<int32_t>(ws, w.o_tokens),
                  a->n_ranges > 0 ? at<int32_t>(ws, w.o_row_src) : nullptr, (const float*)a->embeds, h, T, d, st);
  // Layers in order.  A kept layer runs over all rows (Sec. 2.1).  A run of pruned layers leaves h alone
  // (Sec. 2.2) and stores each layer's K/V projection of it with the layer's own norm scale, W^K, W^V and
  // RoPE (Sec. 3.3); the boundary rows, which are never pruned, leave h for that run and pass its layers
  // in full against the cache (Sec. 3.3, boundary handling), then return to their rows of h.
  float* xb = at<float>(ws, w.o_xb);
  const int32_t* bnd_row = at<int32_t>(ws, w.o_bnd_row);
  const bool boundary = a->mode == POP_MODE_POP;
  for (int l = 1; l <= cfg.n_layers;) {
    if (!plan.pruned[l]) {
      if (pop_status s = layer_f32(x, l, T, h, abuf, qkv, attn, u, at<int32_t>(ws, w.o_row_seq), d_pos, d_slot, max_len))
        return s;
      ++l;
      continue;
    }
    int r = l;
    while (plan.pruned[r + 1]) ++r;
    if (plan.kv_projection)
      for (int j = l; j <= r; ++j) {
        const pop_layer_weights& lw = m->layers[j - 1];
        // a sliding-window layer may store only the tail rows a later token can see (window_kv_writes)
        const bool tail = plan.window_writes && !layer_is_global(cfg, j);
        const int rows = tail ? tr.n : T;
        F::launch_rmsnorm(h, (const float*)lw.norm_in, abuf, tail ? at<int32_t>(ws, w.o_tr_row) : nullptr, rows, d,
                          cfg.rms_eps, st);
        F::launch_gemm(abuf, d, (const float*)lw.wqkv + (size_t)Dq * d, d, qkv, 2 * Dkv, rows, 2 * Dkv, d, F::EPI_STORE, 0,
                       st);
        F::launch_rope_write(qkv, 2 * Dkv, -1, 0, Dkv, cfg.n_q_heads, cfg.n_kv_heads, hd,
                             tail ? at<int32_t>(ws, w.o_tr_pos) : d_pos, tail ? at<int32_t>(ws, w.o_tr_slot) : d_slot,
                             layer_is_global(cfg, j) ? (double)cfg.rope_theta : (double)cfg.rope_theta_local,
                             c->k_pool_f32(j - 1), c->v_pool_f32(j - 1), cfg.page_size, rows, st, nullptr,
                             (const float*)lw.k_norm, cfg.rms_eps, kv_quant(cfg));
      }
    POP_HIP(hipGetLastError());
    if (boundary) {
      pop::launch_gather_rows(h, bnd_row, xb, B, d, st);
      for (int j = l; j <= r; ++j)
        if (pop_status s = layer_f32(x, j, B, xb, at<float>(ws, w.o_ab), at<float>(ws, w.o_qkvb), at<float>(ws, w.o_attnb),
                                     at<float>(ws, w.o_ub), at<int32_t>(ws, w.o_bnd_seq), at<int32_t>(ws, w.o_bnd_pos),
                                     at<int32_t>(ws, w.o_bnd_slot), max_len))
          return s;
      pop::launch_scatter_rows(xb, bnd_row, h, B, d, st);
    }
    l = r + 1;
  }
  // logits of each sequence's last row: the boundary token's (full depth), or, without boundary handling,
  // the pruned model's output for it
  if (a->mode != POP_MODE_BODY_ONLY) {
    pop::launch_gather_rows(h, bnd_row, xb, B, d, st);
    if (pop_status s = lm_head_f32(x, B, dev_logits)) return s;
  }
  POP_HIP(hipGetLastError());
  return POP_OK;
}

pop_status decode_step_f32(pop_model* m, pop_cache* c, const int32_t* host_tokens, int B, const float* host_gates,
                           float* dev_logits, void* ws, size_t workspace_bytes, hipStream_t st) {
  const pop_config& cfg = m->cfg;
  const int P = cfg.page_size, maxp = c->max_pages;
  const WorkspaceF32 w = carve_f32(cfg, B, B, maxp);
  if (workspace_bytes < w.total) return fail(POP_ENOSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  std::vector<unsigned char> meta(w.meta_bytes, 0);
  auto mi = [&](size_t off) { return reinterpret_cast<int32_t*>(meta.data() + off); };
  int max_len = 0;
  for (int b = 0; b < B; ++b) {
    const int pos = c->seq_lens[b];
    mi(w.o_tokens)[b] = host_tokens[b];
    mi(w.o_bnd_pos)[b] = pos;
    mi(w.o_bnd_slot)[b] = c->block_table[(size_t)b * maxp + pos / P] * P + pos % P;
    mi(w.o_bnd_seq)[b] = b;
    max_len = std::max(max_len, pos + 1);
    std::copy(c->block_table.begin() + (size_t)b * maxp, c->block_table.begin() + (size_t)(b + 1) * maxp,
              mi(w.o_bt) + (size_t)b * maxp);
    for (int l = 0; l < cfg.n_layers; ++l) mi(w.o_kv_first)[(size_t)l * B + b] = c->kv_first[(size_t)l * c->max_seqs + b];
  }
  if (max_len > pop::f32::kMaxContext)
    return fail(POP_EUNSUPPORTED, "the fp32 path holds one row of scores in LDS: sequences up to %d tokens",
                pop::f32::kMaxContext);
  if (pop_status us = upload_meta(c, ws, meta.data(), w.meta_bytes, st)) return us;
  for (int b = 0; b < B; ++b) c->seq_lens[b] += 1;
  CtxF32 x{m, c, ws, &w, st};
  x.kv_first = c->any_kv_first ? at<int32_t>(ws, w.o_kv_first) : nullptr;
  x.B = B;
  x.gates = host_gates;
  float* xb = at<float>(ws, w.o_xb);
  pop::f32::launch_embed((const float*)m->w.embed, at<int32_t>(ws, w.o_tokens), nullptr, nullptr, xb, B, cfg.d_model, st);
  for (int l = 1; l <= cfg.n_layers; ++l)
    if (pop_status s = layer_f32(x, l, B, xb, at<float>(ws, w.o_ab), at<float>(ws, w.o_qkvb), at<float>(ws, w.o_attnb),
                                 at<float>(ws, w.o_ub), at<int32_t>(ws, w.o_bnd_seq), at<int32_t>(ws, w.o_bnd_pos),
                                 at<int32_t>(ws, w.o_bnd_slot), max_len))
      return s;
  return lm_head_f32(x, B, dev_logits);
}

pop_status gemm_or_fail(const pop::GemmArgs& g, hipStream_t st, const char* what) {
  hipError_t e = pop::launch_gemm(g, st);
  if (e != hipSuccess) return fail(POP_EHIP, "%s GEMM launch failed: %s", what, hipGetErrorString(e));
  return POP_OK;
}

}  // namespace

// ----------------------------------------------------------------------------------------- C ABI
extern "C" {

const char* pop_last_error(void) { return g_last_error.c_str(); }
const char* pop_version(void) { return "pop-mi355x 0.1 (gfx950)"; }

pop_status pop_load_weights(const pop_config* cfg, const pop_weights* w, pop_model** out) {
  if (!out) return fail(POP_EINVAL, "out is NULL");
  *out = nullptr;
  if (pop_status st = check_config(cfg)) return st;
  if (!w || !w->layers) return fail(POP_EINVAL, "weights / layers is NULL");
  if (!w->embed || !w->final_norm || !w->lm_head) return fail(POP_EINVAL, "embed / final_norm / lm_head is NULL");
  if (!aligned16(w->embed) || !aligned16(w->final_norm) || !aligned16(w->lm_head))
    return fail(POP_EALIGN, "embed / final_norm / lm_head not 16-byte aligned");
  for (int l = 0; l < cfg->n_layers; ++l) {
    const pop_layer_weights& lw = w->layers[l];
    const void* ps[6] = {lw.norm_in, lw.wqkv, lw.wo, lw.norm_post, lw.w_gate_up, lw.w_down};
    for (const void* p : ps) {
      if (!p) return fail(POP_EINVAL, "layer %d has a NULL weight pointer", l + 1);
      if (!aligned16(p)) return fail(POP_EALIGN, "layer %d has a weight pointer that is not 16-byte aligned", l + 1);
    }
    if ((lw.q_norm == nullptr) != (lw.k_norm == nullptr))
      return fail(POP_EINVAL, "layer %d has only one of q_norm / k_norm", l + 1);
    if (!aligned16(lw.q_norm) || !aligned16(lw.k_norm))
      return fail(POP_EALIGN, "layer %d has a QK-norm scale that is not 16-byte aligned", l + 1);
  }
  if (cfg->dtype == POP_DTYPE_BF16) {
    // the bf16 kernels address a matrix through a buffer descriptor with 31-bit byte offsets
    const long long d = cfg->d_model, rows = std::max<long long>(
        std::max<long long>(cfg->vocab, 2LL * cfg->d_ffn), (long long)(cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim);
    const long long inner = std::max<long long>(std::max<long long>(d, cfg->d_ffn), (long long)cfg->n_q_heads * cfg->head_dim);
    if (rows * d * 2 >= (1LL << 31) || d * inner * 2 >= (1LL << 31))
      return fail(POP_ESHAPE, "a weight matrix would reach 2 GiB");
  }
  pop_model* m = new (std::nothrow) pop_model();
  if (!m) return fail(POP_EINVAL, "out of host memory");
  m->cfg = *cfg;
  m->w = *w;
  m->layers.assign(w->layers, w->layers + cfg->n_layers);
  m->w.layers = m->layers.data();
  m->Dq = cfg->n_q_heads * cfg->head_dim;
  m->Dkv = cfg->n_kv_heads * cfg->head_dim;
  m->Dqkv = m->Dq + 2 * m->Dkv;
  *out = m;
  return POP_OK;
}

void pop_free_model(pop_model* m) {
  if (!m) return;
  for (auto& s : m->spans) { (void)hipEventDestroy(s.start); (void)hipEventDestroy(s.stop); }
  for (auto e : m->free_events) (void)hipEventDestroy(e);
  delete m;
}

pop_status pop_timing_enable(pop_model* m, int32_t enable) {
  if (!m) return fail(POP_EINVAL, "model is NULL");
  m->timing = enable != 0;
  return POP_OK;
}

pop_status pop_timing_read(pop_model* m, float* ms_out, int32_t* launches_out) {
  if (!m || !ms_out || !launches_out) return fail(POP_EINVAL, "model / output array is NULL");
  for (int i = 0; i < POP_N_STEPS; ++i) { ms_out[i] = 0.f; launches_out[i] = 0; }
  for (auto& s : m->spans) {
    POP_HIP(hipEventSynchronize(s.stop));
    float ms = 0.f;
    POP_HIP(hipEventElapsedTime(&ms, s.start, s.stop));
    ms_out[s.kind] += ms;
    launches_out[s.kind] += 1;
    m->free_events.push_back(s.start);
    m->free_events.push_back(s.stop);
  }
  m->spans.clear();
  return POP_OK;
}

size_t pop_cache_bytes(const pop_config* cfg, int32_t n_pages) {
  if (!cfg || n_pages < 1 || cfg->n_layers < 1 || cfg->n_kv_heads < 1 || cfg->head_dim < 1 || cfg->page_size < 1)
    return 0;
  if (cfg->kv_dtype != POP_KV_BF16 && cfg->kv_dtype != POP_KV_FP8_E4M3) return 0;
  return (size_t)cfg->n_layers * 2 * n_pages * cfg->n_kv_heads * cfg->page_size * cfg->head_dim * cache_elem_bytes(*cfg);
}

size_t pop_workspace_bytes(const pop_config* cfg, int32_t max_tokens, int32_t max_seqs, int32_t max_pages_per_seq) {
  if (check_config(cfg) != POP_OK || max_tokens < 1 || max_seqs < 1 || max_pages_per_seq < 1) return 0;
  if (cfg->dtype == POP_DTYPE_F32) return carve_f32(*cfg, max_tokens, max_seqs, max_pages_per_seq).total;
  return carve(*cfg, max_tokens, max_seqs, max_pages_per_seq).total;
}

pop_status pop_cache_create(const pop_config* cfg, void* dev_pool, size_t bytes, int32_t n_pages, int32_t max_seqs,
                            int32_t max_pages_per_seq, pop_cache** out) {
  if (!out) return fail(POP_EINVAL, "out is NULL");
  *out = nullptr;
  if (pop_status st = check_config(cfg)) return st;
  if (!dev_pool) return fail(POP_EINVAL, "dev_pool is NULL");
  if (!aligned16(dev_pool)) return fail(POP_EALIGN, "dev_pool not 16-byte aligned");
  if (n_pages < 1 || max_seqs < 1 || max_pages_per_seq < 1) return fail(POP_EINVAL, "non-positive cache geometry");
  if ((long long)n_pages * cfg->page_size >= (1LL << 31)) return fail(POP_EINVAL, "slot index would overflow int32");
  const size_t need = pop_cache_bytes(cfg, n_pages);
  if (bytes < need) return fail(POP_ENOSPACE, "pool has %zu bytes, %zu needed for %d pages", bytes, need, n_pages);
  pop_cache* c = new (std::nothrow) pop_cache();
  if (!c) return fail(POP_EINVAL, "out of host memory");
  c->cfg = *cfg;
  c->pool = reinterpret_cast<bf16_t*>(dev_pool);
  c->bytes = bytes;
  c->n_pages = n_pages;
  c->max_seqs = max_seqs;
  c->max_pages = max_pages_per_seq;
  c->n_seqs = 0;
  c->seq_lens.assign(max_seqs, 0);
  c->block_table.assign((size_t)max_seqs * max_pages_per_seq, -1);
  c->kv_first.assign((size_t)cfg->n_layers * max_seqs, 0);
  *out = c;
  return POP_OK;
}

void pop_cache_destroy(pop_cache* c) {
  if (!c) return;
  for (int k = 0; k < 2; ++k) {
    if (c->stage_done[k]) { (void)hipEventSynchronize(c->stage_done[k]); (void)hipEventDestroy(c->stage_done[k]); }
    if (c->stage_host[k]) (void)hipHostFree(c->stage_host[k]);
  }
  delete c;
}

int32_t pop_cache_n_seqs(const pop_cache* c) { return c ? c->n_seqs : 0; }

pop_status pop_cache_seq_lens(const pop_cache* c, int32_t* host_out) {
  if (!c || !host_out) return fail(POP_EINVAL, "cache / host_out is NULL");
  std::copy(c->seq_lens.begin(), c->seq_lens.end(), host_out);
  return POP_OK;
}

pop_status pop_cache_block_table(const pop_cache* c, int32_t* host_out, int32_t* host_seq_lens) {
  if (!c || !host_out) return fail(POP_EINVAL, "cache / host_out is NULL");
  std::copy(c->block_table.begin(), c->block_table.end(), host_out);
  if (host_seq_lens) std::copy(c->seq_lens.begin(), c->seq_lens.end(), host_seq_lens);
  return POP_OK;
}

pop_status pop_slot_map(const int32_t* host_cu_seqlens, int32_t n_seqs, const int32_t* host_block_table,
                        int32_t max_pages_per_seq, int32_t page_size, int32_t n_pages, int32_t* host_slots_out) {
  if (!host_slots_out) return fail(POP_EINVAL, "host_slots_out is NULL");
  return slot_map_impl(host_cu_seqlens, n_seqs, host_block_table, max_pages_per_seq, page_size, n_pages,
                       host_slots_out, 0);
}

pop_status pop_prefill(pop_model* m, pop_cache* c, const pop_prefill_args* a, float* dev_logits, void* dev_workspace,
                       size_t workspace_bytes, pop_stream stream) {
  // ------------------------------------------------------------------ validation (no launches yet)
  if (!m || !c || !a) return fail(POP_EINVAL, "model / cache / args is NULL");
  const pop_config& cfg = m->cfg;
  if (std::memcmp(&cfg, &c->cfg, sizeof cfg) != 0) return fail(POP_EINVAL, "cache was created for another config");
  if (!a->tokens || !a->cu_seqlens || !a->block_table) return fail(POP_EINVAL, "tokens / cu_seqlens / block_table is NULL");
  if (a->n_seqs < 1 || a->n_seqs > c->max_seqs)
    return fail(POP_EINVAL, "n_seqs %d outside [1, %d]", a->n_seqs, c->max_seqs);
  PrunePlan plan;
  if (pop_status ps = make_plan(cfg, a, &plan)) return ps;
  if (a->mode != POP_MODE_BODY_ONLY && !dev_logits) return fail(POP_EINVAL, "dev_logits is NULL");
  if (dev_logits && !aligned16(dev_logits)) return fail(POP_EALIGN, "dev_logits not 16-byte aligned");
  if (!dev_workspace) return fail(POP_EINVAL, "dev_workspace is NULL");
  if (reinterpret_cast<uintptr_t>(dev_workspace) & 255) return fail(POP_EALIGN, "dev_workspace not 256-byte aligned");
  const int B = a->n_seqs, P = cfg.page_size, maxp = c->max_pages;
  std::vector<int32_t> slots;
  {
    // lengths first (slot_map_impl re-checks), to size the slot array
    if (a->cu_seqlens[0] != 0) return fail(POP_EINVAL, "cu_seqlens[0] = %d, expected 0", a->cu_seqlens[0]);
    for (int b = 0; b < B; ++b)
      if (a->cu_seqlens[b + 1] <= a->cu_seqlens[b])
        return fail(POP_EINVAL, "sequence %d is empty (cu_seqlens must be strictly increasing)", b);
  }
  const int T = a->cu_seqlens[B];
  slots.resize(T);
  if (pop_status st = slot_map_impl(a->cu_seqlens, B, a->block_table, maxp, P, c->n_pages, slots.data(), 0)) return st;
  for (int t = 0; t < T; ++t)
    if (a->tokens[t] < 0 || a->tokens[t] >= cfg.vocab)
      return fail(POP_EINVAL, "token %d at packed index %d is outside [0, %d)", a->tokens[t], t, cfg.vocab);
  std::vector<int32_t> row_src((size_t)T, -1);
  if (a->n_ranges < 0 || (a->n_ranges > 0 && (!a->embed_ranges || !a->embeds)))
    return fail(POP_EINVAL, "embed ranges given without embeds / embed_ranges");
  if (a->embeds && !aligned16(a->embeds)) return fail(POP_EALIGN, "embeds not 16-byte aligned");
  {
    int next_row = 0;
    for (int r = 0; r < a->n_ranges; ++r) {
      const int sb = a->embed_ranges[3 * r], first = a->embed_ranges[3 * r + 1], cnt = a->embed_ranges[3 * r + 2];
      if (sb < 0 || sb >= B || first < 0 || cnt < 0 ||
          (long long)first + cnt > (long long)a->cu_seqlens[sb + 1] - a->cu_seqlens[sb])
        return fail(POP_EINVAL, "embed range %d (seq %d, first %d, count %d) is outside its sequence", r, sb, first, cnt);
      for (int i = 0; i < cnt; ++i) {
        int32_t& rs = row_src[(size_t)a->cu_seqlens[sb] + first + i];
        if (rs >= 0) return fail(POP_EINVAL, "embed ranges overlap at sequence %d position %d", sb, first + i);
        rs = next_row++;
      }
    }
  }
  if (cfg.dtype == POP_DTYPE_F32)
    return prefill_f32(m, c, a, plan, dev_logits, dev_workspace, workspace_bytes, reinterpret_cast<hipStream_t>(stream),
                       slots, row_src);
  const Workspace w = carve(cfg, T, B, maxp);
  if (workspace_bytes < w.total)
    return fail(POP_ENOSPACE, "workspace has %zu bytes, %zu needed for %d tokens in %d sequences", workspace_bytes,
                w.total, T, B);
  const int d = cfg.d_model, f = cfg.d_ffn, hd = cfg.head_dim, Dq = m->Dq, Dkv = m->Dkv, Dqkv = m->Dqkv;
  if ((long long)T * std::max(std::max(Dqkv, f), d) * 2 >= (1LL << 31))
    return fail(POP_ESHAPE, "an activation matrix would exceed 2 GiB; split the batch");

  // ------------------------------------------------------------------ host-side meta
  std::vector<unsigned char> meta(w.meta_bytes, 0);
  auto mi = [&](size_t off) { return reinterpret_cast<int32_t*>(meta.data() + off); };
  std::copy(a->tokens, a->tokens + T, mi(w.o_tokens));
  std::copy(row_src.begin(), row_src.end(), mi(w.o_row_src));
  std::copy(slots.begin(), slots.end(), mi(w.o_slot));
  std::copy(a->cu_seqlens, a->cu_seqlens + B + 1, mi(w.o_cu));
  int n_t64 = 0, n_ta = 0, Tp = 0, max_len = 0;
  for (int b = 0; b < B; ++b) {
    const int s0 = a->cu_seqlens[b], len = a->cu_seqlens[b + 1] - s0;
    max_len = std::max(max_len, len);
    for (int t = 0; t < len; ++t) mi(w.o_pos)[s0 + t] = t;
    mi(w.o_vt_off)[b] = Tp;
    Tp += (int)round_up(len, 64);
    for (int p0 = 0; p0 < len; p0 += 64) {
      mi(w.o_t64_seq)[n_t64] = b;
      mi(w.o_t64_start)[n_t64++] = p0;
    }
    mi(w.o_bnd_row)[b] = s0 + len - 1;
    mi(w.o_bnd_pos)[b] = len - 1;
    mi(w.o_bnd_slot)[b] = slots[s0 + len - 1];
    std::copy(a->block_table + (size_t)b * maxp, a->block_table + (size_t)(b + 1) * maxp, mi(w.o_bt) + (size_t)b * maxp);
  }
  n_ta = build_attention_work(a->cu_seqlens, B, mi(w.o_ta_seq), mi(w.o_ta_start), mi(w.o_ta_start2));
  record_kv_first(c, a, plan, mi(w.o_kv_first));
  // Pruned layers in two lists: those that store an entry for every row, and (window_kv_writes) the
  // sliding-window ones that store the tail rows only.  A run of consecutive pruned layers is a range of each.
  std::vector<int> full_layers, tail_layers;
  {
    const bf16_t** wf = reinterpret_cast<const bf16_t**>(meta.data() + w.o_wl_full);
    const bf16_t** wt = reinterpret_cast<const bf16_t**>(meta.data() + w.o_wl_tail);
    // where each of these layers' entries go and which RoPE table it uses (device addresses inside the workspace)
    pop::KvDest* df = reinterpret_cast<pop::KvDest*>(meta.data() + w.o_kvd_full);
    pop::KvDest* dt = reinterpret_cast<pop::KvDest*>(meta.data() + w.o_kvd_tail);
    for (int l = 1; l <= cfg.n_layers; ++l) {
      if (!plan.pruned[l]) continue;
      const bf16_t* wkv = reinterpret_cast<const bf16_t*>(m->layers[l - 1].wqkv) + (size_t)Dq * d;
      if (plan.window_writes && !layer_is_global(cfg, l)) {
        wt[tail_layers.size()] = wkv;
        dt[tail_layers.size()] = pop::KvDest{c->k_pool(l - 1), at<float2>(dev_workspace, w.o_cs_tail)};
        tail_layers.push_back(l);
      } else {
        wf[full_layers.size()] = wkv;
        df[full_layers.size()] = pop::KvDest{c->k_pool(l - 1), at<float2>(dev_workspace, layer_is_global(cfg, l) ? w.o_cs_g : w.o_cs_l)};
        full_layers.push_back(l);
      }
    }
  }
  TailRows tr;
  if (!tail_layers.empty()) {
    tr = tail_rows(cfg, a, slots);
    std::copy(tr.row.begin(), tr.row.end(), mi(w.o_tr_row));
    std::copy(tr.pos.begin(), tr.pos.end(), mi(w.o_tr_pos));
    std::copy(tr.slot.begin(), tr.slot.end(), mi(w.o_tr_slot));
    std::copy(tr.cu.begin(), tr.cu.end(), mi(w.o_tr_cu));
    std::copy(tr.t64_seq.begin(), tr.t64_seq.end(), mi(w.o_tr_t64_seq));
    std::copy(tr.t64_start.begin(), tr.t64_start.end(), mi(w.o_tr_t64_start));
  }

  // ------------------------------------------------------------------ launches
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  void* ws = dev_workspace;
  if (pop_status us = upload_meta(c, ws, meta.data(), w.meta_bytes, st)) return us;
  // sequences start from empty; record the new state now that nothing can fail on arguments
  c->n_seqs = B;
  std::fill(c->seq_lens.begin(), c->seq_lens.end(), 0);
  std::fill(c->block_table.begin(), c->block_table.end(), -1);
  for (int b = 0; b < B; ++b) {
    c->seq_lens[b] = a->cu_seqlens[b + 1] - a->cu_seqlens[b];
    std::copy(a->block_table + (size_t)b * maxp, a->block_table + (size_t)(b + 1) * maxp,
              c->block_table.begin() + (size_t)b * maxp);
  }

  const int32_t* d_tokens = at<int32_t>(ws, w.o_tokens);
  const int32_t* d_row_src = at<int32_t>(ws, w.o_row_src);
  const int32_t* d_pos = at<int32_t>(ws, w.o_pos);
  const int32_t* d_slot = at<int32_t>(ws, w.o_slot);
  const int32_t* d_cu = at<int32_t>(ws, w.o_cu);
  const int32_t* d_vt_off = at<int32_t>(ws, w.o_vt_off);
  float* h = at<float>(ws, w.o_h);
  bf16_t* abuf = at<bf16_t>(ws, w.o_a);
  bf16_t* qkv = at<bf16_t>(ws, w.o_qkv);
  bf16_t* attn = at<bf16_t>(ws, w.o_attn);
  bf16_t* u = at<bf16_t>(ws, w.o_u);
  bf16_t* vT = at<bf16_t>(ws, w.o_vT);
  float2* cs_g = at<float2>(ws, w.o_cs_g);
  float2* cs_l = at<float2>(ws, w.o_cs_l);

  {
    StepTimer tm(m, st, POP_STEP_EMBED);
    pop::launch_embed((const bf16_t*)m->w.embed, d_tokens, a->n_ranges > 0 ? d_row_src : nullptr,
                      (const bf16_t*)a->embeds, h, T, d, st);
    bool any_local = false;
    for (int l = 1; l <= cfg.n_layers; ++l) any_local |= !layer_is_global(cfg, l);
    pop::launch_rope_table(d_pos, cs_g, T, hd, (double)cfg.rope_theta, st);
    if (any_local) pop::launch_rope_table(d_pos, cs_l, T, hd, (double)cfg.rope_theta_local, st);
    if (tr.n > 0)
      pop::launch_rope_table(at<int32_t>(ws, w.o_tr_pos), at<float2>(ws, w.o_cs_tail), tr.n, hd,
                             (double)cfg.rope_theta_local, st);
  }
  POP_HIP(hipGetLastError());

  pop::RopeWriteArgs rw{};
  rw.n_q_heads = cfg.n_q_heads;
  rw.n_kv_heads = cfg.n_kv_heads;
  rw.hd = hd;
  rw.slot = d_slot;
  rw.page_size = P;
  rw.Tp = Tp;
  rw.cu_seqlens = d_cu;
  rw.vt_off = d_vt_off;
  rw.tile_seq = at<int32_t>(ws, w.o_t64_seq);
  rw.tile_start = at<int32_t>(ws, w.o_t64_start);
  rw.n_tiles = n_t64;
  rw.kvq = kv_quant(cfg);

  // ---- a kept layer over all given rows (Sec. 2.1)
  // abuf_gamma: the norm scale with which abuf already holds RMSNorm(h) (left there by the previous layer's down
  // projection when its K range was split: the kernel that adds the parts to h normalises the sum on the way).
  const float* abuf_gamma = nullptr;
  const int down_parts = down_split_parts(T, d, f);
  auto kept_layer = [&](int l) -> pop_status {
    const pop_layer_weights& lw = m->layers[l - 1];
    const bool glob = layer_is_global(cfg, l);
    if (abuf_gamma == nullptr || abuf_gamma != (const float*)lw.norm_in) {
      StepTimer tm(m, st, POP_STEP_NORM);
      pop::launch_rmsnorm(h, nullptr, nullptr, (const float*)lw.norm_in, abuf, nullptr, T, d, cfg.rms_eps, st);
    }
    abuf_gamma = nullptr;
    pop::GemmArgs g{};
    g.batch = 1;
    g.A = abuf; g.lda = d; g.W = (const bf16_t*)lw.wqkv; g.ldw = d; g.out = qkv; g.ldc = Dqkv;
    // q, k, v leave the GEMM as fp16: they only feed the RoPE/append and attention kernels, and fp16
    // keeps three more mantissa bits than bf16 for the score contraction (the cache itself is bf16)
    g.M = T; g.N = Dqkv; g.K = d; g.epilogue = pop::EPI_STORE_F16;
    g.splitk_ws = w.splitk_bytes ? at<float>(ws, w.o_splitk) : nullptr;
    g.splitk_ws_bytes = w.splitk_bytes;
    {
      StepTimer tm(m, st, POP_STEP_QKV_GEMM);
      if (pop_status s = gemm_or_fail(g, st, "QKV")) return s;
    }
    rw.qkv = qkv; rw.ld = Dqkv; rw.q_col = 0; rw.k_col = Dq; rw.v_col = Dq + Dkv;
    rw.cs = glob ? cs_g : cs_l;
    rw.q_gamma = (const float*)lw.q_norm; rw.k_gamma = (const float*)lw.k_norm; rw.qk_eps = cfg.rms_eps;
    rw.k_pool = c->k_pool(l - 1); rw.v_pool = c->v_pool(l - 1);
    rw.vT = vT;
    rw.fp16_inplace = 1;
    rw.fp16_input = 1;
    {
      StepTimer tm(m, st, POP_STEP_ROPE_WRITE);
      pop::launch_rope_write(rw, st);
    }
    pop::AttnPrefillArgs ap{};
    ap.qkv = qkv; ap.ld = Dqkv; ap.q_col = 0; ap.k_col = Dq; ap.vT = vT; ap.Tp = Tp; ap.out = attn;
    ap.T = T; ap.n_q_heads = cfg.n_q_heads; ap.n_kv_heads = cfg.n_kv_heads; ap.hd = hd;
    ap.window = glob ? 0 : cfg.sliding_window;
    ap.cu_seqlens = d_cu; ap.vt_off = d_vt_off;
    ap.tile_seq = at<int32_t>(ws, w.o_ta_seq); ap.tile_start = at<int32_t>(ws, w.o_ta_start);
    ap.tile_start2 = at<int32_t>(ws, w.o_ta_start2); ap.n_tiles = n_ta;
    {
      StepTimer tm(m, st, POP_STEP_ATTENTION);
      hipError_t e = pop::launch_attention_prefill(ap, st);
      if (e != hipSuccess) return fail(POP_EHIP, "attention launch failed: %s", hipGetErrorString(e));
    }
    g.A = attn; g.lda = Dq; g.W = (const bf16_t*)lw.wo; g.ldw = Dq; g.out = h; g.ldc = d;
    g.M = T; g.N = d; g.K = Dq; g.epilogue = pop::EPI_ADD_F32;
    g.scaled = a->gates != nullptr; g.scale = a->gates ? a->gates[l - 1] : 1.f;   // virtual gate of the layer
    {
      StepTimer tm(m, st, POP_STEP_O_GEMM);
      if (pop_status s = gemm_or_fail(g, st, "O")) return s;
    }
    {
      StepTimer tm(m, st, POP_STEP_NORM);
      pop::launch_rmsnorm(h, nullptr, nullptr, (const float*)lw.norm_post, abuf, nullptr, T, d, cfg.rms_eps, st);
    }
    g.A = abuf; g.lda = d; g.W = (const bf16_t*)lw.w_gate_up; g.ldw = d; g.out = u; g.ldc = f;
    g.M = T; g.N = f; g.K = d; g.epilogue = pop::EPI_GLU_BF16; g.act = cfg.act;
    {
      StepTimer tm(m, st, POP_STEP_GATE_UP_GEMM);
      if (pop_status s = gemm_or_fail(g, st, "gate/up")) return s;
    }
    g.A = u; g.lda = f; g.W = (const bf16_t*)lw.w_down; g.ldw = f; g.out = h; g.ldc = d;
    g.M = T; g.N = d; g.K = f; g.epilogue = pop::EPI_ADD_F32;
    g.scaled = a->gates != nullptr; g.scale = a->gates ? a->gates[l - 1] : 1.f;
    // If the K range is split and another kept layer follows directly, the kernel that adds the parts to h also
    // writes that layer's normalised input (one pass over h instead of two).
    const float* next_gamma = l < cfg.n_layers && !plan.pruned[l + 1] ? (const float*)m->layers[l].norm_in : nullptr;
    int parts = 1;
    g.force_split = down_parts;
    g.partials_only = down_parts > 1 && next_gamma != nullptr && d % 4 == 0;
    g.split_used = &parts;
    {
      StepTimer tm(m, st, POP_STEP_DOWN_GEMM);
      if (pop_status s = gemm_or_fail(g, st, "down")) return s;
    }
    if (g.partials_only && parts > 1) {
      StepTimer tm(m, st, POP_STEP_DOWN_ADD_NORM);
      pop::launch_add_parts_rmsnorm(h, g.splitk_ws, parts, (size_t)T * d, next_gamma, abuf, T, d, cfg.rms_eps, st,
                                    pop::residual_scale(g));
      abuf_gamma = next_gamma;
    }
    return POP_OK;
  };

  // ---- a run first..last of pruned layers: independent KV projections of the hidden state the run leaves
  //      unchanged (Sec. 2.2, Sec. 3.3); layers that share their rows share one normalisation pass and one
  //      batched GEMM (chunks of kKvChunk).  `tail`: only the tail rows of every sequence, gathered.
  bf16_t* a_multi = at<bf16_t>(ws, w.o_a_multi);
  bf16_t* kv_out = at<bf16_t>(ws, w.o_kv_out);
  auto kv_only_layers = [&](const std::vector<int>& layers, int i0, int i1, const bf16_t* const* d_wlist,
                            const pop::KvDest* d_dest, bool tail) -> pop_status {
    const int rows = tail ? tr.n : T;
    if (rows <= 0) return POP_OK;
    pop::RopeWriteArgs rk = rw;
    if (tail) {
      rk.slot = at<int32_t>(ws, w.o_tr_slot);
      rk.cu_seqlens = at<int32_t>(ws, w.o_tr_cu);
      rk.tile_seq = at<int32_t>(ws, w.o_tr_t64_seq);
      rk.tile_start = at<int32_t>(ws, w.o_tr_t64_start);
      rk.n_tiles = (int)tr.t64_seq.size();
    }
    for (int c0 = i0; c0 < i1; c0 += kKvChunk) {
      const int n = std::min(kKvChunk, i1 - c0);
      pop::GammaList gl{};
      for (int j = 0; j < n; ++j) gl.g[j] = (const float*)m->layers[layers[c0 + j] - 1].norm_in;
      {
        StepTimer tm(m, st, POP_STEP_KV_ONLY_NORM);
        pop::launch_rmsnorm_multi(h, gl, n, a_multi, (size_t)rows * d, rows, d, cfg.rms_eps, st,
                                  tail ? at<int32_t>(ws, w.o_tr_row) : nullptr);
      }
      pop::GemmArgs g{};
      g.A = a_multi; g.lda = d; g.W = nullptr; g.ldw = d; g.out = kv_out; g.ldc = 2 * Dkv;
      g.M = rows; g.N = 2 * Dkv; g.K = d; g.epilogue = pop::EPI_STORE_BF16;
      g.batch = n; g.strideA = (long long)rows * d; g.strideC = (long long)rows * 2 * Dkv;
      g.W_list = d_wlist + c0;
      // Straight into the paged cache (RoPE and the page scatter in the GEMM's epilogue) when the layers of the
      // chunk have no per-head key norm (that needs a head's sum of squares first) and the 256 x 256 tiles of that
      // epilogue fill at least three quarters of the chip (one pruned layer of a 2048-token prompt is 64 tiles: the
      // smaller tiles of the plain GEMM plus the append kernel are faster there); otherwise through kv_out and the
      // append kernel.
      bool fused = pop::gemm_kv_cache_supported(cfg.n_kv_heads, hd) &&
                   (long long)((rows + 255) / 256) * ((2 * Dkv + 255) / 256) * n >= 192;
      for (int j = 0; j < n; ++j) fused = fused && m->layers[layers[c0 + j] - 1].k_norm == nullptr;
      if (fused) {
        g.epilogue = pop::EPI_KV_CACHE;
        g.kv_dest = d_dest + c0;
        g.kv_slot = rk.slot;
        g.kv_heads = cfg.n_kv_heads; g.kv_hd = hd; g.kv_page_size = P;
        g.kv_pool_stride = (int64_t)c->pool_stride();
        g.kvq = kv_quant(cfg);
      }
      {
        StepTimer tm(m, st, POP_STEP_KV_ONLY_GEMM);
        if (pop_status s = gemm_or_fail(g, st, "K/V-only")) return s;
      }
      if (fused) continue;
      StepTimer tmw(m, st, POP_STEP_KV_ONLY_WRITE);
      for (int j = 0; j < n; ++j) {
        const int l = layers[c0 + j];
        rk.qkv = kv_out + (size_t)j * rows * 2 * Dkv; rk.ld = 2 * Dkv; rk.q_col = -1; rk.k_col = 0; rk.v_col = Dkv;
        rk.cs = tail ? at<float2>(ws, w.o_cs_tail) : (layer_is_global(cfg, l) ? cs_g : cs_l);
        rk.q_gamma = nullptr; rk.k_gamma = (const float*)m->layers[l - 1].k_norm; rk.qk_eps = cfg.rms_eps;
        rk.k_pool = c->k_pool(l - 1); rk.v_pool = c->v_pool(l - 1);
        rk.vT = nullptr;
        rk.fp16_inplace = 0;
        rk.fp16_input = 0;
        rk.cache_only = 1;
        pop::launch_rope_write(rk, st);
      }
    }
    POP_HIP(hipGetLastError());
    return POP_OK;
  };
  auto kv_only_run = [&](int first, int last) -> pop_status {
    auto range = [&](const std::vector<int>& v, int& i0, int& i1) {
      i0 = (int)(std::lower_bound(v.begin(), v.end(), first) - v.begin());
      i1 = (int)(std::upper_bound(v.begin(), v.end(), last) - v.begin());
    };
    int i0, i1;
    range(full_layers, i0, i1);
    if (pop_status s = kv_only_layers(full_layers, i0, i1, at<const bf16_t*>(ws, w.o_wl_full),
                                      at<const pop::KvDest>(ws, w.o_kvd_full), false))
      return s;
    range(tail_layers, i0, i1);
    return kv_only_layers(tail_layers, i0, i1, at<const bf16_t*>(ws, w.o_wl_tail),
                          at<const pop::KvDest>(ws, w.o_kvd_tail), true);
  };

  // ---- layers in order.  The boundary tokens (Sec. 3.3, boundary handling) are rows of h through kept
  //      layers (identical to their decode step there); through a run of pruned layers they leave h, pass
  //      the run's layers in full against the cache, and return to their rows if a kept layer follows.
  LayerCtx x{m, c, ws, &w, st};
  x.kv_first = c->any_kv_first ? at<int32_t>(ws, w.o_kv_first) : nullptr;
  const bool boundary = a->mode == POP_MODE_POP;
  const int32_t* bnd_row = at<int32_t>(ws, w.o_bnd_row);
  float* xb = at<float>(ws, w.o_xb);
  bool rows_in_xb = false;   // the boundary rows' current state is in xb rather than in h
  bool dec_tables_done = false;
  for (int l = 1; l <= cfg.n_layers;) {
    if (!plan.pruned[l]) {
      if (rows_in_xb) {
        StepTimer tm(m, st, POP_STEP_BOUNDARY);
        pop::launch_scatter_rows(xb, bnd_row, h, B, d, st);
        rows_in_xb = false;
      }
      if (pop_status s = kept_layer(l)) return s;
      ++l;
      continue;
    }
    int r = l;
    while (plan.pruned[r + 1]) ++r;
    if (plan.kv_projection)
      if (pop_status s = kv_only_run(l, r)) return s;
    if (boundary) {
      StepTimer tm(m, st, POP_STEP_BOUNDARY);
      pop::launch_gather_rows(h, bnd_row, xb, B, d, st);
      x.ab_gamma = nullptr;
      rows_in_xb = true;
      if (!dec_tables_done) {
        decode_rope_tables(x, at<int32_t>(ws, w.o_bnd_pos), B);
        dec_tables_done = true;
      }
      for (int j = l; j <= r; ++j) {
        // what reads these rows next: the following layer of the run, the LM head, or (a kept layer follows) h
        const float* next = j < r ? (const float*)m->layers[j].norm_in
                            : (r == cfg.n_layers && a->mode != POP_MODE_BODY_ONLY ? (const float*)m->w.final_norm : nullptr);
        if (pop_status s = decode_layer(x, j, B, at<int32_t>(ws, w.o_bnd_pos), at<int32_t>(ws, w.o_bnd_slot), max_len, next))
          return s;
      }
    }
    l = r + 1;
  }
  // ---- logits of each sequence's last row: the boundary token's, or (no boundary handling) the pruned
  //      model's output for it
  if (a->mode != POP_MODE_BODY_ONLY) {
    StepTimer tm(m, st, POP_STEP_BOUNDARY);
    if (!rows_in_xb) {
      pop::launch_gather_rows(h, bnd_row, xb, B, d, st);
      x.ab_gamma = nullptr;
    }
    if (pop_status s = lm_head(x, B, dev_logits)) return s;
  }
  return POP_OK;
}

pop_status pop_decode_step(pop_model* m, pop_cache* c, const int32_t* host_tokens, int32_t n_seqs, float* dev_logits,
                           void* dev_workspace, size_t workspace_bytes, pop_stream stream) {
  return pop_decode_step_gated(m, c, host_tokens, n_seqs, nullptr, dev_logits, dev_workspace, workspace_bytes, stream);
}

pop_status pop_decode_step_gated(pop_model* m, pop_cache* c, const int32_t* host_tokens, int32_t n_seqs,
                                 const float* host_gates, float* dev_logits, void* dev_workspace,
                                 size_t workspace_bytes, pop_stream stream) {
  if (!m || !c || !host_tokens || !dev_logits) return fail(POP_EINVAL, "model / cache / tokens / logits is NULL");
  const pop_config& cfg = m->cfg;
  if (host_gates)
    for (int l = 0; l < cfg.n_layers; ++l)
      if (!std::isfinite(host_gates[l])) return fail(POP_EINVAL, "gates[%d] is not finite", l);
  if (std::memcmp(&cfg, &c->cfg, sizeof cfg) != 0) return fail(POP_EINVAL, "cache was created for another config");
  if (c->n_seqs < 1) return fail(POP_ESTATE, "no prefilled sequences in this cache");
  if (n_seqs != c->n_seqs) return fail(POP_EINVAL, "n_seqs %d does not match the %d live sequences", n_seqs, c->n_seqs);
  if (!aligned16(dev_logits)) return fail(POP_EALIGN, "dev_logits not 16-byte aligned");
  if (!dev_workspace) return fail(POP_EINVAL, "dev_workspace is NULL");
  if (reinterpret_cast<uintptr_t>(dev_workspace) & 255) return fail(POP_EALIGN, "dev_workspace not 256-byte aligned");
  const int B = n_seqs, P = cfg.page_size, maxp = c->max_pages;
  for (int b = 0; b < B; ++b) {
    if (host_tokens[b] < 0 || host_tokens[b] >= cfg.vocab)
      return fail(POP_EINVAL, "token %d of sequence %d is outside [0, %d)", host_tokens[b], b, cfg.vocab);
    const int pos = c->seq_lens[b];
    if (pos / P >= maxp || c->block_table[(size_t)b * maxp + pos / P] < 0)
      return fail(POP_ENOSPACE, "sequence %d has no page for position %d", b, pos);
  }
  if (cfg.dtype == POP_DTYPE_F32)
    return decode_step_f32(m, c, host_tokens, B, host_gates, dev_logits, dev_workspace, workspace_bytes,
                           reinterpret_cast<hipStream_t>(stream));
  const Workspace w = carve(cfg, B, B, maxp);
  if (workspace_bytes < w.total) return fail(POP_ENOSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  std::vector<unsigned char> meta(w.meta_bytes, 0);
  auto mi = [&](size_t off) { return reinterpret_cast<int32_t*>(meta.data() + off); };
  int max_len = 0;
  for (int b = 0; b < B; ++b) {
    if (host_tokens[b] < 0 || host_tokens[b] >= cfg.vocab)
      return fail(POP_EINVAL, "token %d of sequence %d is outside [0, %d)", host_tokens[b], b, cfg.vocab);
    const int pos = c->seq_lens[b];
    if (pos / P >= maxp || c->block_table[(size_t)b * maxp + pos / P] < 0)
      return fail(POP_ENOSPACE, "sequence %d has no page for position %d", b, pos);
    mi(w.o_tokens)[b] = host_tokens[b];
    mi(w.o_bnd_pos)[b] = pos;
    mi(w.o_bnd_slot)[b] = c->block_table[(size_t)b * maxp + pos / P] * P + pos % P;
    max_len = std::max(max_len, pos + 1);
    std::copy(c->block_table.begin() + (size_t)b * maxp, c->block_table.begin() + (size_t)(b + 1) * maxp,
              mi(w.o_bt) + (size_t)b * maxp);
    for (int l = 0; l < cfg.n_layers; ++l) mi(w.o_kv_first)[(size_t)l * B + b] = c->kv_first[(size_t)l * c->max_seqs + b];
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  void* ws = dev_workspace;
  if (pop_status us = upload_meta(c, ws, meta.data(), w.meta_bytes, st)) return us;
  for (int b = 0; b < B; ++b) c->seq_lens[b] += 1;
  LayerCtx x{m, c, ws, &w, st};
  x.kv_first = c->any_kv_first ? at<int32_t>(ws, w.o_kv_first) : nullptr;
  x.gates = host_gates;
  pop::launch_embed((const bf16_t*)m->w.embed, at<int32_t>(ws, w.o_tokens), nullptr, nullptr, at<float>(ws, w.o_xb),
                    B, cfg.d_model, st);
  decode_rope_tables(x, at<int32_t>(ws, w.o_bnd_pos), B);
  for (int l = 1; l <= cfg.n_layers; ++l) {
    const float* next = (const float*)(l < cfg.n_layers ? m->layers[l].norm_in : m->w.final_norm);
    if (pop_status s = decode_layer(x, l, B, at<int32_t>(ws, w.o_bnd_pos), at<int32_t>(ws, w.o_bnd_slot), max_len, next))
      return s;
  }
  return lm_head(x, B, dev_logits);
}

// ----------------------------------------------------------------------------------------- generation
size_t pop_generate_workspace_bytes(const pop_config* cfg, int32_t max_tokens, int32_t max_seqs,
                                    int32_t max_pages_per_seq, int32_t max_new_tokens) {
  const size_t base = pop_workspace_bytes(cfg, max_tokens, max_seqs, max_pages_per_seq);
  if (base == 0 || max_new_tokens < 1) return 0;
  return base + round_up(4 * (size_t)max_seqs * (2 * (size_t)max_new_tokens + 1), 256);
}

pop_status pop_generate(pop_model* m, pop_cache* c, const pop_prefill_args* a, int32_t max_new_tokens, int32_t eos_token,
                        int32_t* dev_tokens_out, float* dev_logits, void* dev_workspace, size_t workspace_bytes,
                        pop_stream stream) {
  if (!m || !c || !a) return fail(POP_EINVAL, "model / cache / args is NULL");
  if (!dev_tokens_out || !dev_logits) return fail(POP_EINVAL, "dev_tokens_out / dev_logits is NULL");
  if (max_new_tokens < 1) return fail(POP_EINVAL, "max_new_tokens %d < 1", max_new_tokens);
  if (a->mode != POP_MODE_POP && a->mode != POP_MODE_NO_BOUNDARY)
    return fail(POP_EINVAL, "generation needs the last prompt token's logits (POP_MODE_POP or POP_MODE_NO_BOUNDARY)");
  if (a->gates) return fail(POP_EINVAL, "virtual gates belong to pop_prefill / pop_decode_step_gated, not to generation");
  const pop_config& cfg = m->cfg;
  if (eos_token >= cfg.vocab) return fail(POP_EINVAL, "eos_token %d outside the vocabulary", eos_token);
  if (!a->cu_seqlens || !a->block_table) return fail(POP_EINVAL, "cu_seqlens / block_table is NULL");
  if (a->n_seqs < 1 || a->n_seqs > c->max_seqs)
    return fail(POP_EINVAL, "n_seqs %d outside [1, %d]", a->n_seqs, c->max_seqs);
  const int B = a->n_seqs, P = cfg.page_size, maxp = c->max_pages, n_new = max_new_tokens;
  // pages for the prompt and for the n_new - 1 generated tokens that are fed back
  if (pop_status st = slot_map_impl(a->cu_seqlens, B, a->block_table, maxp, P, c->n_pages, nullptr, n_new - 1)) return st;
  const int T = a->cu_seqlens[B];
  const size_t base = pop_workspace_bytes(&cfg, T, B, maxp);
  const size_t need = pop_generate_workspace_bytes(&cfg, T, B, maxp, n_new);
  if (base == 0) return fail(POP_EINVAL, "bad config");
  if (workspace_bytes < need)
    return fail(POP_ENOSPACE, "workspace has %zu bytes, %zu needed to generate %d tokens", workspace_bytes, need, n_new);
  if (cfg.dtype == POP_DTYPE_F32)
    for (int b = 0; b < B; ++b)
      if (a->cu_seqlens[b + 1] - a->cu_seqlens[b] + n_new > pop::f32::kMaxContext)
        return fail(POP_EUNSUPPORTED, "the fp32 path supports sequences up to %d tokens", pop::f32::kMaxContext);
  if (pop_status st = pop_prefill(m, c, a, dev_logits, dev_workspace, base, stream)) return st;

  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  // positions and slots of the fed-back tokens, step-major: entry (s, b) is generated token s of sequence b
  std::vector<int32_t> gmeta((size_t)B * (2 * (size_t)n_new + 1), 0);
  int32_t* g_pos = gmeta.data();
  int32_t* g_slot = g_pos + (size_t)B * n_new;
  int max_len = 0;
  for (int b = 0; b < B; ++b) {
    const int len = a->cu_seqlens[b + 1] - a->cu_seqlens[b];
    max_len = std::max(max_len, len);
    for (int s = 0; s + 1 < n_new; ++s) {
      const int pos = len + s;
      g_pos[(size_t)s * B + b] = pos;
      g_slot[(size_t)s * B + b] = a->block_table[(size_t)b * maxp + pos / P] * P + pos % P;
    }
  }
  char* gbase = reinterpret_cast<char*>(dev_workspace) + base;
  if (pop_status us = upload_meta(c, gbase, gmeta.data(), gmeta.size() * 4, st)) return us;
  const int32_t* d_gpos = reinterpret_cast<const int32_t*>(gbase);
  const int32_t* d_gslot = d_gpos + (size_t)B * n_new;
  int32_t* d_tok = reinterpret_cast<int32_t*>(gbase) + 2 * (size_t)B * n_new;
  void* ws = dev_workspace;
  pop::launch_argmax(dev_logits, cfg.vocab, d_tok, dev_tokens_out, n_new, 0, eos_token, B, st);
  if (cfg.dtype == POP_DTYPE_F32) {
    const WorkspaceF32 w = carve_f32(cfg, T, B, maxp);
    CtxF32 x{m, c, ws, &w, st};
    x.kv_first = c->any_kv_first ? at<int32_t>(ws, w.o_kv_first) : nullptr;   // uploaded by the prefill
    x.B = B;
    float* xb = at<float>(ws, w.o_xb);
    for (int s = 1; s < n_new; ++s) {
      pop::f32::launch_embed((const float*)m->w.embed, d_tok, nullptr, nullptr, xb, B, cfg.d_model, st);
      for (int l = 1; l <= cfg.n_layers; ++l)
        if (pop_status e = layer_f32(x, l, B, xb, at<float>(ws, w.o_ab), at<float>(ws, w.o_qkvb), at<float>(ws, w.o_attnb),
                                     at<float>(ws, w.o_ub), at<int32_t>(ws, w.o_bnd_seq), d_gpos + (size_t)(s - 1) * B,
                                     d_gslot + (size_t)(s - 1) * B, max_len + s))
          return e;
      if (pop_status e = lm_head_f32(x, B, dev_logits)) return e;
      pop::launch_argmax(dev_logits, cfg.vocab, d_tok, dev_tokens_out, n_new, s, eos_token, B, st);
    }
  } else {
    const Workspace w = carve(cfg, T, B, maxp);
    LayerCtx x{m, c, ws, &w, st};
    x.kv_first = c->any_kv_first ? at<int32_t>(ws, w.o_kv_first) : nullptr;   // uploaded by the prefill
    for (int s = 1; s < n_new; ++s) {
      pop::launch_embed((const bf16_t*)m->w.embed, d_tok, nullptr, nullptr, at<float>(ws, w.o_xb), B, cfg.d_model, st);
      x.ab_gamma = nullptr;
      decode_rope_tables(x, d_gpos + (size_t)(s - 1) * B, B);
      for (int l = 1; l <= cfg.n_layers; ++l) {
        const float* next = (const float*)(l < cfg.n_layers ? m->layers[l].norm_in : m->w.final_norm);
        if (pop_status e = decode_layer(x, l, B, d_gpos + (size_t)(s - 1) * B, d_gslot + (size_t)(s - 1) * B, max_len + s,
                                        next))
          return e;
      }
      if (pop_status e = lm_head(x, B, dev_logits)) return e;
      pop::launch_argmax(dev_logits, cfg.vocab, d_tok, dev_tokens_out, n_new, s, eos_token, B, st);
    }
  }
  POP_HIP(hipGetLastError());
  for (int b = 0; b < B; ++b) c->seq_lens[b] += n_new - 1;
  return POP_OK;
}

// ----------------------------------------------------------------------------------------- single steps
pop_status pop_op_rmsnorm(const float* x, const float* gamma, void* out, int32_t rows, int32_t d, float eps,
                          pop_stream stream) {
  if (!x || !gamma || !out) return fail(POP_EINVAL, "NULL pointer");
  if (rows < 0 || d < 8 || d % 8 || d > 8192) return fail(POP_ESHAPE, "rows %d / d %d not supported", rows, d);
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(out)) return fail(POP_EALIGN, "pointer not 16-byte aligned");
  pop::launch_rmsnorm(const_cast<float*>(x), nullptr, nullptr, gamma, (bf16_t*)out, nullptr, rows, d, eps,
                      reinterpret_cast<hipStream_t>(stream));
  POP_HIP(hipGetLastError());
  return POP_OK;
}

pop_status pop_op_gemm(const void* A, int64_t lda, const void* W, int64_t ldw, void* out, int64_t ldc, int32_t M,
                       int32_t N, int32_t K, int32_t epilogue, int32_t act, pop_stream stream) {
  if (!A || !W || !out) return fail(POP_EINVAL, "NULL pointer");
  if (M < 0 || N < 0 || K < 1) return fail(POP_EINVAL, "bad sizes");
  if (epilogue < 0 || epilogue > 3) return fail(POP_EINVAL, "unknown epilogue %d", epilogue);  // fp16 output is internal
  if (K % 8 || lda % 8 || ldw % 8 || ldc % 4 || lda < K || ldw < K || ldc < N)
    return fail(POP_ESHAPE, "K, lda, ldw must be multiples of 8 (ldc of 4) and strides must cover the rows");
  if (!aligned16(A) || !aligned16(W) || !aligned16(out)) return fail(POP_EALIGN, "pointer not 16-byte aligned");
  pop::GemmArgs g{};
  g.A = (const bf16_t*)A; g.lda = lda; g.W = (const bf16_t*)W; g.ldw = ldw; g.out = out; g.ldc = ldc;
  g.M = M; g.N = N; g.K = K; g.epilogue = epilogue; g.act = act; g.batch = 1;
  hipError_t e = pop::launch_gemm(g, reinterpret_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue) return fail(POP_ESHAPE, "operand too large or misaligned for the GEMM kernel");
  if (e != hipSuccess) return fail(POP_EHIP, "GEMM launch failed: %s", hipGetErrorString(e));
  return POP_OK;
}

pop_status pop_op_gemm_splitk(const void* A, int64_t lda, const void* W, int64_t ldw, void* out, int64_t ldc, int32_t M,
                              int32_t N, int32_t K, int32_t epilogue, void* dev_scratch, size_t scratch_bytes,
                              pop_stream stream) {
  if (!A || !W || !out || !dev_scratch) return fail(POP_EINVAL, "NULL pointer");
  if (M < 0 || N < 0 || K < 1) return fail(POP_EINVAL, "bad sizes");
  if (epilogue != 0 && epilogue != 1 && epilogue != 3) return fail(POP_EINVAL, "epilogue %d cannot be split", epilogue);
  if (K % 8 || lda % 8 || ldw % 8 || ldc % 4 || lda < K || ldw < K || ldc < N)
    return fail(POP_ESHAPE, "K, lda, ldw must be multiples of 8 (ldc of 4) and strides must cover the rows");
  if (!aligned16(A) || !aligned16(W) || !aligned16(out) || !aligned16(dev_scratch))
    return fail(POP_EALIGN, "pointer not 16-byte aligned");
  pop::GemmArgs g{};
  g.A = (const bf16_t*)A; g.lda = lda; g.W = (const bf16_t*)W; g.ldw = ldw; g.out = out; g.ldc = ldc;
  g.M = M; g.N = N; g.K = K; g.epilogue = epilogue; g.batch = 1;
  g.splitk_ws = (float*)dev_scratch; g.splitk_ws_bytes = scratch_bytes;
  hipError_t e = pop::launch_gemm(g, reinterpret_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue) return fail(POP_ESHAPE, "operand too large or misaligned for the GEMM kernel");
  if (e != hipSuccess) return fail(POP_EHIP, "GEMM launch failed: %s", hipGetErrorString(e));
  return POP_OK;
}

pop_status pop_op_gemv(const void* x, const void* W, void* out, int64_t ldo, int32_t M, int32_t N, int32_t K,
                       int32_t epilogue, int32_t act, pop_stream stream) {
  if (!x || !W || !out) return fail(POP_EINVAL, "NULL pointer");
  if (M < 0 || M > 64 || N < 0 || K < 8 || K % 8) return fail(POP_ESHAPE, "bad sizes");
  if (epilogue < 0 || epilogue > 2) return fail(POP_EINVAL, "unknown epilogue %d", epilogue);
  if (!aligned16(x) || !aligned16(W) || !aligned16(out)) return fail(POP_EALIGN, "pointer not 16-byte aligned");
  pop::launch_gemv((const bf16_t*)x, (const bf16_t*)W, out, M, N, K, ldo, epilogue, act,
                   reinterpret_cast<hipStream_t>(stream));
  POP_HIP(hipGetLastError());
  return POP_OK;
}

pop_status pop_op_gemv_norm(const void* x, const void* gamma, float eps, const void* W, void* out, int64_t ldo,
                            int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t act, pop_stream stream) {
  if (!x || !gamma || !W || !out) return fail(POP_EINVAL, "NULL pointer");
  if (M < 0 || N < 0 || K < 8 || K % 8) return fail(POP_ESHAPE, "bad sizes");
  if (M > 0 && !pop::gemv_norm_supported(M, K)) return fail(POP_ESHAPE, "the fused form holds at most 4 rows of at most 48 KB in all");
  if (epilogue < 0 || epilogue > 2) return fail(POP_EINVAL, "unknown epilogue %d", epilogue);
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(W) || !aligned16(out))
    return fail(POP_EALIGN, "pointer not 16-byte aligned");
  pop::launch_gemv_norm((const float*)x, (const float*)gamma, eps, (const bf16_t*)W, out, M, N, K, ldo, epilogue, act,
                        reinterpret_cast<hipStream_t>(stream));
  POP_HIP(hipGetLastError());
  return POP_OK;
}

namespace {
struct RopeAttnWs {
  size_t o_pos, o_cu, o_vt_off, o_t64_seq, o_t64_start, o_ta_seq, o_ta_start, o_ta_start2, meta_bytes, o_cs, o_vT, total;
  int Tp_max;
};
RopeAttnWs carve_rope_attn(int T, int B, int Hkv, int hd) {
  RopeAttnWs w{};
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t a = o; o += round_up(bytes, 256); return a; };
  w.Tp_max = (int)round_up((size_t)T + 63 * (size_t)B, 64);
  w.o_pos = take(4 * (size_t)T);
  w.o_cu = take(4 * ((size_t)B + 1));
  w.o_vt_off = take(4 * (size_t)B);
  w.o_t64_seq = take(4 * ((size_t)T / 64 + B));
  w.o_t64_start = take(4 * ((size_t)T / 64 + B));
  w.o_ta_seq = take(4 * ((size_t)T / 128 + B));
  w.o_ta_start = take(4 * ((size_t)T / 128 + B));
  w.o_ta_start2 = take(4 * ((size_t)T / 128 + B));
  w.meta_bytes = o;
  w.o_cs = take(8 * (size_t)T * (hd / 2));
  w.o_vT = take(2 * (size_t)Hkv * hd * w.Tp_max);
  w.total = o;
  return w;
}
}  // namespace

size_t pop_op_rope_attention_workspace(int32_t T, int32_t n_seqs, int32_t n_kv_heads, int32_t head_dim) {
  if (T < 1 || n_seqs < 1 || n_kv_heads < 1 || head_dim < 2) return 0;
  return carve_rope_attn(T, n_seqs, n_kv_heads, head_dim).total;
}

pop_status pop_op_rope_attention(void* qkv, const int32_t* cu, int32_t B, int32_t Hq, int32_t Hkv, int32_t hd,
                                 float rope_theta, int32_t window, void* out, void* workspace, size_t workspace_bytes,
                                 pop_stream stream) {
  if (!qkv || !cu || !out || !workspace) return fail(POP_EINVAL, "NULL pointer");
  if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || window < 0) return fail(POP_EINVAL, "bad head counts / window");
  if (hd != 64 && hd != 128 && hd != 256) return fail(POP_ESHAPE, "head_dim %d is not one of 64, 128, 256", hd);
  if (!aligned16(qkv) || !aligned16(out) || (reinterpret_cast<uintptr_t>(workspace) & 255))
    return fail(POP_EALIGN, "pointer misaligned");
  if (cu[0] != 0) return fail(POP_EINVAL, "cu_seqlens[0] != 0");
  for (int b = 0; b < B; ++b)
    if (cu[b + 1] <= cu[b]) return fail(POP_EINVAL, "sequence %d is empty", b);
  const int T = cu[B];
  const RopeAttnWs w = carve_rope_attn(T, B, Hkv, hd);
  if (workspace_bytes < w.total) return fail(POP_ENOSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  std::vector<unsigned char> meta(w.meta_bytes, 0);
  auto mi = [&](size_t off) { return reinterpret_cast<int32_t*>(meta.data() + off); };
  std::copy(cu, cu + B + 1, mi(w.o_cu));
  int n64 = 0, nta = 0, Tp = 0;
  for (int b = 0; b < B; ++b) {
    const int len = cu[b + 1] - cu[b];
    for (int t = 0; t < len; ++t) mi(w.o_pos)[cu[b] + t] = t;
    mi(w.o_vt_off)[b] = Tp;
    Tp += (int)round_up(len, 64);
    for (int p0 = 0; p0 < len; p0 += 64) { mi(w.o_t64_seq)[n64] = b; mi(w.o_t64_start)[n64++] = p0; }
  }
  nta = build_attention_work(cu, B, mi(w.o_ta_seq), mi(w.o_ta_start), mi(w.o_ta_start2));
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  POP_HIP(hipMemcpyAsync(workspace, meta.data(), w.meta_bytes, hipMemcpyHostToDevice, st));
  POP_HIP(hipStreamSynchronize(st));   // `meta` is pageable memory of this call: wait until it has been read
  const int Dq = Hq * hd, Dkv = Hkv * hd, ld = Dq + 2 * Dkv;
  float2* cs = at<float2>(workspace, w.o_cs);
  bf16_t* vT = at<bf16_t>(workspace, w.o_vT);
  pop::launch_rope_table(at<int32_t>(workspace, w.o_pos), cs, T, hd, (double)rope_theta, st);
  pop::RopeWriteArgs rw{};
  rw.qkv = (bf16_t*)qkv; rw.ld = ld; rw.q_col = 0; rw.k_col = Dq; rw.v_col = Dq + Dkv;
  rw.n_q_heads = Hq; rw.n_kv_heads = Hkv; rw.hd = hd; rw.cs = cs; rw.slot = nullptr;
  rw.k_pool = nullptr; rw.v_pool = nullptr; rw.page_size = 1; rw.vT = vT; rw.Tp = Tp; rw.fp16_inplace = 1;
  rw.kvq = pop::KvQuant{0, 1.f, 1.f, 1.f, 1.f};
  rw.cu_seqlens = at<int32_t>(workspace, w.o_cu); rw.vt_off = at<int32_t>(workspace, w.o_vt_off);
  rw.tile_seq = at<int32_t>(workspace, w.o_t64_seq); rw.tile_start = at<int32_t>(workspace, w.o_t64_start);
  rw.n_tiles = n64;
  pop::launch_rope_write(rw, st);
  pop::AttnPrefillArgs ap{};
  ap.qkv = (const bf16_t*)qkv; ap.ld = ld; ap.q_col = 0; ap.k_col = Dq; ap.vT = vT; ap.Tp = Tp; ap.out = (bf16_t*)out;
  ap.T = T; ap.n_q_heads = Hq; ap.n_kv_heads = Hkv; ap.hd = hd; ap.window = window;
  ap.cu_seqlens = rw.cu_seqlens; ap.vt_off = rw.vt_off;
  ap.tile_seq = at<int32_t>(workspace, w.o_ta_seq); ap.tile_start = at<int32_t>(workspace, w.o_ta_start);
  ap.tile_start2 = at<int32_t>(workspace, w.o_ta_start2);
  ap.n_tiles = nta;
  hipError_t e = pop::launch_attention_prefill(ap, st);
  if (e != hipSuccess) return fail(POP_EHIP, "attention launch failed: %s", hipGetErrorString(e));
  return POP_OK;
}

}  // extern "C"
