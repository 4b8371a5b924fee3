// Host side of libalora: the C ABI of include/alora.h -- argument validation, staging of
// the small per-sequence arrays, workspace management and launch planning.  No arithmetic
// of the method happens here; every step runs in the kernels.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <type_traits>
#include <vector>

#include "../../include/alora.h"
#include "common.h"
#include "mfma_kernels.h"

using namespace alora;

// ---- scratch of the entry point that may not allocate (alora_decode_static) --------------------------------
// One array per GPU the library is loaded on, alive until the process ends.  Host code never uses this name as
// an address: alora_create asks the runtime for the array's device address once per context
// (hipGetSymbolAddress, with the context's device current) and everything below works with that pointer.
constexpr size_t SCRATCH_BYTES = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

namespace {

constexpr int N_SLOTS = 8;

// per-sequence records travel to the device as kernel arguments (no staging buffer, no copy from host memory)
constexpr int STAGE_SEQS = 32;
struct SeqChunk { SeqMeta m[STAGE_SEQS]; };
__global__ void stage_seqs_kernel(SeqChunk c, int n, SeqMeta *dst) {
  if ((int)threadIdx.x < n) dst[threadIdx.x] = c.m[threadIdx.x];
}
// the work list of the decode attention kernel for sequences without shared prefixes, in the order the host
// builds it: item ((row * n_groups) + gb) * n_own + split covers split `split` of row `row`, kv heads gb * heads_per_wg ...
__global__ void make_decode_items_kernel(DecItem *items, int n_items, int n_groups, int heads_per_wg, int n_own) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_items) return;
  DecItem it{};
  it.n_rows = 1;
  it.split = i % n_own;
  it.g = ((i / n_own) % n_groups) * heads_per_wg;
  it.n_splits = n_own;
  it.part = it.split;
  it.shared = 0;
  it.rows[0] = i / (n_own * n_groups);
  items[i] = it;
}

// copies the staged metadata from the pinned host buffer (which the GPU can read directly) into device memory: as a
// kernel it is one more dispatch in the stream's queue, where a copy operation is a hand-over to another engine
__global__ void stage_meta_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int n16) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

struct MetaSlot {
  char *host = nullptr;      // pinned
  char *dev = nullptr;
  size_t cap = 0;            // bytes
  hipEvent_t ev = nullptr;
  bool in_flight = false;
};

}  // namespace

struct ProfEvent {
  hipEvent_t start, stop;
  int kernel;
};

static const char *const KERNEL_NAMES[] = {"prep_rows", "qkv_gemm", "rope_append", "attn_prefill", "attn_decode",
                                           "attn_merge", "o_proj", "mlp_norm", "gate_up", "silu_mul", "down_proj",
                                           "lm_head", "lm_argmax"};
enum KernelId { K_PREP = 0, K_QKV, K_ROPE, K_ATTN_PREFILL, K_ATTN_DECODE, K_ATTN_MERGE, K_OPROJ, K_MLPNORM,
                K_GATEUP, K_SILU, K_DOWN, K_LMHEAD, K_ARGMAX, K_COUNT };

struct alora_ctx {
  int opt_profile = 0;
  std::vector<ProfEvent> prof_pending;
  std::vector<hipEvent_t> prof_free;
  double prof_ms[K_COUNT] = {};
  int64_t prof_n[K_COUNT] = {};
  int device = 0;
  std::string err;
  char *ws = nullptr;
  size_t ws_cap = 0;
  unsigned char *scratch_dev = nullptr;      // device address of the static scratch array on this context's GPU
  float2 *rope = nullptr;
  int rope_pos = 0, rope_half = 0;
  float rope_theta = 0.f;
  MetaSlot slots[N_SLOTS];
  int next_slot = 0;
  int opt_kernels = 0;
  int opt_splits = 0;
  int opt_gemm_splits = 0;
  int opt_gemm_tile = 0;
  int opt_prep_split = 1;        // calls without adapters: 1: many rows take the row-per-wave RMSNorm kernel; 0: never; 2: always
  int opt_attn_waves = 0;
  int opt_lora_split = 0;        // 0 = automatic, 1 = always, 2 = never: low-rank term in workgroups of its own
  int opt_stage_copy = 0;        // 1: the staged metadata travels by hipMemcpyAsync instead of a copy kernel
  int opt_attn_lazy = 3;         // lazy-maximum threshold of the prefill attention kernels, log2 units
  int opt_attn_partials16 = 1;   // split prefill attention (MFMA path): compact partial records
  int opt_rope_fuse = 1;         // rotation + cache append in the epilogue of the QKV projection where the shape allows
  int opt_attn_fold = 1;         // 1 = prefill attention takes prescaled queries and starts its score accumulators at -m_ref
  int n_cu = 256;
};

namespace {

alora_status fail(alora_ctx *ctx, alora_status st, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf;
  return st;
}

#define HIP_TRY(ctx, call)                                                                   \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess)                                                                    \
      return fail(ctx, ALORA_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));           \
  } while (0)

// Brackets one kernel launch with events when profiling is on.
struct ProfScope {
  alora_ctx *ctx;
  hipStream_t s;
  ProfEvent ev{};
  bool on;
  ProfScope(alora_ctx *c, int kernel, hipStream_t st) : ctx(c), s(st), on(c->opt_profile != 0) {
    if (!on) return;
    ev.kernel = kernel;
    for (hipEvent_t *e : {&ev.start, &ev.stop}) {
      if (!ctx->prof_free.empty()) { *e = ctx->prof_free.back(); ctx->prof_free.pop_back(); }
      else if (hipEventCreate(e) != hipSuccess) { on = false; return; }
    }
    (void)hipEventRecord(ev.start, s);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(ev.stop, s);
    ctx->prof_pending.push_back(ev);
  }
};

struct Bump {
  char *base;
  size_t off = 0;
  explicit Bump(char *b) : base(b) {}
  template <typename U> U *take(size_t n) {
    size_t bytes = (n * sizeof(U) + 255) & ~(size_t)255;
    U *p = base ? reinterpret_cast<U *>(base + off) : nullptr;
    off += bytes;
    return p;
  }
};

alora_status ensure_workspace(alora_ctx *ctx, size_t bytes) {
  if (bytes <= ctx->ws_cap) return ALORA_OK;
  HIP_TRY(ctx, hipDeviceSynchronize());        // earlier calls may still be using the old block
  if (ctx->ws) HIP_TRY(ctx, hipFree(ctx->ws));
  ctx->ws = nullptr;
  ctx->ws_cap = 0;
  size_t want = bytes + bytes / 8;
  HIP_TRY(ctx, hipMalloc((void **)&ctx->ws, want));
  ctx->ws_cap = want;
  return ALORA_OK;
}

alora_status ensure_rope(alora_ctx *ctx, int n_pos, int half, float theta, hipStream_t s) {
  if (ctx->rope && ctx->rope_pos >= n_pos && ctx->rope_half == half && ctx->rope_theta == theta)
    return ALORA_OK;
  HIP_TRY(ctx, hipDeviceSynchronize());
  if (ctx->rope) HIP_TRY(ctx, hipFree(ctx->rope));
  ctx->rope = nullptr;
  int want = std::max(n_pos + n_pos / 4, 4096);
  HIP_TRY(ctx, hipMalloc((void **)&ctx->rope, (size_t)want * half * sizeof(float2)));
  launch_rope_table(ctx->rope, want, half, theta, s);
  HIP_TRY(ctx, hipGetLastError());
  ctx->rope_pos = want;
  ctx->rope_half = half;
  ctx->rope_theta = theta;
  return ALORA_OK;
}

alora_status acquire_slot(alora_ctx *ctx, size_t bytes, MetaSlot **out) {
  MetaSlot &sl = ctx->slots[ctx->next_slot];
  ctx->next_slot = (ctx->next_slot + 1) % N_SLOTS;
  if (sl.in_flight) {
    HIP_TRY(ctx, hipEventSynchronize(sl.ev));
    sl.in_flight = false;
  }
  if (sl.cap < bytes) {
    // grow every slot of the ring now, not one per call: each growth is an allocation (and a wait for the slot's
    // last user), which belongs in the first call of a given size and not in the seven after it
    const size_t cap = (std::max<size_t>(4096, bytes + bytes / 2) + 15) & ~(size_t)15;
    for (MetaSlot &o : ctx->slots) {
      if (o.cap >= cap) continue;
      if (o.in_flight) {
        HIP_TRY(ctx, hipEventSynchronize(o.ev));
        o.in_flight = false;
      }
      if (o.host) HIP_TRY(ctx, hipHostFree(o.host));
      if (o.dev) HIP_TRY(ctx, hipFree(o.dev));
      o.host = nullptr; o.dev = nullptr; o.cap = 0;
      HIP_TRY(ctx, hipHostMalloc((void **)&o.host, cap, hipHostMallocDefault));
      HIP_TRY(ctx, hipMalloc((void **)&o.dev, cap));
      o.cap = cap;
      if (!o.ev) HIP_TRY(ctx, hipEventCreateWithFlags(&o.ev, hipEventDisableTiming));
    }
  }
  if (!sl.ev) HIP_TRY(ctx, hipEventCreateWithFlags(&sl.ev, hipEventDisableTiming));
  *out = &sl;
  return ALORA_OK;
}

struct Plan {
  LayerDims L;
  int T = 0, B = 0;
  int max_len = 0;        // max over sequences of P_b + S_b
  bool any_adapter = false;
  bool any_prefix = false;   // some sequence reads a shared prefix
  std::vector<SeqMeta> seqs;
};

alora_status check_layer(alora_ctx *ctx, const alora_layer_desc *ly, bool need_tail, LayerDims *L) {
  if (!ly) return fail(ctx, ALORA_EINVAL, "layer descriptor is NULL");
  if (ly->dtype != ALORA_F32 && ly->dtype != ALORA_BF16)
    return fail(ctx, ALORA_EDTYPE, "dtype %d is neither ALORA_F32 nor ALORA_BF16", ly->dtype);
  if (ly->d < 1 || ly->d > 16000) return fail(ctx, ALORA_ESHAPE, "d = %d outside [1, 16000]", ly->d);
  if (ly->n_q_heads < 1 || ly->n_kv_heads < 1 || ly->n_q_heads % ly->n_kv_heads != 0)
    return fail(ctx, ALORA_ESHAPE, "n_q_heads = %d must be a positive multiple of n_kv_heads = %d",
                ly->n_q_heads, ly->n_kv_heads);
  if (ly->head_dim < 2 || ly->head_dim > 256 || (ly->head_dim & 1))
    return fail(ctx, ALORA_ESHAPE, "head_dim = %d must be even and in [2, 256]", ly->head_dim);
  if (ly->n_adapters < 0) return fail(ctx, ALORA_ESHAPE, "n_adapters = %d is negative", ly->n_adapters);
  if (ly->rank < 0 || ly->rank > 256 || (ly->n_adapters > 0 && ly->rank < 1))
    return fail(ctx, ALORA_ESHAPE, "rank = %d outside [1, 256]", ly->rank);
  if (!ly->W_qkv) return fail(ctx, ALORA_EINVAL, "W_qkv is NULL");
  if (ly->n_adapters > 0 && (!ly->A || !ly->B_q || !ly->B_k || !ly->B_v || !ly->scale))
    return fail(ctx, ALORA_EINVAL, "adapter tensors (A, B_q, B_k, B_v, scale) must be given when n_adapters > 0");
  if (!(ly->rope_theta > 0.f)) return fail(ctx, ALORA_ESHAPE, "rope_theta must be positive");
  if (need_tail) {
    if (ly->intermediate < 1) return fail(ctx, ALORA_ESHAPE, "intermediate = %d must be positive", ly->intermediate);
    if (!ly->W_o || !ly->rms2_gain || !ly->W_gate || !ly->W_up || !ly->W_down)
      return fail(ctx, ALORA_EINVAL, "W_o, rms2_gain, W_gate, W_up and W_down are required for a layer stack");
    const bool any_rest = ly->A_o || ly->B_o || ly->A_gu || ly->B_gate || ly->B_up || ly->A_down || ly->B_down;
    if (any_rest && ly->n_adapters < 1)
      return fail(ctx, ALORA_EINVAL, "adapters of W_o / the MLP are given but n_adapters = 0");
    if ((ly->A_o != nullptr) != (ly->B_o != nullptr)) return fail(ctx, ALORA_EINVAL, "A_o and B_o go together");
    if ((ly->A_down != nullptr) != (ly->B_down != nullptr)) return fail(ctx, ALORA_EINVAL, "A_down and B_down go together");
    if ((ly->A_gu != nullptr) != (ly->B_gate != nullptr) || (ly->A_gu != nullptr) != (ly->B_up != nullptr))
      return fail(ctx, ALORA_EINVAL, "A_gu, B_gate and B_up go together");
  }
  L->d = ly->d; L->n_q_heads = ly->n_q_heads; L->n_kv_heads = ly->n_kv_heads; L->head_dim = ly->head_dim;
  L->rank = ly->rank; L->n_adapters = ly->n_adapters;
  L->n_q = ly->n_q_heads * ly->head_dim;
  L->n_kv = ly->n_kv_heads * ly->head_dim;
  L->n_qkv = L->n_q + 2 * L->n_kv;
  return ALORA_OK;
}

alora_status check_batch(alora_ctx *ctx, const alora_layer_desc *ly, const alora_kv_cache *cache,
                         const int32_t *cu, const int32_t *kps, const int32_t *aps, int B, int n_steps, Plan *pl) {
  if (!cache) return fail(ctx, ALORA_EINVAL, "cache is NULL");
  if (B < 1) return fail(ctx, ALORA_EINVAL, "B = %d must be at least 1", B);
  if (!cu || !kps || !aps) return fail(ctx, ALORA_EINVAL, "cu_seqlens / k_per_seq / adapter_per_seq is NULL");
  if (!cache->seq_offset || !cache->seq_capacity || !cache->seq_len)
    return fail(ctx, ALORA_EINVAL, "cache seq_offset / seq_capacity / seq_len is NULL");
  if (!cache->k || !cache->v) return fail(ctx, ALORA_EINVAL, "cache k / v is NULL");
  if (cache->prefix_len && !cache->prefix_offset)
    return fail(ctx, ALORA_EINVAL, "cache prefix_len is given without prefix_offset");
  if (cu[0] != 0) return fail(ctx, ALORA_EINVAL, "cu_seqlens[0] = %d must be 0", cu[0]);
  pl->B = B;
  pl->seqs.resize(B);
  pl->max_len = 0;
  pl->any_adapter = false;
  pl->any_prefix = false;
  for (int b = 0; b < B; ++b) {
    const int S = cu[b + 1] - cu[b];
    if (S < 0) return fail(ctx, ALORA_EINVAL, "cu_seqlens decreases at sequence %d", b);
    const int P = cache->seq_len[b];
    const int cap = cache->seq_capacity[b];
    const int64_t off = cache->seq_offset[b];
    if (P < 0) return fail(ctx, ALORA_EINVAL, "seq_len[%d] = %d is negative", b, P);
    if (kps[b] < 0) return fail(ctx, ALORA_EINVAL, "k_per_seq[%d] = %d is negative", b, kps[b]);
    if (aps[b] < -1 || aps[b] >= ly->n_adapters)
      return fail(ctx, ALORA_EADAPTER, "adapter_per_seq[%d] = %d outside [-1, %d)", b, aps[b], ly->n_adapters);
    if (cap < 0 || off < 0 || off + cap > cache->pool_tokens)
      return fail(ctx, ALORA_ECAPACITY, "sequence %d: rows [%lld, %lld) lie outside the pool of %lld tokens", b,
                  (long long)off, (long long)(off + cap), (long long)cache->pool_tokens);
    const int plen = cache->prefix_len ? cache->prefix_len[b] : 0;
    const int64_t poff = plen > 0 ? cache->prefix_offset[b] : 0;
    if (plen < 0 || plen > P)
      return fail(ctx, ALORA_EINVAL, "sequence %d: prefix_len = %d outside [0, seq_len = %d]", b, plen, P);
    if (plen > 0 && (poff < 0 || poff + plen > cache->pool_tokens))
      return fail(ctx, ALORA_ECAPACITY, "sequence %d: shared prefix rows [%lld, %lld) lie outside the pool of %lld tokens",
                  b, (long long)poff, (long long)(poff + plen), (long long)cache->pool_tokens);
    const int64_t grown = (int64_t)P + (int64_t)S * n_steps;      // cached length after the call
    if (grown - plen > cap)
      return fail(ctx, ALORA_ECAPACITY, "sequence %d: %d cached + %lld new tokens exceed its capacity %d", b, P - plen,
                  (long long)S * n_steps, cap);
    if (grown > (1 << 24))
      return fail(ctx, ALORA_ECAPACITY, "sequence %d: position %lld beyond the supported 2^24", b, (long long)grown);
    SeqMeta &m = pl->seqs[b];
    m.row_start = cu[b]; m.n_new = S; m.P = P; m.k = kps[b]; m.adapter = aps[b];
    m.scale = aps[b] >= 0 ? ly->scale[aps[b]] : 0.f;
    m.pool_off = off - plen;
    m.prefix_off = poff;
    m.prefix_len = plen;
    m.pad_ = 0;
    if (plen > 0) pl->any_prefix = true;
    if (aps[b] >= 0 && S > 0 && grown > kps[b]) pl->any_adapter = true;
    pl->max_len = std::max(pl->max_len, (int)grown);
  }
  pl->T = cu[B];
  // The regions the sequences own must be disjoint, and nobody may write where somebody reads a shared prefix:
  // the kernels would write those cache rows concurrently, silently.
  {
    struct Iv { int64_t lo, hi; int b; };
    std::vector<Iv> own, wr, pf;
    for (int b = 0; b < B; ++b) {
      const SeqMeta &m = pl->seqs[b];
      const int64_t off = cache->seq_offset[b];
      if (cache->seq_capacity[b] > 0) own.push_back(Iv{off, off + cache->seq_capacity[b], b});
      if (m.n_new > 0) {
        const int64_t w0 = off + (m.P - m.prefix_len);
        wr.push_back(Iv{w0, w0 + (int64_t)m.n_new * n_steps, b});
      }
      if (m.prefix_len > 0) pf.push_back(Iv{m.prefix_off, m.prefix_off + m.prefix_len, b});
    }
    auto by_lo = [](const Iv &x, const Iv &y) { return x.lo < y.lo; };
    std::sort(own.begin(), own.end(), by_lo);
    for (size_t i = 1; i < own.size(); ++i)
      if (own[i].lo < own[i - 1].hi)
        return fail(ctx, ALORA_ECAPACITY, "sequences %d and %d own overlapping cache rows [%lld, %lld) and [%lld, %lld)",
                    own[i - 1].b, own[i].b, (long long)own[i - 1].lo, (long long)own[i - 1].hi, (long long)own[i].lo,
                    (long long)own[i].hi);
    if (!pf.empty() && !wr.empty()) {
      std::sort(wr.begin(), wr.end(), by_lo);       // disjoint (inside disjoint regions), so sorted by hi as well
      std::sort(pf.begin(), pf.end(), by_lo);
      size_t j = 0;
      for (const Iv &p : pf) {
        while (j < wr.size() && wr[j].hi <= p.lo) ++j;     // prefixes come in ascending lo: skipped writes end before all later ones too
        for (size_t q = j; q < wr.size() && wr[q].lo < p.hi; ++q)
          if (wr[q].hi > p.lo)
            return fail(ctx, ALORA_ECAPACITY, "sequence %d would write rows [%lld, %lld) that sequence %d reads as its shared prefix",
                        wr[q].b, (long long)wr[q].lo, (long long)wr[q].hi, p.b);
      }
    }
  }
  return ALORA_OK;
}

// decode batches have one row per sequence: the sequence whose new token is packed row `row`
static int a_seq_of_row(const Plan &pl, int row) {
  for (int b = 0; b < pl.B; ++b)
    if (pl.seqs[b].n_new > 0 && pl.seqs[b].row_start == row) return b;
  return 0;
}

struct Workspace {
  RowMeta rm;
  void *xh;        // [T, d]
  float *tlow;     // [T, 3r]
  float *Y;        // [k_splits, T, n_qkv] fp32 projection partials; also split-K scratch of the dense layers
  size_t y_floats;
  void *Q;         // [T, n_q]
  float *partials;
  // layer-stack buffers
  void *attn, *h1, *hn, *gate, *up, *xa, *xb;
  int dec_hw = 1, dec_kr = 1, dec_cols_max = 1;      // shape of the decode attention workgroups
  float *f0 = nullptr, *f1 = nullptr;      // plain bf16 stack: sums of a linear before their one rounding
  size_t bytes;
  bool mfma = false;
  int k_splits = 1;                  // workgroups per output tile along the reduction axis of the QKV projection
  int k_segments = 1;                // its fixed reduction segments (from the weight shape alone)
  int lora_split = 0;                // the low-rank term of the QKV projection has a partial of its own
  bool attn_mfma = false;
  bool decode_mfma = false;
  int attn_waves = 8;
  const AttnItem *qtiles = nullptr;
  int n_qtiles = 0;
  const DecItem *ditems = nullptr;   // work list of the MFMA decode kernel
  int n_ditems = 0;
  const float *scale_dev = nullptr;  // [n_adapters] s_a on the device (adapters of W_o / the MLP)
  bool any_adapter = false;
  const float2 *rope = nullptr;      // rotary table: one line per position, or (rope_by_row) one per packed row
  bool rope_by_row = false;
  float2 *rope_rows = nullptr;       // where the per-row table is built after row preparation
};

int pick_splits(const alora_ctx *ctx, int T, int n_kv_heads, int max_len) {
  if (ctx->opt_splits > 0) return ctx->opt_splits;
  // enough (row, kv head, split) work items to fill the chip, chunks of at least 256 keys
  int64_t items = (int64_t)T * n_kv_heads;
  int want = (int)std::min<int64_t>(64, std::max<int64_t>(1, (4 * ctx->n_cu + items - 1) / std::max<int64_t>(items, 1)));
  int max_by_len = std::max(1, max_len / 256);
  return std::max(1, std::min(want, max_by_len));
}

Workspace layout_workspace(char *base, const LayerDims &L, int T, size_t esz, int n_splits, int k_splits,
                           int intermediate, bool stack, bool f32_tail = false) {
  Bump b(base);
  Workspace w{};
  w.rm.seq = b.take<int32_t>(T);
  w.rm.pos = b.take<int32_t>(T);
  w.rm.adapter = b.take<int32_t>(T);
  w.rm.slot = b.take<int64_t>(T);
  w.rm.present16 = b.take<unsigned long long>((T + 15) / 16);
  w.xh = b.take<char>((size_t)T * L.d * esz);
  w.tlow = b.take<float>((size_t)T * 3 * std::max(L.rank, 1));
  w.y_floats = (size_t)T * L.n_qkv * (std::max(k_splits, 1) + 1);
  if (stack) {      // split-K partials of W_o / W_down and of the down-projections of their adapters
    w.y_floats = std::max(w.y_floats, (size_t)8 * T * L.d);
    w.y_floats = std::max(w.y_floats, (size_t)8 * T * std::max(L.n_adapters, 1) * 2 * std::max(L.rank, 1));
  }
  w.Y = b.take<float>(w.y_floats);
  w.Q = b.take<char>((size_t)T * L.n_q * 4);      // fp16 for the MFMA attention kernels, fp32 for the plain one
  w.partials = b.take<float>(attn_plain_partial_floats(L, T, n_splits));
  if (stack) {
    w.attn = b.take<char>((size_t)T * L.n_q * esz);
    w.h1 = b.take<char>((size_t)T * L.d * esz);
    w.hn = b.take<char>((size_t)T * L.d * esz);
    w.gate = b.take<char>((size_t)T * intermediate * esz);
    w.up = b.take<char>((size_t)T * intermediate * esz);
    w.xa = b.take<char>((size_t)T * L.d * esz);
    w.xb = b.take<char>((size_t)T * L.d * esz);
    if (f32_tail) {
      w.f0 = b.take<float>((size_t)T * std::max(intermediate, L.d));
      w.f1 = b.take<float>((size_t)T * std::max(intermediate, L.d));
    }
  }
  w.bytes = b.off;
  return w;
}

// One attention block on already-staged metadata: rows -> projections -> rotation/append ->
// attention.  write_meta is false for layers after the first of a stack (same rows).
template <typename T>
void attention_block(alora_ctx *ctx, const alora_layer_desc *ly, const LayerDims &L, const alora_kv_cache *cache,
                     const T *x, const Plan &pl, const SeqMeta *seqs_dev, const Workspace &w, bool write_meta,
                     int n_splits, bool decode, int pos_shift, T *out, hipStream_t s) {
  const bool mfma = w.mfma && std::is_same<T, bf16>::value;
  const int rank_used = pl.any_adapter ? L.rank : 0;
  const bool prep_mfma = mfma && prep_rows_mfma_supported(L.d, rank_used);      // it also leaves the adapter masks
  {
    ProfScope p(ctx, K_PREP, s);
    if (prep_mfma) {
      PrepArgs pa{};
      pa.x = (const bf16 *)x; pa.gain = (const bf16 *)ly->rms_gain; pa.eps = ly->rms_eps;
      pa.T = pl.T; pa.d = L.d; pa.seqs = seqs_dev; pa.n_seqs = pl.B; pa.pos_shift = pos_shift;
      pa.one = pl.seqs[0];
      pa.A = rank_used ? (const bf16 *)ly->A : nullptr; pa.rank = rank_used;
      pa.n_adapters = L.n_adapters;
      pa.write_meta = write_meta ? 1 : 0;
      pa.xh = (bf16 *)w.xh; pa.tlow16 = (bf16 *)w.tlow; pa.rm = w.rm;
      // Many rows and no adapter in the call (a base-model prefill): the kernel that holds 16 rows per workgroup
      // in registers runs one workgroup per compute unit and needs several rounds; a row-per-wave kernel does
      // metadata and RMSNorm at streaming rate, with the same bits.
      if (rank_used == 0 && ctx->opt_prep_split != 0 && norm_rows_mfma_supported(L.d) &&
          (pl.T >= 512 || ctx->opt_prep_split == 2))
        launch_norm_rows_mfma(pa, s);
      else
        launch_prep_rows_mfma(pa, s);
    } else {
      launch_prep_rows<T>(x, (const T *)ly->rms_gain, ly->rms_eps, pl.T, L.d, seqs_dev, pl.B, pos_shift,
                          (const T *)ly->A, rank_used, write_meta, (T *)w.xh, w.tlow, mfma ? (bf16 *)w.tlow : nullptr, w.rm, s);
    }
  }
  if (w.rope_by_row) launch_rope_rows(w.rope_rows, w.rm.pos, pl.T, L.head_dim / 2, ly->rope_theta, s);
  // the MFMA attention kernels (prefill and decode) take their queries as fp16 (every operand of its matrix products is fp16),
  // in its folded-softmax form premultiplied by sm_scale * log2(e)
  // (the plain attention kernel reads them as fp32: the Q buffer holds four bytes per element)
  const bool q_half = (w.attn_mfma || w.decode_mfma) && std::is_same<T, bf16>::value;
  const int q_mode = q_half ? 1 : 2;
  const float q_scale = (w.attn_mfma && q_half) ? attn_prefill_mfma_q_scale(L, ctx->opt_attn_fold != 0) : 1.0f;
  bool rope_fused = false;
  {
    ProfScope p(ctx, K_QKV, s);
    if (mfma) {
      GemmArgs g{};
      g.A = (const bf16 *)w.xh; g.lda = L.d;
      g.B = (const bf16 *)ly->W_qkv; g.ldb = L.d;
      g.M = pl.T; g.N = L.n_qkv; g.K = L.d;
      g.k_splits = w.k_splits;
      g.k_segments = w.k_segments;
      g.lora_split = (pl.any_adapter && w.lora_split) ? 1 : 0;
      g.tile_hint = ctx->opt_gemm_tile;
      g.Cpart = w.Y;
      g.tlow = pl.any_adapter ? (const bf16 *)w.tlow : nullptr;
      g.rank = L.rank;
      g.lr_parts = 3;
      g.Bq = (const bf16 *)ly->B_q; g.Bk = (const bf16 *)ly->B_k; g.Bv = (const bf16 *)ly->B_v;
      g.n_q = L.n_q; g.n_kv = L.n_kv;
      g.row_adapter = w.rm.adapter;
      g.present16 = prep_mfma ? w.rm.present16 : nullptr;
      // many rows, unsplit reduction, one head per column tile: rotation and cache append happen in the
      // projection's epilogue and the fp32 projection never goes to memory
      if (ctx->opt_gemm_tile == 0 && ctx->opt_rope_fuse && q_half && !w.rope_by_row &&
          gemm_mfma_rope_supported(g, L.head_dim)) {
        g.rope_pos = w.rm.pos; g.rope_slot = w.rm.slot; g.rope_table = w.rope; g.q_scale = q_scale;
        g.Qout = (bf16 *)w.Q; g.cacheK = (bf16 *)cache->k; g.cacheV = (bf16 *)cache->v;
        g.q_half = q_half ? 1 : 0;
        launch_gemm_mfma(g, GEMM_EPI_ROPE, s);
        rope_fused = true;
      } else {
        launch_gemm_mfma(g, GEMM_EPI_PARTIAL, s);
      }
    } else {
      launch_qkv_gemm_plain<T>((const T *)w.xh, (const T *)ly->W_qkv, w.tlow, (const T *)ly->B_q,
                               (const T *)ly->B_k, (const T *)ly->B_v, L, w.rm, pl.T, w.Y, s);
    }
  }
  if (!rope_fused) {
    ProfScope p(ctx, K_ROPE, s);
    launch_rope_append<T>(w.Y, mfma ? w.k_splits + ((pl.any_adapter && w.lora_split) ? 1 : 0) : 1, L, w.rm, pl.T, w.rope, w.rope_by_row, q_scale, q_mode, w.Q,
                          (T *)cache->k, (T *)cache->v, s);
  }
  const bool direct = w.attn_mfma && std::is_same<T, bf16>::value && n_splits == 1;
  // split prefill attention on the MFMA path: partial results travel in the compact record
  const bool compact16 = w.attn_mfma && std::is_same<T, bf16>::value && !direct && ctx->opt_attn_partials16;
  {
    ProfScope p(ctx, decode ? K_ATTN_DECODE : K_ATTN_PREFILL, s);
    if (w.attn_mfma && std::is_same<T, bf16>::value) {
      AttnArgs a{};
      a.Q = (const _Float16 *)w.Q; a.K = (const bf16 *)cache->k; a.V = (const bf16 *)cache->v;
      a.work = w.qtiles;
      a.n_q = L.n_q; a.n_kv = L.n_kv; a.n_q_heads = L.n_q_heads; a.n_kv_heads = L.n_kv_heads;
      a.n_parts = n_splits;
      a.sm_scale = 1.0f / sqrtf((float)L.head_dim);
      a.lazy = (float)ctx->opt_attn_lazy;
      a.q_prescaled = q_scale != 1.0f;
      a.partials = direct ? nullptr : w.partials;
      a.compact = compact16 ? 1 : 0;
      a.out = direct ? (bf16 *)out : nullptr;
      // the kernels' fast tile loads use 32-bit byte offsets from an item's first key row; (absurdly) long
      // sequences take the variant with full address arithmetic
      bool generic_addr = false;
      for (const SeqMeta &q : pl.seqs)
        if ((uint64_t)(q.P + q.n_new) * (uint64_t)L.n_kv * 2u >= (1ull << 31)) generic_addr = true;
      launch_attn_prefill_mfma(a, w.n_qtiles, L.n_q_heads / L.n_kv_heads, w.attn_waves, generic_addr, s);
    } else if (w.decode_mfma && std::is_same<T, bf16>::value) {
      DecodeArgs a{};
      a.Q = (const _Float16 *)w.Q; a.K = (const bf16 *)cache->k; a.V = (const bf16 *)cache->v;
      a.seqs = seqs_dev; a.rm = w.rm;
      a.n_q = L.n_q; a.n_kv = L.n_kv; a.n_q_heads = L.n_q_heads; a.n_kv_heads = L.n_kv_heads;
      a.items = w.ditems;
      a.n_parts = n_splits;
      a.heads_per_wg = w.dec_hw; a.ranges_per_wg = w.dec_kr; a.cols_max = w.dec_cols_max;
      a.sm_scale = 1.0f / sqrtf((float)L.head_dim);
      a.partials = w.partials;
      launch_attn_decode_mfma(a, w.n_ditems, s);
    } else {
      launch_attn_plain<T>((const float *)w.Q, (const T *)cache->k, (const T *)cache->v, seqs_dev, w.rm, L, pl.T,
                           n_splits, w.partials, s);
    }
  }
  if (!direct) {
    ProfScope p(ctx, K_ATTN_MERGE, s);
    if (compact16) launch_attn_merge16(w.partials, L, pl.T, n_splits, (bf16 *)out, s);
    else launch_attn_merge<T>(w.partials, L, pl.T, n_splits, out, s);
  }
}

template <typename T>
void layer_tail(alora_ctx *ctx, const alora_layer_desc *ly, const LayerDims &L, const T *x, const Workspace &w,
                int T_rows, T *out, hipStream_t s) {
  RowMeta none{};
  const bool mfma = w.mfma && std::is_same<T, bf16>::value;
  const int r = L.rank, n_ad = L.n_adapters;
  // Adapters of these linears (Eq.6 applied to them): on the MFMA path t = s_a A_a z is computed for all
  // adapters at once as a skinny GEMM against the stacked down-matrices [n_ad * parts * r, K] (exactly how
  // they are stored), each adapted row then picks its adapter's slice as a bf16 (hi, lo) pair, and the
  // up-projection runs as extra k-steps of the base GEMM; on the plain path the term is added afterwards.
  auto lowrank_t = [&](const void *z, int K, const void *A_all, int parts) {
    GemmArgs g{};
    g.A = (const bf16 *)z; g.lda = K;
    g.B = (const bf16 *)A_all; g.ldb = K;
    g.M = T_rows; g.N = n_ad * parts * r; g.K = K;
    int splits = gemm_mfma_pick_splits(T_rows, g.N, K, ctx->n_cu);
    while (splits > 1 && (size_t)splits * T_rows * g.N > w.y_floats) splits /= 2;
    g.k_splits = splits;
    g.k_segments = splits;
    g.Cpart = w.Y;
    launch_gemm_mfma(g, GEMM_EPI_PARTIAL, s);
    launch_tlow_select(w.Y, splits, T_rows, n_ad, parts, r, w.rm.adapter, w.scale_dev, (bf16 *)w.tlow, s);
  };
  auto set_lowrank = [&](GemmArgs &g, const void *B0, const void *B1, int parts, int width) {
    g.tlow = (const bf16 *)w.tlow; g.rank = r; g.lr_parts = parts;
    g.Bq = (const bf16 *)B0; g.Bk = (const bf16 *)B1; g.Bv = nullptr;
    g.n_q = width; g.n_kv = parts == 1 ? 0 : width;
    g.row_adapter = w.rm.adapter;
    g.present16 = prep_rows_mfma_supported(L.d, r) ? w.rm.present16 : nullptr;      // (the row preparation that wrote it)
  };
  // reduction segments of a linear [N, K]: fixed by the weight shape (or by the gemm_splits option), so that a
  // row's result does not depend on the number of rows in the call
  auto segments_of = [&](int N, int K) {
    if (ctx->opt_gemm_splits > 0) return K % (64 * ctx->opt_gemm_splits) == 0 ? ctx->opt_gemm_splits : 1;
    return gemm_mfma_fixed_segments(N, K, ctx->n_cu);
  };
  // C = A W^T (+ R), with the gated low-rank term of (Al, Bl) when given
  auto dense = [&](const void *A, const void *W, const void *R, void *C, int N, int K, const void *Al, const void *Bl,
                   int parts = 1, int part = 0) {
    const bool lr = Al != nullptr && w.any_adapter;
    if (mfma) {
      if (lr) lowrank_t(A, K, Al, 1);
      GemmArgs g{};
      g.A = (const bf16 *)A; g.lda = K;
      g.B = (const bf16 *)W; g.ldb = K;
      g.M = T_rows; g.N = N; g.K = K;
      g.tile_hint = (ctx->opt_gemm_tile >= 4 || ctx->opt_gemm_tile == 1) ? ctx->opt_gemm_tile : 0;
      if (lr) set_lowrank(g, Bl, nullptr, 1, N);
      // few row tiles: every segment gets workgroups of its own to fill the chip, the segment sums go through
      // the Y buffer; otherwise one workgroup adds them itself, in the same order
      const int segs = segments_of(N, K);
      g.k_segments = segs;
      if (segs > 1 && gemm_mfma_split_segments(T_rows, N, ctx->n_cu) && (size_t)segs * T_rows * N <= w.y_floats &&
          ((int64_t)T_rows * N) % 4 == 0) {
        g.k_splits = segs;
        g.Cpart = w.Y;
        launch_gemm_mfma(g, GEMM_EPI_PARTIAL, s);
        launch_splitk_reduce(w.Y, segs, (int64_t)T_rows * N, (const bf16 *)R, (bf16 *)C, s);
      } else {
        g.k_splits = 1;
        g.C = (bf16 *)C; g.ldc = N; g.R = (const bf16 *)R;
        launch_gemm_mfma(g, GEMM_EPI_BF16, s);
      }
    } else if (w.f0 != nullptr) {
      // bf16 on the plain kernels: base product, low-rank term and residual are added in fp32 and rounded once
      launch_gemm_plain_f32<T>((const T *)A, (const T *)W, w.f0, T_rows, N, K, s);
      if (lr)
        launch_lowrank_add_plain<T, float>((const T *)A, K, (const T *)Al, parts, part, (const T *)Bl, N, r, w.rm.adapter,
                                           w.scale_dev, w.f0, T_rows, s);
      launch_residual_store<T>(w.f0, (const T *)R, (T *)C, (int64_t)T_rows * N, s);
    } else {
      launch_gemm_plain<T>((const T *)A, (const T *)W, (const T *)R, (T *)C, T_rows, N, K, s);
      if (lr)
        launch_lowrank_add_plain<T, T>((const T *)A, K, (const T *)Al, parts, part, (const T *)Bl, N, r, w.rm.adapter,
                                       w.scale_dev, (T *)C, T_rows, s);
    }
  };
  // h1 = x + attn W_o^T, hn = RMSNorm(h1).  When the projection is split over the reduction axis anyway, the
  // kernel that adds the partial sums also normalises the row (from its fp32 value) -- one launch less.
  bool normed = false;
  {
    ProfScope p(ctx, K_OPROJ, s);
    const int splits = mfma ? segments_of(L.d, L.n_q) : 1;
    if (mfma && splits > 1 && gemm_mfma_split_segments(T_rows, L.d, ctx->n_cu) &&
        (size_t)splits * T_rows * L.d <= w.y_floats && splitk_reduce_norm_supported(L.d)) {
      GemmArgs g{};
      g.A = (const bf16 *)w.attn; g.lda = L.n_q;
      g.B = (const bf16 *)ly->W_o; g.ldb = L.n_q;
      g.M = T_rows; g.N = L.d; g.K = L.n_q;
      g.tile_hint = (ctx->opt_gemm_tile >= 4 || ctx->opt_gemm_tile == 1) ? ctx->opt_gemm_tile : 0;
      if (ly->A_o && w.any_adapter) {
        lowrank_t(w.attn, L.n_q, ly->A_o, 1);
        set_lowrank(g, ly->B_o, nullptr, 1, L.d);
      }
      g.k_splits = splits;
      g.k_segments = splits;
      g.Cpart = w.Y;
      launch_gemm_mfma(g, GEMM_EPI_PARTIAL, s);
      launch_splitk_reduce_norm(w.Y, splits, T_rows, L.d, (const bf16 *)x, (const bf16 *)ly->rms2_gain, ly->rms_eps,
                                (bf16 *)w.h1, (bf16 *)w.hn, s);
      normed = true;
    } else {
      dense(w.attn, ly->W_o, x, w.h1, L.d, L.n_q, ly->A_o, ly->B_o);
    }
  }
  if (!normed) {
    ProfScope p(ctx, K_MLPNORM, s);
    if (mfma && prep_rows_mfma_supported(L.d, 0)) {
      PrepArgs pa{};
      pa.x = (const bf16 *)w.h1; pa.gain = (const bf16 *)ly->rms2_gain; pa.eps = ly->rms_eps;
      pa.T = T_rows; pa.d = L.d; pa.xh = (bf16 *)w.hn; pa.rm = none;
      launch_prep_rows_mfma(pa, s);
    } else {
      launch_prep_rows<T>((const T *)w.h1, (const T *)ly->rms2_gain, ly->rms_eps, T_rows, L.d, nullptr, 0, 0,
                          (const T *)nullptr, 0, false, (T *)w.hn, nullptr, nullptr, none, s);
    }
  }
  if (mfma) {   // act = silu(hn W_gate^T) * (hn W_up^T) in one pass
    ProfScope p(ctx, K_GATEUP, s);
    GemmArgs g{};
    g.A = (const bf16 *)w.hn; g.lda = L.d;
    g.B = (const bf16 *)ly->W_gate; g.B2 = (const bf16 *)ly->W_up; g.ldb = L.d;
    g.M = T_rows; g.N = 2 * ly->intermediate; g.K = L.d; g.k_splits = 1; g.k_segments = 1;
    g.tile_hint = (ctx->opt_gemm_tile >= 4 || ctx->opt_gemm_tile == 1) ? ctx->opt_gemm_tile : 0;
    if (ly->A_gu && w.any_adapter) {
      lowrank_t(w.hn, L.d, ly->A_gu, 2);
      set_lowrank(g, ly->B_gate, ly->B_up, 2, ly->intermediate);
    }
    g.C = (bf16 *)w.gate; g.ldc = ly->intermediate;
    launch_gemm_mfma(g, GEMM_EPI_SWIGLU, s);
  } else if (w.f0 != nullptr) {
    // bf16 on the plain kernels: gate and up stay in fp32 until silu(gate) * up is rounded, once
    const bool lr = ly->A_gu != nullptr && w.any_adapter;
    {
      ProfScope p(ctx, K_GATEUP, s);
      launch_gemm_plain_f32<T>((const T *)w.hn, (const T *)ly->W_gate, w.f0, T_rows, ly->intermediate, L.d, s);
      launch_gemm_plain_f32<T>((const T *)w.hn, (const T *)ly->W_up, w.f1, T_rows, ly->intermediate, L.d, s);
      if (lr) {
        launch_lowrank_add_plain<T, float>((const T *)w.hn, L.d, (const T *)ly->A_gu, 2, 0, (const T *)ly->B_gate,
                                           ly->intermediate, r, w.rm.adapter, w.scale_dev, w.f0, T_rows, s);
        launch_lowrank_add_plain<T, float>((const T *)w.hn, L.d, (const T *)ly->A_gu, 2, 1, (const T *)ly->B_up,
                                           ly->intermediate, r, w.rm.adapter, w.scale_dev, w.f1, T_rows, s);
      }
    }
    {
      ProfScope p(ctx, K_SILU, s);
      launch_silu_mul_f32<T>(w.f0, w.f1, (T *)w.gate, (int64_t)T_rows * ly->intermediate, s);
    }
  } else {
    {
      ProfScope p(ctx, K_GATEUP, s);
      dense(w.hn, ly->W_gate, nullptr, w.gate, ly->intermediate, L.d, ly->A_gu, ly->B_gate, 2, 0);
      dense(w.hn, ly->W_up, nullptr, w.up, ly->intermediate, L.d, ly->A_gu, ly->B_up, 2, 1);
    }
    {
      ProfScope p(ctx, K_SILU, s);
      launch_silu_mul<T>((const T *)w.gate, (const T *)w.up, (T *)w.gate, (int64_t)T_rows * ly->intermediate, s);
    }
  }
  {
    ProfScope p(ctx, K_DOWN, s);
    dense(w.gate, ly->W_down, w.h1, out, L.d, ly->intermediate, ly->A_down, ly->B_down);
  }
}

// Work list of the MFMA decode kernel: per (row, group of up to eight kv heads) n_own items over the row's own
// cache rows, and -- when sequences name shared prefixes -- per (group of up to 16 / G rows with the same prefix,
// group of kv heads) n_shared items over that prefix.  Every (row, head) ends up with n_own + n_shared partial
// records.  A workgroup's eight waves are hw kv heads x kr sub-ranges of the item's keys.
struct DecodePlan {
  std::vector<DecItem> items;      // empty when the list is built on the device (the static entry point)
  int n_own = 1, n_shared = 0;
  int n_device_items = 0;          // size of the device-built list: rows x head groups x n_own
  int hw = 1, kr = 1, groups = 1, cols_max = 1;
};
DecodePlan plan_decode_items(const alora_ctx *ctx, const Plan &pl, const LayerDims &L, int B, int n_steps, bool on_device) {
  DecodePlan dp;
  const int G = L.n_q_heads / L.n_kv_heads;
  const int pack = std::max(1, 16 / G);
  decode_mfma_shape(L.n_kv_heads, &dp.hw, &dp.kr);
  dp.groups = (L.n_kv_heads + dp.hw - 1) / dp.hw;
  dp.cols_max = G;
  int max_own = 1, max_pfx = 0;
  for (int b = 0; b < B; ++b) {
    max_own = std::max(max_own, pl.seqs[b].P + n_steps - pl.seqs[b].prefix_len);
    max_pfx = std::max(max_pfx, pl.seqs[b].prefix_len);
  }
  // 16 waves per compute unit (two rounds of workgroups), each over a key range of at least 1024 keys (every range
  // of a head costs a partial record unless it shares its workgroup): `items` (row, kv head) pairs need so many
  // ranges each, kr of which share a workgroup (and a partial record).  A handful of sequences over long caches
  // cannot fill the chip with ranges that long: down to 256 keys then, up to 128 records per head.
  auto splits_for = [&](int64_t items, int longest) {
    if (ctx->opt_splits > 0) return ctx->opt_splits;
    const bool few = 2 * items < ctx->n_cu;
    const int64_t ranges = std::max<int64_t>(1, std::min<int64_t>((16 * (int64_t)ctx->n_cu + items - 1) / std::max<int64_t>(items, 1),
                                                                  std::max(1, longest / (few ? 256 : 1024))));
    return (int)std::max<int64_t>(1, std::min<int64_t>(few ? 128 : 64, (ranges + dp.kr - 1) / dp.kr));
  };
  dp.n_own = splits_for((int64_t)pl.T * L.n_kv_heads, max_own);
  std::vector<std::vector<int>> chunks;      // rows that share one prefix, at most `pack` each
  if (pl.any_prefix) {
    std::vector<int> order(B);
    for (int b = 0; b < B; ++b) order[b] = b;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
      if (pl.seqs[x].prefix_off != pl.seqs[y].prefix_off) return pl.seqs[x].prefix_off < pl.seqs[y].prefix_off;
      return pl.seqs[x].prefix_len < pl.seqs[y].prefix_len;
    });
    for (int i = 0; i < B; ++i) {
      const SeqMeta &m = pl.seqs[order[i]];
      if (m.n_new <= 0 || m.prefix_len <= 0) continue;     // nothing to read: its records are zero-filled below
      const bool same = !chunks.empty() && (int)chunks.back().size() < pack &&
                        pl.seqs[order[i - 1]].prefix_off == m.prefix_off && pl.seqs[order[i - 1]].prefix_len == m.prefix_len &&
                        pl.seqs[order[i - 1]].prefix_len > 0 && pl.seqs[order[i - 1]].n_new > 0;
      if (!same) chunks.emplace_back();
      chunks.back().push_back(m.row_start);
    }
    // rows without a prefix still need their shared-part records: empty items (no keys) write them
    for (int b = 0; b < B; ++b) {
      const SeqMeta &m = pl.seqs[b];
      if (m.n_new <= 0 || m.prefix_len > 0) continue;
      if (chunks.empty() || (int)chunks.back().size() >= pack ||
          pl.seqs[a_seq_of_row(pl, chunks.back()[0])].prefix_len > 0) chunks.emplace_back();
      chunks.back().push_back(m.row_start);
    }
    dp.n_shared = splits_for((int64_t)chunks.size() * L.n_kv_heads, max_pfx);
  }
  dp.n_device_items = pl.T * dp.groups * dp.n_own;
  for (const auto &rows : chunks) dp.cols_max = std::max(dp.cols_max, (int)rows.size() * G);
  if (on_device) return dp;
  for (const auto &rows : chunks)
    for (int gb = 0; gb < dp.groups; ++gb)
      for (int sp = 0; sp < dp.n_shared; ++sp) {
        DecItem it{};
        it.n_rows = (int)rows.size(); it.g = gb * dp.hw; it.split = sp; it.n_splits = dp.n_shared; it.part = dp.n_own + sp; it.shared = 1;
        for (size_t i = 0; i < rows.size(); ++i) it.rows[i] = rows[i];
        dp.items.push_back(it);
      }
  for (int row = 0; row < pl.T; ++row)
    for (int gb = 0; gb < dp.groups; ++gb)
      for (int sp = 0; sp < dp.n_own; ++sp) {
        DecItem it{};
        it.n_rows = 1; it.g = gb * dp.hw; it.split = sp; it.n_splits = dp.n_own; it.part = sp; it.shared = 0;
        it.rows[0] = row;
        dp.items.push_back(it);
      }
  return dp;
}

// Work list of the MFMA prefill attention kernel, part 1: how the keys of a (row, head) are cut up.  Sequences that
// name no shared prefix cut their visible keys into n_own ranges.  Sequences that do cut their own keys (positions
// from prefix_len on) into n_own ranges, and the prefix into n_sh ranges that are walked once for ALL rows of a run
// of consecutive sequences naming that same prefix (Section 2, "Cache reuse patterns": several adapters invoked on
// one context): the rows of such a run are neighbours in the packed batch, so up to 256 / G of them share a
// workgroup and the prefix keys and values are fetched once per run instead of once per sequence.
struct PrefixRun { int64_t prefix_off; int prefix_len, row0, n_rows; };
struct PrefillPlan {
  std::vector<PrefixRun> runs;
  int n_own = 1, n_sh = 0;
};
PrefillPlan plan_prefill_ranges(const alora_ctx *ctx, const Plan &pl, const LayerDims &L, int B, int attn_waves) {
  PrefillPlan pp;
  const int tq = attn_prefill_mfma_tokens_per_tile(L, attn_waves);
  int64_t tiles = 0;
  int max_own = 1, max_pfx = 0;
  for (int b = 0; b < B; ++b) {
    const SeqMeta &m = pl.seqs[b];
    if (m.n_new <= 0) continue;
    tiles += (m.n_new + tq - 1) / tq;
    max_own = std::max(max_own, m.P + m.n_new - m.prefix_len);
    max_pfx = std::max(max_pfx, m.prefix_len);
    if (m.prefix_len <= 0) continue;
    if (!pp.runs.empty() && pp.runs.back().prefix_off == m.prefix_off && pp.runs.back().prefix_len == m.prefix_len &&
        pp.runs.back().row0 + pp.runs.back().n_rows == m.row_start)
      pp.runs.back().n_rows += m.n_new;
    else
      pp.runs.push_back(PrefixRun{m.prefix_off, m.prefix_len, m.row_start, m.n_new});
  }
  if (pp.runs.empty()) {
    // aim at one full wave of workgroups over the chip, with at least 256 keys per range
    tiles *= L.n_kv_heads;
    const int want = (int)std::min<int64_t>(16, std::max<int64_t>(1, ctx->n_cu / std::max<int64_t>(tiles, 1)));
    pp.n_own = ctx->opt_splits > 0 ? ctx->opt_splits : std::max(1, std::min(want, pl.max_len / 256));
    return pp;
  }
  // The work is uneven (long contexts walked by few packed tiles, short own parts walked by many): size the
  // ranges by work.  One unit = one 64-key tile of one workgroup; aim at two workgroups per compute unit of
  // equal length, at least four tiles each.
  int64_t units = 0;
  for (int b = 0; b < B; ++b) {
    const SeqMeta &m = pl.seqs[b];
    for (int q0 = 0; q0 < m.n_new; q0 += tq) units += (m.P + std::min(m.n_new, q0 + tq) - m.prefix_len + 63) / 64;
  }
  for (const PrefixRun &r : pp.runs) units += (int64_t)((r.n_rows + tq - 1) / tq) * ((r.prefix_len + 63) / 64);
  units *= L.n_kv_heads;
  const int64_t target = std::max<int64_t>(4, units / (2 * (int64_t)ctx->n_cu));
  auto ranges = [&](int longest) {
    if (ctx->opt_splits > 0) return ctx->opt_splits;
    return (int)std::max<int64_t>(1, std::min<int64_t>(16, ((longest + 63) / 64 + target - 1) / target));
  };
  pp.n_own = ranges(max_own);
  pp.n_sh = ranges(max_pfx);
  return pp;
}

// Part 2: the items, one per workgroup, in launch order.  Workgroups are dealt round-robin to the 8 XCDs, each with
// its own L2, and an XCD starts them in list order as compute units become free.  All q-tiles of one (sequence or
// prefix run, kv head, key range) read the same keys and values, so such a group goes to one XCD: groups are
// handed out heaviest first to the XCD with the least work so far, and inside an XCD the items run longest first
// (which keeps the q-tiles of a group next to each other: their lengths differ least).
std::vector<AttnItem> build_prefill_items(const Plan &pl, const LayerDims &L, int B, int attn_waves, const PrefillPlan &pp) {
  const int tq = attn_prefill_mfma_tokens_per_tile(L, attn_waves);
  const int n_own = pp.n_own, n_sh = pp.n_sh;
  struct Group { int64_t cost; std::vector<AttnItem> items; };      // the items of a group stream the same keys
  std::vector<Group> groups;
  // range `sp` of `parts` over the key positions [lo, hi), in whole tiles of 64 keys
  auto cut = [](int lo, int hi, int parts, int sp, AttnItem *it) {
    int chunk = (std::max(hi - lo, 0) + parts - 1) / parts;
    chunk = (chunk + 63) & ~63;
    it->kbeg = (int)std::min<int64_t>(hi, lo + (int64_t)sp * chunk);
    it->kend = (int)std::min<int64_t>(hi, (int64_t)it->kbeg + chunk);
  };
  auto key_tiles = [](const AttnItem &it) { return (int64_t)(it.kend - it.kbeg + 63) / 64 + 1; };
  for (int b = 0; b < B; ++b) {
    const SeqMeta &m = pl.seqs[b];
    if (m.n_new <= 0) continue;
    // (a sequence without prefix still writes n_own + n_sh records per (row, head): all of them over its own keys)
    const int parts = m.prefix_len > 0 ? n_own : n_own + n_sh;
    const int last = ((m.n_new - 1) / tq) * tq;
    for (int g = 0; g < L.n_kv_heads; ++g)
      for (int sp = 0; sp < parts; ++sp) {
        Group gr{0, {}};
        for (int q0 = last; q0 >= 0; q0 -= tq) {
          AttnItem it{};
          it.ntok = std::min(tq, m.n_new - q0);
          it.row0 = m.row_start + q0;
          // key positions count from the sequence's first own row (position prefix_len)
          it.pos0 = m.P + q0 - m.prefix_len;
          it.key_row0 = m.pool_off + m.prefix_len;
          it.n_addr = it.pos0 + it.ntok;                  // keys visible to the item's last token
          cut(0, it.n_addr, parts, sp, &it);
          it.g = g;
          it.part = sp;
          gr.cost += key_tiles(it);
          gr.items.push_back(it);
        }
        groups.push_back(std::move(gr));
      }
  }
  for (const PrefixRun &r : pp.runs)
    for (int g = 0; g < L.n_kv_heads; ++g)
      for (int sp = 0; sp < n_sh; ++sp) {
        Group gr{0, {}};
        for (int r0 = 0; r0 < r.n_rows; r0 += tq) {
          AttnItem it{};
          it.ntok = std::min(tq, r.n_rows - r0);
          it.row0 = r.row0 + r0;
          it.pos0 = 1 << 30;                              // every prefix key is visible to every row of the run
          it.key_row0 = r.prefix_off;
          it.n_addr = r.prefix_len;
          cut(0, r.prefix_len, n_sh, sp, &it);
          it.g = g;
          it.part = n_own + sp;
          gr.cost += key_tiles(it);
          gr.items.push_back(it);
        }
        groups.push_back(std::move(gr));
      }
  std::stable_sort(groups.begin(), groups.end(), [](const Group &x, const Group &y) { return x.cost > y.cost; });
  std::vector<AttnItem> per_xcd[8];
  int64_t load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (const Group &gr : groups) {
    int x = 0;
    for (int i = 1; i < 8; ++i)
      if (load[i] < load[x]) x = i;
    load[x] += gr.cost;
    per_xcd[x].insert(per_xcd[x].end(), gr.items.begin(), gr.items.end());
  }
  size_t longest = 0;
  for (int x = 0; x < 8; ++x) {
    std::stable_sort(per_xcd[x].begin(), per_xcd[x].end(),
                     [&](const AttnItem &p, const AttnItem &q) { return key_tiles(p) > key_tiles(q); });
    longest = std::max(longest, per_xcd[x].size());
  }
  std::vector<AttnItem> qtiles;
  qtiles.reserve(longest * 8);
  for (size_t i = 0; i < longest; ++i)
    for (int x = 0; x < 8; ++x)
      qtiles.push_back(i < per_xcd[x].size() ? per_xcd[x][i] : AttnItem{});        // ntok = 0: padding
  return qtiles;
}


alora_status run(alora_ctx *ctx, const alora_layer_desc *layers, int n_layers, alora_kv_cache *caches,
                 const void *x, const int32_t *cu, const int32_t *kps, const int32_t *aps, int B, void *out,
                 void *stream, bool stack, bool decode = false, int n_steps = 1, bool use_static = false) {
  if (!ctx) return ALORA_EINVAL;
  ctx->err.clear();
  if (n_layers < 1) return fail(ctx, ALORA_EINVAL, "n_layers = %d must be at least 1", n_layers);
  if (!layers || !caches) return fail(ctx, ALORA_EINVAL, "layers / caches is NULL");
  LayerDims L{};
  alora_status st = check_layer(ctx, &layers[0], stack, &L);
  if (st != ALORA_OK) return st;
  for (int l = 1; l < n_layers; ++l) {
    LayerDims Ll{};
    st = check_layer(ctx, &layers[l], stack, &Ll);
    if (st != ALORA_OK) return st;
    if (memcmp(&Ll, &L, sizeof L) != 0 || layers[l].dtype != layers[0].dtype ||
        layers[l].intermediate != layers[0].intermediate)
      return fail(ctx, ALORA_ESHAPE, "layer %d differs in shape or dtype from layer 0", l);
    if (layers[l].rope_theta != layers[0].rope_theta || layers[l].rms_eps != layers[0].rms_eps)
      return fail(ctx, ALORA_ESHAPE, "layer %d differs in rope_theta or rms_eps from layer 0 (one rotary table per call)", l);
    if (!caches[l].k || !caches[l].v) return fail(ctx, ALORA_EINVAL, "caches[%d] k / v is NULL", l);
    if (caches[l].pool_tokens != caches[0].pool_tokens)
      return fail(ctx, ALORA_ECAPACITY, "caches[%d] pool size differs from caches[0]", l);
  }
  Plan pl;
  pl.L = L;
  if (n_steps < 1) return fail(ctx, ALORA_EINVAL, "n_steps = %d must be at least 1", n_steps);
  st = check_batch(ctx, &layers[0], &caches[0], cu, kps, aps, B, n_steps, &pl);
  if (st != ALORA_OK) return st;
  if (pl.T > 0 && (!x || !out)) return fail(ctx, ALORA_EINVAL, "x / out is NULL");
  if (pl.T == 0) return ALORA_OK;
  if (use_static && pl.any_prefix)
    return fail(ctx, ALORA_EINVAL, "alora_decode_static does not take shared prefixes (prefix_len must be NULL or all zero)");
  const size_t esz0 = layers[0].dtype == ALORA_BF16 ? 2 : 4;
  if (ctx->device < 0) {
    // a validation-only context still answers the size question of the static entry point
    if (use_static) {
      const int ns = std::max(1, std::min(128, pl.max_len / 256));      // upper bound on the key splits
      const size_t need = layout_workspace(nullptr, L, pl.T, esz0, ns, 8, 0, false).bytes + (size_t)B * sizeof(SeqMeta) +
                          (size_t)pl.T * L.n_kv_heads * ns * sizeof(DecItem) + (size_t)pl.T * (L.head_dim / 2) * sizeof(float2) + 1024;
      if (need > SCRATCH_BYTES)
        return fail(ctx, ALORA_ECAPACITY, "alora_decode_static: this call needs up to %zu bytes of scratch, the static buffer holds %zu",
                    need, SCRATCH_BYTES);
    }
    return fail(ctx, ALORA_EHIP, "arguments are valid, but this is a validation-only context (device -1)");
  }

  HIP_TRY(ctx, hipSetDevice(ctx->device));
  hipStream_t s = (hipStream_t)stream;
  const size_t esz = layers[0].dtype == ALORA_BF16 ? 2 : 4;
  const bool attn_mfma = layers[0].dtype == ALORA_BF16 && ctx->opt_kernels == 0 && !decode &&
                         attn_prefill_mfma_supported(L);
  const int attn_waves = ctx->opt_attn_waves == 4 ? 4 : 8;
  int n_splits = pick_splits(ctx, pl.T, L.n_kv_heads, pl.max_len);
  const bool decode_mfma = layers[0].dtype == ALORA_BF16 && ctx->opt_kernels == 0 && decode &&
                           attn_decode_mfma_supported(L);
  // work lists of the MFMA attention kernels (the number of partial records per (row, head) comes out of them)
  DecodePlan dp;
  PrefillPlan pp;
  if (decode_mfma) {
    dp = plan_decode_items(ctx, pl, L, B, n_steps, use_static);
    n_splits = dp.n_own + dp.n_shared;
  }
  if (attn_mfma) {
    pp = plan_prefill_ranges(ctx, pl, L, B, attn_waves);
    n_splits = pp.n_own + pp.n_sh;
  }
  const std::vector<DecItem> &ditems = dp.items;
  const int n_static_items = dp.n_device_items, n_static_n_own = dp.n_own;
  const int dec_hw = dp.hw, dec_kr = dp.kr, dec_groups = dp.groups, dec_cols_max = dp.cols_max;
  // kernel family: MFMA for bf16 shapes it covers, plain otherwise
  const bool mfma = layers[0].dtype == ALORA_BF16 && ctx->opt_kernels == 0 && L.d % 64 == 0 &&
                    (L.n_adapters == 0 || (L.rank % 16 == 0 && L.n_adapters <= 64)) && L.n_q % 32 == 0 &&
                    L.n_kv % 32 == 0 && (!stack || (layers[0].intermediate % 64 == 0 && L.n_q % 64 == 0));
  // The reduction axis of the QKV projection is cut into segments fixed by the weight shape (or by the
  // gemm_splits option); whether they run in workgroups of their own or one after the other inside one
  // is a scheduling choice that does not change a single bit of the result.
  int k_segments = mfma ? gemm_mfma_fixed_segments(L.n_qkv, L.d, ctx->n_cu) : 1;
  if (mfma && ctx->opt_gemm_splits > 0) k_segments = L.d % (64 * ctx->opt_gemm_splits) == 0 ? ctx->opt_gemm_splits : 1;
  const int k_splits = (k_segments > 1 && gemm_mfma_split_segments(pl.T, L.n_qkv, ctx->n_cu)) ? k_segments : 1;
  const bool f32_tail = stack && !mfma && layers[0].dtype == ALORA_BF16;
  Workspace probe = layout_workspace(nullptr, L, pl.T, esz, n_splits, k_splits, layers[0].intermediate, stack, f32_tail);
  if (use_static) {
    // Everything the call needs beyond its inputs and outputs lives in the static scratch array of this GPU:
    //   [ workspace | per-sequence records | decode work list | rotary lines, one per row ]
    // No allocation, no staging copy: the records travel as kernel arguments, the work list and the rotary lines
    // are computed on the device.  Nothing in there has to start at zero (every byte a kernel reads was written
    // by a kernel of this call), so nothing is cleared.
    const size_t ws_bytes = (probe.bytes + 255) & ~(size_t)255;
    const size_t seq_b = ((size_t)B * sizeof(SeqMeta) + 255) & ~(size_t)255;
    const size_t item_b = ((size_t)n_static_items * sizeof(DecItem) + 255) & ~(size_t)255;
    const size_t rope_b = (size_t)pl.T * (L.head_dim / 2) * sizeof(float2);
    const size_t need = ws_bytes + seq_b + item_b + rope_b;
    if (need > SCRATCH_BYTES)
      return fail(ctx, ALORA_ECAPACITY, "alora_decode_static: this call needs %zu bytes of scratch, the static buffer holds %zu",
                  need, SCRATCH_BYTES);
    if (!ctx->scratch_dev) return fail(ctx, ALORA_EHIP, "the static scratch array has no device address on this context");
    char *base = (char *)ctx->scratch_dev;
    SeqMeta *seqs_dev = (SeqMeta *)(base + ws_bytes);
    DecItem *items_dev = (DecItem *)(base + ws_bytes + seq_b);
    for (int b0 = 0; b0 < B; b0 += STAGE_SEQS) {
      SeqChunk c;
      const int n = std::min(STAGE_SEQS, B - b0);
      memcpy(c.m, pl.seqs.data() + b0, (size_t)n * sizeof(SeqMeta));
      hipLaunchKernelGGL(stage_seqs_kernel, dim3(1), dim3(64), 0, s, c, n, seqs_dev + b0);
    }
    if (decode_mfma && n_static_items > 0)
      hipLaunchKernelGGL(make_decode_items_kernel, dim3((n_static_items + 255) / 256), dim3(256), 0, s, items_dev,
                         n_static_items, dec_groups, dec_hw, n_static_n_own);
    Workspace w = layout_workspace(base, L, pl.T, esz, n_splits, k_splits, 0, false);
    w.mfma = mfma;
    w.k_splits = k_splits;
    w.k_segments = k_segments;
    w.lora_split = (k_splits > 1 && ctx->opt_lora_split != 2) || ctx->opt_lora_split == 1 ? 1 : 0;
    w.attn_mfma = false;
    w.decode_mfma = decode_mfma;
    w.attn_waves = attn_waves;
    w.ditems = items_dev;
    w.n_ditems = decode_mfma ? n_static_items : 0;
    w.dec_hw = dec_hw; w.dec_kr = dec_kr; w.dec_cols_max = dec_cols_max;
    w.any_adapter = pl.any_adapter;
    w.rope_by_row = true;
    w.rope_rows = (float2 *)(base + ws_bytes + seq_b + item_b);
    w.rope = w.rope_rows;
    const int saved_profile = ctx->opt_profile;
    ctx->opt_profile = 0;             // the event brackets of the profiling option create events: not here
    if (layers[0].dtype == ALORA_BF16)
      attention_block<bf16>(ctx, &layers[0], L, &caches[0], (const bf16 *)x, pl, seqs_dev, w, true, n_splits, true, 0, (bf16 *)out, s);
    else
      attention_block<float>(ctx, &layers[0], L, &caches[0], (const float *)x, pl, seqs_dev, w, true, n_splits, true, 0, (float *)out, s);
    ctx->opt_profile = saved_profile;
    HIP_TRY(ctx, hipGetLastError());
    for (int b = 0; b < B; ++b) caches[0].seq_len[b] += 1;
    return ALORA_OK;
  }
  st = ensure_workspace(ctx, probe.bytes);
  if (st != ALORA_OK) return st;
  st = ensure_rope(ctx, pl.max_len, L.head_dim / 2, layers[0].rope_theta, s);
  if (st != ALORA_OK) return st;
  // staged metadata: per-sequence records, then the work list of the MFMA attention kernel
  std::vector<AttnItem> qtiles;
  if (attn_mfma) qtiles = build_prefill_items(pl, L, B, attn_waves, pp);
  const size_t seq_bytes = ((size_t)B * sizeof(SeqMeta) + 15) & ~(size_t)15;
  const size_t work_bytes = (qtiles.size() * sizeof(AttnItem) + ditems.size() * sizeof(DecItem) + 15) & ~(size_t)15;   // one of the two lists
  const size_t scale_bytes = stack ? (((size_t)L.n_adapters * sizeof(float) + 15) & ~(size_t)15) : 0;
  const size_t meta_bytes = seq_bytes + work_bytes + scale_bytes;
  MetaSlot *slot = nullptr;
  st = acquire_slot(ctx, meta_bytes, &slot);
  if (st != ALORA_OK) return st;
  memcpy(slot->host, pl.seqs.data(), (size_t)B * sizeof(SeqMeta));
  if (!qtiles.empty()) memcpy(slot->host + seq_bytes, qtiles.data(), qtiles.size() * sizeof(AttnItem));
  if (!ditems.empty()) memcpy(slot->host + seq_bytes, ditems.data(), ditems.size() * sizeof(DecItem));
  if (scale_bytes) memcpy(slot->host + seq_bytes + work_bytes, layers[0].scale, (size_t)L.n_adapters * sizeof(float));
  if (ctx->opt_stage_copy) {
    HIP_TRY(ctx, hipMemcpyAsync(slot->dev, slot->host, meta_bytes, hipMemcpyHostToDevice, s));
  } else {
    const int n16 = (int)((meta_bytes + 15) / 16);
    hipLaunchKernelGGL(stage_meta_kernel, dim3((n16 + 255) / 256), dim3(256), 0, s, (const uint4 *)slot->host,
                       (uint4 *)slot->dev, n16);
  }
  const SeqMeta *seqs_dev = (const SeqMeta *)slot->dev;
  Workspace w = layout_workspace(ctx->ws, L, pl.T, esz, n_splits, k_splits, layers[0].intermediate, stack, f32_tail);
  w.mfma = mfma;
  w.k_splits = k_splits;
  w.k_segments = k_segments;
  // few row tiles and a split reduction: the workgroups are short and the prologue of split 0 would stick out
  w.lora_split = (k_splits > 1 && ctx->opt_lora_split != 2) || ctx->opt_lora_split == 1 ? 1 : 0;
  w.attn_mfma = attn_mfma;
  w.decode_mfma = decode_mfma;
  w.attn_waves = attn_waves;
  w.qtiles = (const AttnItem *)(slot->dev + seq_bytes);
  w.n_qtiles = (int)qtiles.size();
  w.ditems = (const DecItem *)(slot->dev + seq_bytes);
  w.n_ditems = (int)ditems.size();
  w.dec_hw = dec_hw; w.dec_kr = dec_kr; w.dec_cols_max = dec_cols_max;
  w.scale_dev = scale_bytes ? (const float *)(slot->dev + seq_bytes + work_bytes) : nullptr;
  w.any_adapter = pl.any_adapter;
  w.rope = ctx->rope;

  const bool bf = layers[0].dtype == ALORA_BF16;
  if (!stack) {
    // n_steps > 1: a run of decode steps on the metadata staged once; step t sits t positions further on
    for (int t = 0; t < n_steps; ++t) {
      const char *xt = (const char *)x + (size_t)t * pl.T * L.d * esz;
      char *ot = (char *)out + (size_t)t * pl.T * L.n_q * esz;
      if (bf) attention_block<bf16>(ctx, &layers[0], L, &caches[0], (const bf16 *)xt, pl, seqs_dev, w, true, n_splits, decode, t, (bf16 *)ot, s);
      else attention_block<float>(ctx, &layers[0], L, &caches[0], (const float *)xt, pl, seqs_dev, w, true, n_splits, decode, t, (float *)ot, s);
    }
  } else {
    const void *cur = x;
    for (int l = 0; l < n_layers; ++l) {
      void *nxt = (l == n_layers - 1) ? out : ((l & 1) ? w.xb : w.xa);
      if (bf) {
        attention_block<bf16>(ctx, &layers[l], L, &caches[l], (const bf16 *)cur, pl, seqs_dev, w, l == 0, n_splits, decode, 0, (bf16 *)w.attn, s);
        layer_tail<bf16>(ctx, &layers[l], L, (const bf16 *)cur, w, pl.T, (bf16 *)nxt, s);
      } else {
        attention_block<float>(ctx, &layers[l], L, &caches[l], (const float *)cur, pl, seqs_dev, w, l == 0, n_splits, decode, 0, (float *)w.attn, s);
        layer_tail<float>(ctx, &layers[l], L, (const float *)cur, w, pl.T, (float *)nxt, s);
      }
      cur = nxt;
    }
  }
  HIP_TRY(ctx, hipGetLastError());
  HIP_TRY(ctx, hipEventRecord(slot->ev, s));
  slot->in_flight = true;
  for (int b = 0; b < B; ++b) caches[0].seq_len[b] += (cu[b + 1] - cu[b]) * n_steps;
  return ALORA_OK;
}

}  // namespace

alora_status drain_profile(alora_ctx *ctx) {
  for (ProfEvent &e : ctx->prof_pending) {
    HIP_TRY(ctx, hipEventSynchronize(e.stop));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, e.start, e.stop));
    ctx->prof_ms[e.kernel] += ms;
    ctx->prof_n[e.kernel] += 1;
    ctx->prof_free.push_back(e.start);
    ctx->prof_free.push_back(e.stop);
  }
  ctx->prof_pending.clear();
  return ALORA_OK;
}

extern "C" {

alora_status alora_create(alora_ctx **out, int device) {
  if (!out) return ALORA_EINVAL;
  *out = nullptr;
  if (device == -1) {              // validation-only context: checks arguments, never launches
    alora_ctx *ctx = new alora_ctx();
    ctx->device = -1;
    *out = ctx;
    return ALORA_OK;
  }
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return ALORA_EHIP;
  if (hipSetDevice(device) != hipSuccess) return ALORA_EHIP;
  alora_ctx *ctx = new alora_ctx();
  ctx->device = device;
  // the device address of this GPU's copy of the static scratch array (the array's name is not one)
  void *sp = nullptr;
  if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || sp == nullptr) {
    delete ctx;
    return ALORA_EHIP;
  }
  ctx->scratch_dev = (unsigned char *)sp;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) == hipSuccess) ctx->n_cu = prop.multiProcessorCount;
  *out = ctx;
  return ALORA_OK;
}

void alora_destroy(alora_ctx *ctx) {
  if (!ctx) return;
  if (ctx->device < 0) { delete ctx; return; }
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  if (ctx->ws) (void)hipFree(ctx->ws);
  if (ctx->rope) (void)hipFree(ctx->rope);
  (void)drain_profile(ctx);
  for (hipEvent_t e : ctx->prof_free) (void)hipEventDestroy(e);
  for (MetaSlot &sl : ctx->slots) {
    if (sl.host) (void)hipHostFree(sl.host);
    if (sl.dev) (void)hipFree(sl.dev);
    if (sl.ev) (void)hipEventDestroy(sl.ev);
  }
  delete ctx;
}

const char *alora_last_error(const alora_ctx *ctx) { return ctx ? ctx->err.c_str() : "context is NULL"; }

const char *alora_status_string(alora_status s) {
  switch (s) {
    case ALORA_OK: return "ALORA_OK";
    case ALORA_EINVAL: return "ALORA_EINVAL";
    case ALORA_ESHAPE: return "ALORA_ESHAPE";
    case ALORA_ECAPACITY: return "ALORA_ECAPACITY";
    case ALORA_EADAPTER: return "ALORA_EADAPTER";
    case ALORA_EDTYPE: return "ALORA_EDTYPE";
    case ALORA_EHIP: return "ALORA_EHIP";
  }
  return "unknown status";
}

alora_status alora_set_option(alora_ctx *ctx, const char *key, int value) {
  if (!ctx) return ALORA_EINVAL;
  ctx->err.clear();
  if (!key) return fail(ctx, ALORA_EINVAL, "option key is NULL");
  if (!strcmp(key, "kernels")) {
    if (value != 0 && value != 1) return fail(ctx, ALORA_EINVAL, "kernels must be 0 or 1");
    ctx->opt_kernels = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "kv_splits")) {
    if (value < 0 || value > 256) return fail(ctx, ALORA_EINVAL, "kv_splits must be in [0, 256]");
    ctx->opt_splits = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "gemm_splits")) {
    if (value < 0 || value > 64) return fail(ctx, ALORA_EINVAL, "gemm_splits must be in [0, 64]");
    ctx->opt_gemm_splits = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "lora_split")) {
    if (value < 0 || value > 2) return fail(ctx, ALORA_EINVAL, "lora_split must be 0, 1 or 2");
    ctx->opt_lora_split = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "stage_copy")) {
    if (value < 0 || value > 1) return fail(ctx, ALORA_EINVAL, "stage_copy must be 0 or 1");
    ctx->opt_stage_copy = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "attn_lazy")) {
    if (value < 0 || value > 16) return fail(ctx, ALORA_EINVAL, "attn_lazy must be in [0, 16]");
    ctx->opt_attn_lazy = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "attn_partials16")) {
    if (value != 0 && value != 1) return fail(ctx, ALORA_EINVAL, "attn_partials16 must be 0 or 1");
    ctx->opt_attn_partials16 = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "rope_fuse")) {
    if (value != 0 && value != 1) return fail(ctx, ALORA_EINVAL, "rope_fuse must be 0 or 1");
    ctx->opt_rope_fuse = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "attn_fold")) {
    if (value != 0 && value != 1) return fail(ctx, ALORA_EINVAL, "attn_fold must be 0 or 1");
    ctx->opt_attn_fold = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "attn_waves")) {
    if (value != 0 && value != 4 && value != 8) return fail(ctx, ALORA_EINVAL, "attn_waves must be 0, 4 or 8");
    ctx->opt_attn_waves = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "prep_split")) {
    if (value < 0 || value > 2) return fail(ctx, ALORA_EINVAL, "prep_split must be 0, 1 or 2");
    ctx->opt_prep_split = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "gemm_tile")) {
    if (value < 0 || value > 6) return fail(ctx, ALORA_EINVAL, "gemm_tile must be in [0, 6]");
    ctx->opt_gemm_tile = value;
    return ALORA_OK;
  }
  if (!strcmp(key, "profile")) {
    if (value != 0 && value != 1) return fail(ctx, ALORA_EINVAL, "profile must be 0 or 1");
    ctx->opt_profile = value;
    return ALORA_OK;
  }
  return fail(ctx, ALORA_EINVAL, "unknown option '%s'", key);
}

alora_status alora_profile_read(alora_ctx *ctx, const char *kernel, double *total_ms, int64_t *launches) {
  if (!ctx) return ALORA_EINVAL;
  ctx->err.clear();
  if (!kernel || !total_ms || !launches) return fail(ctx, ALORA_EINVAL, "NULL argument");
  alora_status st = drain_profile(ctx);
  if (st != ALORA_OK) return st;
  for (int i = 0; i < K_COUNT; ++i)
    if (!strcmp(kernel, KERNEL_NAMES[i])) {
      *total_ms = ctx->prof_ms[i];
      *launches = ctx->prof_n[i];
      return ALORA_OK;
    }
  return fail(ctx, ALORA_EINVAL, "unknown kernel name '%s'", kernel);
}

alora_status alora_lm_head(alora_ctx *ctx, alora_dtype dtype, int32_t d, int32_t vocab, const void *x_last,
                           const void *final_gain, float rms_eps, const void *W_vocab, int32_t B, float *logits,
                           int32_t *token, void *stream) {
  if (!ctx) return ALORA_EINVAL;
  ctx->err.clear();
  if (dtype != ALORA_F32 && dtype != ALORA_BF16)
    return fail(ctx, ALORA_EDTYPE, "dtype %d is neither ALORA_F32 nor ALORA_BF16", (int)dtype);
  if (d < 1 || d > 16000) return fail(ctx, ALORA_ESHAPE, "d = %d outside [1, 16000]", d);
  if (vocab < 1) return fail(ctx, ALORA_ESHAPE, "vocab = %d must be positive", vocab);
  if (B < 1 || B > 4096) return fail(ctx, ALORA_EINVAL, "B = %d outside [1, 4096]", B);
  if (!x_last || !W_vocab) return fail(ctx, ALORA_EINVAL, "x_last / W_vocab is NULL");
  if (!logits && !token) return fail(ctx, ALORA_EINVAL, "logits and token are both NULL: nothing to compute");
  if (ctx->device < 0) return fail(ctx, ALORA_EHIP, "validation-only context (device -1)");
  HIP_TRY(ctx, hipSetDevice(ctx->device));
  hipStream_t s = (hipStream_t)stream;
  const bool bf = dtype == ALORA_BF16;
  const size_t esz = bf ? 2 : 4;
  const int n_slabs = argmax_slabs(vocab);
  // workspace: normalised rows | logits (unless the caller keeps them) | per-slab maxima
  Bump probe(nullptr);
  probe.take<char>((size_t)B * d * esz);
  if (!logits) probe.take<float>((size_t)B * vocab);
  probe.take<float>((size_t)B * n_slabs);
  probe.take<int>((size_t)B * n_slabs);
  alora_status st = ensure_workspace(ctx, probe.off);
  if (st != ALORA_OK) return st;
  Bump b(ctx->ws);
  char *xh = b.take<char>((size_t)B * d * esz);
  float *lg = logits ? logits : b.take<float>((size_t)B * vocab);
  float *pv = b.take<float>((size_t)B * n_slabs);
  int *pi = b.take<int>((size_t)B * n_slabs);
  const bool mfma = bf && ctx->opt_kernels == 0 && gemm_mfma_supported(B, vocab, d);
  RowMeta none{};
  const void *rows = x_last;
  if (final_gain) {
    ProfScope p(ctx, K_MLPNORM, s);
    if (mfma && prep_rows_mfma_supported(d, 0)) {
      PrepArgs pa{};
      pa.x = (const bf16 *)x_last; pa.gain = (const bf16 *)final_gain; pa.eps = rms_eps;
      pa.T = B; pa.d = d; pa.xh = (bf16 *)xh; pa.rm = none;
      launch_prep_rows_mfma(pa, s);
    } else if (bf) {
      launch_prep_rows<bf16>((const bf16 *)x_last, (const bf16 *)final_gain, rms_eps, B, d, nullptr, 0, 0, nullptr, 0,
                             false, (bf16 *)xh, nullptr, nullptr, none, s);
    } else {
      launch_prep_rows<float>((const float *)x_last, (const float *)final_gain, rms_eps, B, d, nullptr, 0, 0, nullptr,
                              0, false, (float *)xh, nullptr, nullptr, none, s);
    }
    rows = xh;
  }
  {
    ProfScope p(ctx, K_LMHEAD, s);
    if (mfma) {
      GemmArgs g{};
      g.A = (const bf16 *)rows; g.lda = d;
      g.B = (const bf16 *)W_vocab; g.ldb = d;
      g.M = B; g.N = vocab; g.K = d;
      g.k_splits = 1;
      g.k_segments = 1;
      g.Cpart = lg;
      launch_gemm_mfma(g, GEMM_EPI_PARTIAL, s);
    } else if (bf) {
      launch_lm_logits_plain<bf16>((const bf16 *)rows, (const bf16 *)W_vocab, B, vocab, d, lg, s);
    } else {
      launch_lm_logits_plain<float>((const float *)rows, (const float *)W_vocab, B, vocab, d, lg, s);
    }
  }
  if (token) {
    ProfScope p(ctx, K_ARGMAX, s);
    launch_argmax(lg, B, vocab, pv, pi, token, s);
  }
  HIP_TRY(ctx, hipGetLastError());
  return ALORA_OK;
}

alora_status alora_profile_reset(alora_ctx *ctx) {
  if (!ctx) return ALORA_EINVAL;
  ctx->err.clear();
  alora_status st = drain_profile(ctx);
  if (st != ALORA_OK) return st;
  for (int i = 0; i < K_COUNT; ++i) { ctx->prof_ms[i] = 0.0; ctx->prof_n[i] = 0; }
  return ALORA_OK;
}

alora_status alora_prefill(alora_ctx *ctx, const alora_layer_desc *layer, alora_kv_cache *cache,
                           const void *x_suffix, const int32_t *cu_seqlens, const int32_t *k_per_seq,
                           const int32_t *adapter_per_seq, int32_t B, void *attn_out, void *stream) {
  return run(ctx, layer, 1, cache, x_suffix, cu_seqlens, k_per_seq, adapter_per_seq, B, attn_out, stream, false);
}

alora_status alora_decode(alora_ctx *ctx, const alora_layer_desc *layer, alora_kv_cache *cache, const void *x_tok,
                          const int32_t *k_per_seq, const int32_t *adapter_per_seq, int32_t B, void *attn_out,
                          void *stream) {
  if (!ctx) return ALORA_EINVAL;
  if (B < 1) return fail(ctx, ALORA_EINVAL, "B = %d must be at least 1", B);
  std::vector<int32_t> cu(B + 1);
  for (int b = 0; b <= B; ++b) cu[b] = b;
  return run(ctx, layer, 1, cache, x_tok, cu.data(), k_per_seq, adapter_per_seq, B, attn_out, stream, false, true);
}

alora_status alora_decode_static(alora_ctx *ctx, const alora_layer_desc *layer, alora_kv_cache *cache, const void *x_tok,
                                 const int32_t *k_per_seq, const int32_t *adapter_per_seq, int32_t B, void *attn_out,
                                 void *stream) {
  if (!ctx) return ALORA_EINVAL;
  if (B < 1) return fail(ctx, ALORA_EINVAL, "B = %d must be at least 1", B);
  if (B > 4096) return fail(ctx, ALORA_ECAPACITY, "alora_decode_static takes at most 4096 sequences per call (B = %d)", B);
  int32_t cu[4097];
  for (int b = 0; b <= B; ++b) cu[b] = b;
  return run(ctx, layer, 1, cache, x_tok, cu, k_per_seq, adapter_per_seq, B, attn_out, stream, false, true, 1, true);
}

alora_status alora_decode_steps(alora_ctx *ctx, const alora_layer_desc *layer, alora_kv_cache *cache,
                                const void *x_steps, const int32_t *k_per_seq, const int32_t *adapter_per_seq,
                                int32_t B, int32_t n_steps, void *attn_out, void *stream) {
  if (!ctx) return ALORA_EINVAL;
  if (B < 1) return fail(ctx, ALORA_EINVAL, "B = %d must be at least 1", B);
  std::vector<int32_t> cu(B + 1);
  for (int b = 0; b <= B; ++b) cu[b] = b;
  return run(ctx, layer, 1, cache, x_steps, cu.data(), k_per_seq, adapter_per_seq, B, attn_out, stream, false, true,
             n_steps);
}

alora_status alora_stack_prefill(alora_ctx *ctx, const alora_layer_desc *layers, int32_t n_layers,
                                 alora_kv_cache *caches, const void *x, const int32_t *cu_seqlens,
                                 const int32_t *k_per_seq, const int32_t *adapter_per_seq, int32_t B, void *out,
                                 void *stream) {
  return run(ctx, layers, n_layers, caches, x, cu_seqlens, k_per_seq, adapter_per_seq, B, out, stream, true);
}

alora_status alora_stack_decode(alora_ctx *ctx, const alora_layer_desc *layers, int32_t n_layers, alora_kv_cache *caches,
                                const void *x_tok, const int32_t *k_per_seq, const int32_t *adapter_per_seq, int32_t B,
                                void *out, void *stream) {
  if (!ctx) return ALORA_EINVAL;
  if (B < 1) return fail(ctx, ALORA_EINVAL, "B = %d must be at least 1", B);
  std::vector<int32_t> cu(B + 1);
  for (int b = 0; b <= B; ++b) cu[b] = b;
  return run(ctx, layers, n_layers, caches, x_tok, cu.data(), k_per_seq, adapter_per_seq, B, out, stream, true, true);
}

}  // extern "C"
