// C-ABI of libsfi: argument checks, workspace carving, launch sequencing.  No arithmetic here.
#include <math.h>
#include <mutex>
#include <new>
#include <string.h>

#include "sfi_internal.h"

using namespace sfi;

struct sfi_ctx {
  sfi_config cfg;
  float scale;
  int G;
  Workspace ws;
  int n_cu;
  float alpha;              // power-mean exponent of the evidence, in (0, 1]
  const int32_t* table;     // paged cache: device block table, nullptr until sfi_set_block_table
  int table_stride, page_lg, page_rpb, n_blocks;
  int dense_target_wgs;     // workgroups the dense launch aims for; 0 = decided per launch
  int fast_tiles_per_wave;  // 32-row tiles each wave of the gather launch should get; 0 = decided per launch
  int tail_merge;           // split fast-step launches merge in the attention kernel (no merge launch)
  int dense_wide;           // dense kernel reads K rows as whole 128-byte lines (A/B knob, sfi_set_dense_k_layout)
  int mixed_plan;           // the ragged step's dense launch plans itself on the device (default; A/B knob, sfi_set_mixed_plan)
  int last_dense_splits, last_fast_splits;
  int selector_ran;         // a Selector pass has used the evidence now in the workspace: its histogram and state
                            // words are no longer the cleared ones the dense kernel left
  // profiling: a ring of event pairs, one set of stages per hot call, read back in one go so that
  // no host synchronisation sits between the profiled calls
  int profiling;
  int prof_calls;                     // hot calls recorded since profiling was switched on
  int prof_cap;                       // calls the ring holds
  hipEvent_t* ev;                     // [prof_cap][SFI_N_STAGES][2]
  unsigned char* ev_used;             // [prof_cap][SFI_N_STAGES]
};

namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int validate(const sfi_config* c) {
  if (c == nullptr) return SFI_EINVAL;
  if (c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->max_ctx < 1 || c->max_budget < 0 ||
      c->n_sink < 0 || c->recent < 0 || !(c->scale >= 0.f))
    return SFI_EINVAL;
  if (c->n_q_heads % c->n_kv_heads != 0) return SFI_EINVAL;
  if (c->head_dim != kHeadDim) return SFI_EUNSUPPORTED;
  if (c->n_q_heads / c->n_kv_heads > 16) return SFI_EUNSUPPORTED;
  if (c->selector_mode != 0 && c->selector_mode != 1) return SFI_EUNSUPPORTED;
  if (c->out_bf16 != 0 && c->out_bf16 != 1) return SFI_EINVAL;
  if (!(c->alpha >= 0.f) || c->alpha > 1.f) return SFI_EINVAL;
  if (c->page_size != 0) {
    if (c->page_size < 16 || c->page_size > 65536 || (c->page_size & (c->page_size - 1)) != 0) return SFI_EINVAL;
    if (c->k_stride_b != 0 || c->v_stride_b != 0) return SFI_EINVAL;
    if (c->k_stride_page < 0 || c->v_stride_page < 0 || (c->k_stride_page == 0) != (c->v_stride_page == 0)) return SFI_EINVAL;
    if (c->k_stride_page != 0) {  // whole row strides, enough for a block, the same count for K and V
      if (c->k_stride_t == 0 || c->v_stride_t == 0 || c->k_stride_page % c->k_stride_t != 0 ||
          c->v_stride_page % c->v_stride_t != 0 || c->k_stride_page / c->k_stride_t != c->v_stride_page / c->v_stride_t ||
          c->k_stride_page / c->k_stride_t < c->page_size || c->k_stride_page / c->k_stride_t > (1 << 24))
        return SFI_EINVAL;
    }
  }
  if (c->selector_mode == 1) {
    if (!(c->gamma >= 0.f) || !(c->beta >= 0.f) || !(c->p >= 1.f) || !(c->eta >= 0.f) || !(c->lambda_clip >= 0.f) ||
        !(c->lambda_clip <= 1.f) || !(c->alpha_soft >= 0.f) || !(c->alpha_cross >= 0.f) || !(c->temp > 0.f) ||
        !(c->eps >= 0.f) || c->nms_radius < 0)
      return SFI_EINVAL;
    if (c->nms_radius > kMaxNmsRadius) return SFI_EUNSUPPORTED;
    const float eps = c->eps > 0.f ? c->eps : 1e-8f;
    // the ranking key exp(z) must stay a normal fp32 number: z >= (1 + alpha_soft + alpha_cross) * log(eps)
    if (!(eps < 1.f) || (1.f + c->alpha_soft + c->alpha_cross) * -log2f(eps) >= 120.f) return SFI_EUNSUPPORTED;
  }
  if ((int64_t)c->max_ctx > (int64_t)1 << 30) return SFI_EUNSUPPORTED;
  const int64_t st[6] = {c->k_stride_b, c->k_stride_h, c->k_stride_t, c->v_stride_b, c->v_stride_h, c->v_stride_t};
  for (int i = 0; i < 6; ++i) {
    if (st[i] < 0) return SFI_EINVAL;
    if (st[i] % 8 != 0) return SFI_EALIGN;
  }
  if (c->k_stride_t < kHeadDim || c->v_stride_t < kHeadDim) return SFI_EINVAL;
  // row offsets inside one (sequence, KV head) are 32-bit byte offsets in the kernels
  if (c->page_size == 0 && ((int64_t)c->max_ctx * c->k_stride_t * 2 >= ((int64_t)1 << 32) ||
                            (int64_t)c->max_ctx * c->v_stride_t * 2 >= ((int64_t)1 << 32)))
    return SFI_EUNSUPPORTED;
  return SFI_OK;
}

// Carves the workspace; base may be null (size computation only).  Returns total bytes.
size_t carve(const sfi_config* c, char* base, Workspace* ws) {
  const int64_t B = c->batch, Hq = c->n_q_heads, Hkv = c->n_kv_heads;
  const int64_t ld = (int64_t)align_up((size_t)c->max_ctx, kSelSeg);
  const int n_seg = (int)(ld / kSelSeg);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  ws->part = (float*)take((size_t)(B * Hq) * kSlotCap * kPartStride * sizeof(float));
  const bool full = c->selector_mode == 1;
  // exposed rows per (b, h): the G heads' y and, for the full Selector, the squared key norms
  ws->logits = (float*)take((size_t)(B * Hq + (full ? B * Hkv : 0)) * ld * sizeof(float));
  ws->keys = (uint32_t*)take((size_t)(B * Hkv) * ld * sizeof(uint32_t));
  ws->cand = (uint32_t*)take((size_t)(B * Hkv) * ld * 2 * sizeof(uint32_t));
  ws->hist1 = (uint32_t*)take((size_t)(B * Hkv) * kHist1Bins * sizeof(uint32_t));
  ws->state = (uint32_t*)take((size_t)(B * Hkv) * kStateWords * sizeof(uint32_t));
  ws->segcnt = (uint32_t*)take((size_t)(B * Hkv) * n_seg * sizeof(uint32_t));
  ws->jstat = (float2*)take((size_t)(B * Hq) * sizeof(float2));
  ws->mu = (float*)take((size_t)(B * Hkv) * ld * sizeof(float));
  ws->arrive = (uint32_t*)take((size_t)(B * Hkv) * sizeof(uint32_t));
  ws->guard = (int32_t*)take(sizeof(int32_t));  // directly behind the counters: one memset clears both
  ws->prior = full ? (float*)take((size_t)(B * Hkv) * ld * sizeof(float)) : nullptr;
  ws->znms = full ? (float*)take((size_t)(B * Hkv) * ld * sizeof(float)) : nullptr;
  ws->segstat = full ? (double*)take((size_t)(B * Hkv) * n_seg * kSegStats * sizeof(double)) : nullptr;
  ws->seq_splits = (int32_t*)take((size_t)B * sizeof(int32_t));
  ws->ld_pos = ld;
  ws->n_seg_cap = n_seg;
  return off;
}

inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// Workgroups per (sequence, KV head) pair for a launch whose pairs each hold `tiles` 32-row tiles.
// A compute unit pulls rows at a fixed rate however many workgroups share it, so a launch takes as
// long as its busiest compute unit: w = pairs * s workgroups over n_cu units cost ceil(w / n_cu)
// shares where w / n_cu would do (264 workgroups on 256 units take twice as long as 256).  A share
// is a wave's tiles plus a start and an end worth about three tiles; in a single round the waves
// move in step, one trip to memory per tile, so the wave with the most tiles counts.  A launch that
// merges its records in the kernel pays about two thirds of a tile for every further group of eight
// workgroups per pair.  Take the s with the lowest cost, the smaller s on a tie.  (Measured at 12, 24,
// 33 and 40 sequences of 8 KV heads: 13 to 43 % faster dense launches than one workgroup per compute
// unit rounded down; one long stream: 18 workgroups per pair instead of 32, 6 % faster fast steps; the
// same choice as one workgroup per compute unit where the pairs divide the compute units.)
int balanced_splits(int pairs, int tiles, int cap, int n_cu, bool merges_in_kernel) {
  int best = 1;
  double best_cost = 1e300;
  for (int s = 1; s <= cap; ++s) {
    const double r = (double)pairs * s / n_cu;
    const double t = (double)tiles / (kWaves * s);
    const double share = (r <= 1.0 ? ceil(t) : t) + 3.0;
    const double cost = ceil(r) * share + (merges_in_kernel ? (2.0 / 3.0) * ((s + 7) / 8 - 1) : 0.0);
    if (cost < best_cost * (1.0 - 1e-9)) {
      best = s;
      best_cost = cost;
    }
  }
  return best;
}

// Split workgroups per (sequence, KV head) of a dense launch.  All sequences dense: the balanced
// split above (config 2: one workgroup per compute unit, all resident at once, one round of equal
// shares of the prefix, sink and recent rows included); dense_target_wgs > 0 overrides with that many
// workgroups in total.  Mixed step: the host cannot know how many sequences are slow, so take the
// finest split; workgroups of fast sequences exit at once.
int dense_splits_for(const sfi_ctx* x, int max_len, bool mixed) {
  const int nJ = max_len - x->cfg.recent - x->cfg.n_sink;
  const int tiles_sr = (x->cfg.n_sink + x->cfg.recent + kTile - 1) / kTile;
  const int tiles = (nJ > 0 ? (nJ + kTile - 1) / kTile : 0) + tiles_sr;
  const int pairs = x->cfg.batch * x->cfg.n_kv_heads;
  int cap = (tiles + kWaves - 1) / kWaves;
  if (cap > kMaxSplits) cap = kMaxSplits;
  // records per query head: one per wave for J plus one per wave that owns sink / recent tiles
  while (cap > 1 && cap * kWaves + (cap * kWaves < tiles_sr ? cap * kWaves : tiles_sr) > kSlotCap) --cap;
  int s;
  if (mixed) s = cap;
  else if (x->dense_target_wgs > 0) s = x->dense_target_wgs / pairs;
  else s = balanced_splits(pairs, tiles, cap, x->n_cu, false);
  if (s > cap) s = cap;
  if (s < 1) s = 1;
  return s;
}

void set_dense_bounds(const sfi_ctx* x, AttnArgs* a, int max_len) {
  const int nJ = max_len - x->cfg.recent - x->cfg.n_sink;
  a->max_tiles = nJ > 0 ? (nJ + kTile - 1) / kTile : 0;
  a->row_cap = max_len - 1;
  a->len_cap = max_len;
}

// Gather launch geometry: the balanced split above.  With one workgroup per pair the workgroup
// finishes the softmax itself (no records, no merge).  A split that leaves every wave at most one
// tile runs the one-tile kernel, any other the pipelined one.  (Config 2: 6 workgroups per pair, up to
// 3 tiles per wave; 33 sequences of 8 KV heads: 2 workgroups per pair instead of 1, 10 % faster.)
// fast_tiles_per_wave > 0 overrides: 1 = one tile per wave, t > 1 = pipelined with about t tiles per
// wave.
int fast_splits_for(const sfi_ctx* x, int sel_stride, int* pipelined, int max_splits = kMaxSplits) {
  const int rows = x->cfg.n_sink + sel_stride + x->cfg.recent;
  const int tiles = (rows + kTile - 1) / kTile;
  const int pairs = x->cfg.batch * x->cfg.n_kv_heads;
  int one = (tiles + kWaves - 1) / kWaves;
  if (one > kMaxSplits) one = kMaxSplits;
  if (one > max_splits) one = max_splits;  // records the buffer has room for
  int s;
  if (x->fast_tiles_per_wave > 0)
    s = (tiles + kWaves * x->fast_tiles_per_wave - 1) / (kWaves * x->fast_tiles_per_wave);
  else
    s = balanced_splits(pairs, tiles, one, x->n_cu, x->tail_merge != 0);
  if (s > one) s = one;
  if (s < 1) s = 1;
  *pipelined = s * kWaves < tiles;
  return s;
}

// The compact segment and the recent window are tiled separately (no tile straddles them); the kernel walks
// several tiles per wave with the same pipelined loop, so the gather policy's workgroup counts apply.
int compact_splits_for(const sfi_ctx* x, int sel_stride) {
  const int tiles = (x->cfg.n_sink + sel_stride + kTile - 1) / kTile + (x->cfg.recent + kTile - 1) / kTile;
  const int pairs = x->cfg.batch * x->cfg.n_kv_heads;
  int one = (tiles + kWaves - 1) / kWaves;
  if (one > kMaxSplits) one = kMaxSplits;
  int s;
  if (x->fast_tiles_per_wave > 0)
    s = (tiles + kWaves * x->fast_tiles_per_wave - 1) / (kWaves * x->fast_tiles_per_wave);
  else
    s = balanced_splits(pairs, tiles, one, x->n_cu, x->tail_merge != 0);
  if (s > one) s = one;
  if (s < 1) s = 1;
  return s;
}

struct StageTimer {
  sfi_ctx* x;
  hipStream_t s;
  int stage;
  bool ok;
  StageTimer(sfi_ctx* ctx, hipStream_t st, int stg) : x(ctx), s(st), stage(stg), ok(true) {
    if (recording()) {
      ok = hipEventRecord(slot()[0], s) == hipSuccess;
      x->ev_used[(size_t)x->prof_calls * SFI_N_STAGES + stage] = 1;
    }
  }
  bool recording() const { return x->profiling && x->prof_calls < x->prof_cap; }
  hipEvent_t* slot() const { return x->ev + ((size_t)x->prof_calls * SFI_N_STAGES + stage) * 2; }
  bool stop() {
    if (recording()) ok = ok && hipEventRecord(slot()[1], s) == hipSuccess;
    return ok;
  }
};

void fill_attn(const sfi_ctx* x, AttnArgs* a, const void* q, const void* K, const void* V,
               const int32_t* ctx_len) {
  memset(a, 0, sizeof(*a));
  const sfi_config& c = x->cfg;
  a->q = (const uint16_t*)q;
  a->K = (const uint16_t*)K;
  a->V = (const uint16_t*)V;
  a->k_sb = c.k_stride_b; a->k_sh = c.k_stride_h; a->k_st = c.k_stride_t;
  a->v_sb = c.v_stride_b; a->v_sh = c.v_stride_h; a->v_st = c.v_stride_t;
  a->ctx_len = ctx_len;
  a->ms = 1; a->fs = 1;
  a->dense_wide = x->dense_wide;
  a->part = x->ws.part;
  a->slot_cap = kSlotCap;
  a->ld_pos = x->ws.ld_pos;
  a->Hq = c.n_q_heads; a->Hkv = c.n_kv_heads; a->G = x->G;
  a->n_sink = c.n_sink; a->recent = c.recent;
  a->scale_log2 = (float)((double)x->scale * 1.4426950408889634);
  a->table = x->table; a->table_stride = x->table_stride; a->page_lg = x->page_lg; a->page_rpb = x->page_rpb;
  a->n_blocks = x->n_blocks;
  a->len_cap = c.max_ctx;  // calls with a max_len lower it (set_dense_bounds)
  a->out_bf16 = c.out_bf16;
  a->guard = x->ws.guard;
}

void fill_sel(const sfi_ctx* x, SelArgs* s, const int32_t* ctx_len, int max_len, const uint8_t* is_slow, int budget,
              int n_split, int32_t* sel_idx, int32_t* n_sel) {
  memset(s, 0, sizeof(*s));
  const sfi_config& c = x->cfg;
  s->jstat = x->ws.jstat; s->logits = x->ws.logits; s->keys = x->ws.keys; s->cand = x->ws.cand;
  s->hist1 = x->ws.hist1; s->state = x->ws.state; s->segcnt = x->ws.segcnt;
  s->ctx_len = ctx_len; s->is_slow = is_slow; s->sel_idx = sel_idx; s->n_sel = n_sel;
  s->ms = 1; s->fs = 1;
  s->ld_pos = x->ws.ld_pos; s->n_seg_cap = x->ws.n_seg_cap;
  s->Hq = c.n_q_heads; s->Hkv = c.n_kv_heads; s->G = x->G;
  s->n_sink = c.n_sink; s->recent = c.recent; s->n_jrec = n_split * kWaves; s->budget = budget;
  s->prior = x->ws.prior; s->znms = x->ws.znms; s->segstat = x->ws.segstat;
  s->gamma = c.gamma; s->beta = c.beta; s->p = c.p; s->eta = c.eta; s->lambda_clip = c.lambda_clip;
  s->alpha_soft = c.alpha_soft; s->alpha_cross = c.alpha_cross;
  s->inv_temp = c.temp > 0.f ? 1.0f / c.temp : 1.0f;
  s->eps = c.eps > 0.f ? c.eps : 1e-8f;
  s->nms_radius = c.nms_radius;
  s->alpha = x->alpha;
  s->inv_alpha = 1.0f / x->alpha;
  s->mu = x->ws.mu; s->mu_scale = 1.0f;
  s->lg_rows = x->G + (c.selector_mode == 1 ? 1 : 0);
  s->len_cap = max_len;
  s->out_bf16 = c.out_bf16;
}

#define SFI_TRY(expr)                         \
  do {                                        \
    if ((expr) != hipSuccess) return SFI_ELAUNCH; \
  } while (0)

// Selector kernels after a dense launch that exposed logits.
// windowed: rank the accumulated evidence (sa.mu_scale set) instead of the last query's.
int run_selector(sfi_ctx* x, const SelArgs& sa, int max_len, hipStream_t st, bool windowed = false) {
  const int B = x->cfg.batch;
  const int nJ = max_len - x->cfg.recent - x->cfg.n_sink;
  int n_seg = nJ > 0 ? (nJ + kSelSeg - 1) / kSelSeg : 1;
  if (n_seg > x->ws.n_seg_cap) n_seg = x->ws.n_seg_cap;
  if (x->selector_ran) SFI_TRY(launch_sel_clear(sa, B, st));  // a second pass over the same evidence
  x->selector_ran = 1;
  {
    StageTimer t(x, st, SFI_STAGE_SCORE);
    if (x->cfg.selector_mode == 1) SFI_TRY(launch_sel_full(sa, B, n_seg, st));
    else if (windowed) SFI_TRY(launch_sel_finalize(sa, B, n_seg, st));
    else SFI_TRY(launch_sel_score(sa, B, n_seg, st));
    if (!t.stop()) return SFI_ELAUNCH;
  }
  { StageTimer t(x, st, SFI_STAGE_CAND);  SFI_TRY(launch_sel_cand(sa, B, n_seg, st));  if (!t.stop()) return SFI_ELAUNCH; }
  { StageTimer t(x, st, SFI_STAGE_WRITE); SFI_TRY(launch_sel_write(sa, B, n_seg, st)); if (!t.stop()) return SFI_ELAUNCH; }
  return SFI_OK;
}

int check_common(const sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                 const void* out) {
  if (x == nullptr || q == nullptr || K == nullptr || V == nullptr || ctx_len == nullptr || out == nullptr)
    return SFI_EINVAL;
  if (misaligned(q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(out, 16) || misaligned(ctx_len, 4))
    return SFI_EALIGN;
  if (x->cfg.page_size != 0 && x->table == nullptr) return SFI_EINVAL;  // paged cache without a block table
  return SFI_OK;
}

int resolve_max_len(const sfi_ctx* x, int32_t max_len, int* out) {
  if (max_len < 0 || max_len > x->cfg.max_ctx) return SFI_EINVAL;
  *out = max_len == 0 ? x->cfg.max_ctx : max_len;
  return SFI_OK;
}

// Closes the profiling record of one hot call (its stages were bracketed by StageTimer).
struct CallRecord {
  sfi_ctx* x;
  explicit CallRecord(sfi_ctx* ctx) : x(ctx) {}
  ~CallRecord() {
    if (x->profiling && x->prof_calls < x->prof_cap) ++x->prof_calls;
  }
};

}  // namespace

extern "C" {

size_t sfi_workspace_bytes(const sfi_config* cfg) {
  if (validate(cfg) != SFI_OK) return 0;
  Workspace ws;
  return carve(cfg, nullptr, &ws);
}

int sfi_create(const sfi_config* cfg, void* workspace, size_t workspace_bytes, sfi_ctx** out) {
  if (out == nullptr) return SFI_EINVAL;
  *out = nullptr;
  const int v = validate(cfg);
  if (v != SFI_OK) return v;
  if (workspace == nullptr) return SFI_EINVAL;
  if (misaligned(workspace, 256)) return SFI_EWORKSPACE;
  Workspace ws;
  const size_t need = carve(cfg, (char*)workspace, &ws);
  if (workspace_bytes < need) return SFI_EWORKSPACE;
  sfi_ctx* x = new (std::nothrow) sfi_ctx;
  if (x == nullptr) return SFI_ENOMEM;
  memset(x, 0, sizeof(*x));
  x->cfg = *cfg;
  x->scale = cfg->scale > 0.f ? cfg->scale : 1.0f / sqrtf((float)cfg->head_dim);
  x->G = cfg->n_q_heads / cfg->n_kv_heads;
  x->alpha = cfg->alpha > 0.f ? cfg->alpha : 1.0f;
  for (int p = cfg->page_size; p > 1; p >>= 1) ++x->page_lg;
  x->page_rpb = cfg->k_stride_page != 0 ? (int)(cfg->k_stride_page / cfg->k_stride_t) : cfg->page_size;
  x->ws = ws;
  x->n_cu = 256;
  int dev = 0;
  hipDeviceProp_t prop;
  bool have_device = false;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
      prop.multiProcessorCount > 0) {
    x->n_cu = prop.multiProcessorCount;
    have_device = true;
  } else {
    (void)hipGetLastError();  // no device here: keep the MI355X default
  }
  x->dense_target_wgs = 0;
  x->fast_tiles_per_wave = 0;
  x->tail_merge = 1;
  x->mixed_plan = 1;
  // The arrival counters of split fast-step launches start at zero (and every launch leaves them there).
  // A workspace the runtime knows (device, managed, pinned) is cleared here and a failure to do so is an error: with stale
  // counters no workgroup would ever take itself for the last one.  (Without a device, or with a
  // pointer the runtime does not know, nothing can be launched on this context anyway.)
  hipPointerAttribute_t attr;
  if (have_device && hipPointerGetAttributes(&attr, ws.arrive) == hipSuccess &&
      attr.type != hipMemoryTypeUnregistered) {  // device, managed or pinned host memory: all of it is cleared here
    const size_t n_clear = (size_t)((char*)ws.guard - (char*)ws.arrive) + sizeof(int32_t);  // counters and guard word
    if (hipMemset(ws.arrive, 0, n_clear) != hipSuccess ||
        hipDeviceSynchronize() != hipSuccess) {
      (void)hipGetLastError();
      delete x;
      return SFI_ELAUNCH;
    }
  } else {
    (void)hipGetLastError();
  }
  *out = x;
  return SFI_OK;
}

int sfi_set_block_table(sfi_ctx* x, const int32_t* block_table, int32_t table_stride, int32_t n_blocks) {
  if (x == nullptr) return SFI_EINVAL;
  if (block_table == nullptr) {
    x->table = nullptr;
    return SFI_OK;
  }
  const sfi_config& c = x->cfg;
  if (c.page_size == 0) return SFI_EINVAL;  // the context was created for a flat cache
  if (misaligned(block_table, 4)) return SFI_EALIGN;
  const int64_t pages = ((int64_t)c.max_ctx + c.page_size - 1) / c.page_size;
  if (table_stride < pages || n_blocks < 1) return SFI_EINVAL;
  if ((int64_t)n_blocks * x->page_rpb >= ((int64_t)1 << 31)) return SFI_EUNSUPPORTED;  // row numbers are 32-bit
  x->table = block_table;
  x->table_stride = table_stride;
  x->n_blocks = n_blocks;
  return SFI_OK;
}

int sfi_destroy(sfi_ctx* x) {
  if (x == nullptr) return SFI_EINVAL;
  if (x->ev != nullptr) {
    for (size_t i = 0; i < (size_t)x->prof_cap * SFI_N_STAGES * 2; ++i) (void)hipEventDestroy(x->ev[i]);
    delete[] x->ev;
    delete[] x->ev_used;
  }
  delete x;
  return SFI_OK;
}

const char* sfi_strerror(int status) {
  switch (status) {
    case SFI_OK: return "ok";
    case SFI_EINVAL: return "invalid argument";
    case SFI_EUNSUPPORTED: return "unsupported shape or mode";
    case SFI_EWORKSPACE: return "workspace too small or misaligned";
    case SFI_EALIGN: return "pointer or stride alignment violated";
    case SFI_ELAUNCH: return "HIP launch or event call failed";
    case SFI_ENOMEM: return "host allocation failed";
    default: return "unknown status";
  }
}

int sfi_dense_attn(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                   int32_t max_len, void* out_, void* stream) {
  float* out = (float*)out_;
  int rc = check_common(x, q, K, V, ctx_len, out);
  if (rc != SFI_OK) return rc;
  int ml;
  if ((rc = resolve_max_len(x, max_len, &ml)) != SFI_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  CallRecord call_record(x);
  AttnArgs a;
  fill_attn(x, &a, q, K, V, ctx_len);
  a.n_split = dense_splits_for(x, ml, false);
  set_dense_bounds(x, &a, ml);
  x->last_dense_splits = a.n_split;
  { StageTimer t(x, st, SFI_STAGE_ATTN); SFI_TRY(launch_attn_dense(a, x->cfg.batch, a.n_split, st)); if (!t.stop()) return SFI_ELAUNCH; }
  MergeArgs m{x->ws.part, out, nullptr, x->cfg.n_q_heads, a.n_split * kWaves, 0, 0, nullptr, 0, x->G, ctx_len, nullptr, x->cfg.n_sink, x->cfg.recent, x->alpha, ml, x->cfg.out_bf16};
  { StageTimer t(x, st, SFI_STAGE_MERGE); SFI_TRY(launch_merge(m, x->cfg.batch, st)); if (!t.stop()) return SFI_ELAUNCH; }
  return SFI_OK;
}

// Memory skeleton of the dense launch (measurement aid): the launch plan of sfi_dense_attn, loads only.
int sfi_dense_attn_floor(sfi_ctx* x, const void* K, const void* V, const int32_t* ctx_len, int32_t max_len, int32_t variant,
                         void* stream) {
  if (x == nullptr || K == nullptr || V == nullptr || ctx_len == nullptr) return SFI_EINVAL;
  if (misaligned(K, 16) || misaligned(V, 16) || misaligned(ctx_len, 4)) return SFI_EALIGN;
  const int idle_units = (variant >> 4) & 127, writer = variant >> 11;
  if (variant < 0 || (variant & 15) > 1 || idle_units > 64 || writer > 2 || x->table != nullptr || x->cfg.page_size != 0) return SFI_EUNSUPPORTED;
  int ml;
  const int rc = resolve_max_len(x, max_len, &ml);
  if (rc != SFI_OK) return rc;
  AttnArgs a;
  fill_attn(x, &a, K /* q is not read */, K, V, ctx_len);
  a.n_split = dense_splits_for(x, ml, false);
  set_dense_bounds(x, &a, ml);
  x->last_dense_splits = a.n_split;
  a.logits = x->ws.logits;  // where the writer wave's stores go (the slow step's logits buffer)
  SFI_TRY(launch_attn_dense_floor(a, x->cfg.batch, a.n_split, variant & 1, idle_units, writer, (hipStream_t)stream));
  return SFI_OK;
}

namespace {
// First half of a slow step: dense attention with the evidence (y over J, Selector state cleared,
// J-only softmax statistics) left in the workspace.
int slow_attn_impl(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* ctx_len, int ml,
                   float* out, hipStream_t st, bool merge_later = false, const int32_t* q_len = nullptr) {
  AttnArgs a;
  fill_attn(x, &a, q, K, V, ctx_len);
  a.q_len = q_len;
  a.n_split = dense_splits_for(x, ml, false);
  set_dense_bounds(x, &a, ml);
  a.logits = x->ws.logits;
  a.with_knorm = x->cfg.selector_mode == 1;
  a.big_stash = 1;  // every sequence is dense: one workgroup per compute unit, half as many write bursts
  a.no_v = out == nullptr;  // evidence only (sfi_evidence_add without an output)
  a.hist1 = x->ws.hist1;
  a.state = x->ws.state;
  x->last_dense_splits = a.n_split;
  { StageTimer t(x, st, SFI_STAGE_ATTN); SFI_TRY(launch_attn_dense(a, x->cfg.batch, a.n_split, st)); if (!t.stop()) return SFI_ELAUNCH; }
  x->selector_ran = 0;  // fresh evidence, Selector state cleared by the launch above
  if (merge_later) return SFI_OK;  // the Selector's scoring launch merges
  MergeArgs m{x->ws.part, out, nullptr, x->cfg.n_q_heads, a.n_split * kWaves, 0, 0, x->ws.jstat, a.n_split * kWaves, x->G, ctx_len, q_len, x->cfg.n_sink, x->cfg.recent, x->alpha, ml, x->cfg.out_bf16};
  { StageTimer t(x, st, SFI_STAGE_MERGE); SFI_TRY(launch_merge(m, x->cfg.batch, st)); if (!t.stop()) return SFI_ELAUNCH; }
  return SFI_OK;
}

int check_select(const sfi_ctx* x, const int32_t* ctx_len, int32_t budget, const int32_t* sel_idx, const int32_t* n_sel) {
  if (x == nullptr || ctx_len == nullptr || sel_idx == nullptr || n_sel == nullptr) return SFI_EINVAL;
  if (budget < 0 || budget > x->cfg.max_budget) return SFI_EINVAL;
  if (misaligned(ctx_len, 4) || misaligned(sel_idx, 4) || misaligned(n_sel, 4)) return SFI_EALIGN;
  return SFI_OK;
}
}  // namespace

int sfi_slow_step(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                  int32_t max_len, int32_t budget, void* out_, int32_t* sel_idx, int32_t* n_sel,
                  void* stream) {
  float* out = (float*)out_;
  int rc = check_common(x, q, K, V, ctx_len, out);
  if (rc != SFI_OK) return rc;
  if ((rc = check_select(x, ctx_len, budget, sel_idx, n_sel)) != SFI_OK) return rc;
  int ml;
  if ((rc = resolve_max_len(x, max_len, &ml)) != SFI_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  CallRecord call_record(x);
  // no merge launch: the merge rides in the Selector's first launch (one launch less on the step's critical path)
  if ((rc = slow_attn_impl(x, q, K, V, ctx_len, ml, out, st, true)) != SFI_OK) return rc;
  SelArgs sa;
  fill_sel(x, &sa, ctx_len, ml, nullptr, budget, x->last_dense_splits, sel_idx, n_sel);
  sa.part = x->ws.part;
  sa.merge_out = out;
  return run_selector(x, sa, ml, st);
}

int sfi_slow_attn(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                  int32_t max_len, void* out_, void* stream) {
  float* out = (float*)out_;
  int rc = check_common(x, q, K, V, ctx_len, out);
  if (rc != SFI_OK) return rc;
  int ml;
  if ((rc = resolve_max_len(x, max_len, &ml)) != SFI_OK) return rc;
  CallRecord call_record(x);
  return slow_attn_impl(x, q, K, V, ctx_len, ml, out, (hipStream_t)stream);
}

int sfi_slow_select(sfi_ctx* x, const int32_t* ctx_len, int32_t max_len, int32_t budget, int32_t* sel_idx,
                    int32_t* n_sel, void* stream) {
  int rc = check_select(x, ctx_len, budget, sel_idx, n_sel);
  if (rc != SFI_OK) return rc;
  int ml;
  if ((rc = resolve_max_len(x, max_len, &ml)) != SFI_OK) return rc;
  CallRecord call_record(x);
  SelArgs sa;
  fill_sel(x, &sa, ctx_len, ml, nullptr, budget, x->last_dense_splits, sel_idx, n_sel);
  return run_selector(x, sa, ml, (hipStream_t)stream);
}

namespace {
int evidence_add_impl(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* ctx_len, const int32_t* q_len,
                      int32_t max_len, float* out, int32_t first, hipStream_t st) {
  // out == nullptr: evidence only -- V is not read (and may be null), no attention output is produced
  const bool evidence_only = out == nullptr;
  if (x == nullptr || q == nullptr || K == nullptr || ctx_len == nullptr || (!evidence_only && V == nullptr))
    return SFI_EINVAL;
  if (misaligned(q, 16) || misaligned(K, 16) || misaligned(ctx_len, 4) || misaligned(q_len, 4) ||
      (!evidence_only && (misaligned(V, 16) || misaligned(out, 16))))
    return SFI_EALIGN;
  if (x->cfg.page_size != 0 && x->table == nullptr) return SFI_EINVAL;  // paged cache without a block table
  int rc;
  int ml;
  if ((rc = resolve_max_len(x, max_len, &ml)) != SFI_OK) return rc;
  CallRecord call_record(x);
  if ((rc = slow_attn_impl(x, q, K, V, ctx_len, ml, out, st, false, q_len)) != SFI_OK) return rc;
  SelArgs sa;
  fill_sel(x, &sa, ctx_len, ml, nullptr, 0, x->last_dense_splits, nullptr, nullptr);
  sa.accum_first = first != 0;
  sa.q_len = q_len;
  // a query under the causal mask may see up to `recent` more positions of its own, shorter context as allowed set
  const int nJ = ml - (q_len != nullptr ? 0 : x->cfg.recent) - x->cfg.n_sink;
  int n_seg = nJ > 0 ? (nJ + kSelSeg - 1) / kSelSeg : 1;
  if (n_seg > x->ws.n_seg_cap) n_seg = x->ws.n_seg_cap;
  { StageTimer t(x, st, SFI_STAGE_SCORE); SFI_TRY(launch_sel_accum(sa, x->cfg.batch, n_seg, st)); if (!t.stop()) return SFI_ELAUNCH; }
  return SFI_OK;
}
}  // namespace

int sfi_evidence_add(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                     int32_t max_len, void* out, int32_t first, void* stream) {
  return evidence_add_impl(x, q, K, V, ctx_len, nullptr, max_len, (float*)out, first, (hipStream_t)stream);
}

int sfi_evidence_add_causal(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* ctx_len,
                            const int32_t* q_len, int32_t max_len, void* out, int32_t first, void* stream) {
  if (q_len == nullptr) return SFI_EINVAL;
  return evidence_add_impl(x, q, K, V, ctx_len, q_len, max_len, (float*)out, first, (hipStream_t)stream);
}

int sfi_evidence_select(sfi_ctx* x, int32_t n_added, const int32_t* ctx_len, int32_t max_len, int32_t budget,
                        int32_t* sel_idx, int32_t* n_sel, void* stream) {
  int rc = check_select(x, ctx_len, budget, sel_idx, n_sel);
  if (rc != SFI_OK) return rc;
  if (n_added < 1) return SFI_EINVAL;
  int ml;
  if ((rc = resolve_max_len(x, max_len, &ml)) != SFI_OK) return rc;
  CallRecord call_record(x);
  SelArgs sa;
  fill_sel(x, &sa, ctx_len, ml, nullptr, budget, x->last_dense_splits, sel_idx, n_sel);
  sa.mu_scale = 1.0f / (float)n_added;
  sa.f_from_mu = 1;
  return run_selector(x, sa, ml, (hipStream_t)stream, true);
}

namespace {
// The fast step's launches on records / counters / status word given by the caller of this function: the
// context's workspace (sfi_fast_step) or the library's static scratch (sfi_fast_step_static).  max_splits bounds
// the workgroups per pair by the records the buffer has room for.
int fast_step_on(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* sel_idx, const int32_t* n_sel,
                 int32_t sel_stride, const int32_t* recent_start, const int32_t* ctx_len, float* out, hipStream_t st,
                 float* part, int slot_cap, uint32_t* arrive, int32_t* guard, const int32_t* one_word, int max_splits) {
  AttnArgs a;
  fill_attn(x, &a, q, K, V, ctx_len);
  a.part = part;
  a.slot_cap = slot_cap;
  a.guard = guard;
  a.recent_start = recent_start;
  // an index list of width 0: the pipelined kernel still reads one word where the list would start
  a.sel_idx = sel_stride > 0 ? sel_idx : one_word;
  a.n_sel = n_sel;
  a.sel_stride = sel_stride;
  a.n_split = fast_splits_for(x, sel_stride, &a.pipelined, max_splits);
  x->last_fast_splits = a.n_split;
  if (a.n_split == 1) a.out_direct = out;  // one workgroup per pair finishes the softmax itself
  else if (x->tail_merge) { a.out_merge = out; a.arrive = arrive; }
  { StageTimer t(x, st, SFI_STAGE_ATTN); SFI_TRY(launch_attn_gather(a, x->cfg.batch, a.n_split, st)); if (!t.stop()) return SFI_ELAUNCH; }
  if (a.n_split == 1 || a.out_merge != nullptr) return SFI_OK;
  MergeArgs m{part, out, nullptr, x->cfg.n_q_heads, 0, a.n_split, 1, nullptr, 0, x->G, ctx_len, nullptr, x->cfg.n_sink, x->cfg.recent, x->alpha, x->cfg.max_ctx, x->cfg.out_bf16};
  { StageTimer t(x, st, SFI_STAGE_MERGE); SFI_TRY(launch_merge(m, x->cfg.batch, st)); if (!t.stop()) return SFI_ELAUNCH; }
  return SFI_OK;
}

int check_fast(const sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* sel_idx, const int32_t* n_sel,
               int32_t sel_stride, const int32_t* recent_start, const int32_t* ctx_len, const void* out) {
  int rc = check_common(x, q, K, V, ctx_len, out);
  if (rc != SFI_OK) return rc;
  if (sel_stride < 0 || sel_stride > x->cfg.max_budget) return SFI_EINVAL;
  if ((sel_idx == nullptr && sel_stride > 0) || n_sel == nullptr || recent_start == nullptr) return SFI_EINVAL;
  if (misaligned(sel_idx, 4) || misaligned(n_sel, 4) || misaligned(recent_start, 4)) return SFI_EALIGN;
  return SFI_OK;
}
}  // namespace

int sfi_fast_step(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* sel_idx,
                  const int32_t* n_sel, int32_t sel_stride, const int32_t* recent_start,
                  const int32_t* ctx_len, void* out, void* stream) {
  const int rc = check_fast(x, q, K, V, sel_idx, n_sel, sel_stride, recent_start, ctx_len, out);
  if (rc != SFI_OK) return rc;
  CallRecord call_record(x);
  return fast_step_on(x, q, K, V, sel_idx, n_sel, sel_stride, recent_start, ctx_len, (float*)out, (hipStream_t)stream,
                      x->ws.part, kSlotCap, x->ws.arrive, x->ws.guard, x->ws.guard, kMaxSplits);
}

// Memory skeleton of the fast step (measurement aid): the launch plan of sfi_fast_step, no arithmetic.
int sfi_fast_step_floor(sfi_ctx* x, const void* q, const void* K, const void* V, const int32_t* sel_idx,
                        const int32_t* n_sel, int32_t sel_stride, const int32_t* recent_start,
                        const int32_t* ctx_len, void* out, int32_t variant, void* stream) {
  const int rc = check_fast(x, q, K, V, sel_idx, n_sel, sel_stride, recent_start, ctx_len, out);
  if (rc != SFI_OK) return rc;
  if (variant < 0 || variant > 15 || x->table != nullptr) return SFI_EUNSUPPORTED;
  const bool tail = (variant & 1) != 0, burst = (variant & 2) != 0;
  const int depth = variant >> 2;
  if ((tail && burst) || depth > 2 || (depth != 0 && (tail || burst))) return SFI_EUNSUPPORTED;
  AttnArgs a;
  fill_attn(x, &a, q, K, V, ctx_len);
  a.recent_start = recent_start;
  a.sel_idx = sel_stride > 0 ? sel_idx : x->ws.guard;
  a.n_sel = n_sel;
  a.sel_stride = sel_stride;
  a.n_split = fast_splits_for(x, sel_stride, &a.pipelined);
  const int tiles = (x->cfg.n_sink + sel_stride + x->cfg.recent + kTile - 1) / kTile;
  int tpw = (tiles + a.n_split - 1) / a.n_split;
  if (burst) {  // the workgroup's tiles must fit its LDS (nine tiles of 16 KB)
    while (tpw > 9 && a.n_split < kMaxSplits) {
      ++a.n_split;
      tpw = (tiles + a.n_split - 1) / a.n_split;
    }
    if (tpw > 9) return SFI_EUNSUPPORTED;
  }
  x->last_fast_splits = a.n_split;
  if (tail && a.n_split == 1) a.out_direct = (float*)out;
  else if (tail) { a.out_merge = (float*)out; a.arrive = x->ws.arrive; }
  SFI_TRY(launch_attn_gather_floor(a, x->cfg.batch, a.n_split, tail, burst, tpw, depth, (hipStream_t)stream));
  return SFI_OK;
}

// ---- the fast step for callers that cannot allocate ------------------------------------------------------
// Split records and arrival counters live in a file-scope device array instead of a caller's workspace.
namespace {
constexpr int kStaticRecords = 8192;   // split records the scratch holds: batch * n_q_heads * splits per pair
constexpr int kStaticPairs = 4096;     // arrival counters: batch * n_kv_heads
constexpr size_t kStaticRecordBytes = (size_t)kStaticRecords * kPartStride * sizeof(float);
constexpr size_t kStaticBytes = kStaticRecordBytes + (size_t)kStaticPairs * sizeof(uint32_t) + 256;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticBytes];
namespace {
struct StaticScratch {
  unsigned char* ptr;   // this device's copy of `scratch` (hipGetSymbolAddress), nullptr until its first call
  int n_cu;
  bool counters_clean;  // the arrival counters are known to be zero (every completed launch leaves them so)
};
StaticScratch g_static[kMaxDevices];
std::mutex g_static_mutex;

__global__ void clear_words_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}
}  // namespace

int sfi_fast_step_static(const sfi_config* cfg, const void* q, const void* K, const void* V, const int32_t* sel_idx,
                         const int32_t* n_sel, int32_t sel_stride, const int32_t* recent_start,
                         const int32_t* ctx_len, void* out, void* stream) {
  int rc = validate(cfg);
  if (rc != SFI_OK) return rc;
  if (cfg->page_size != 0) return SFI_EUNSUPPORTED;  // no context to hold a block table
  const int64_t heads = (int64_t)cfg->batch * cfg->n_q_heads, pairs = (int64_t)cfg->batch * cfg->n_kv_heads;
  if (heads > kStaticRecords || pairs > kStaticPairs) return SFI_EUNSUPPORTED;  // beyond the static scratch
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return SFI_ELAUNCH; }
  if (dev < 0 || dev >= kMaxDevices) return SFI_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_static_mutex);  // calls that share a device's scratch must not overlap anyway
  StaticScratch& S = g_static[dev];
  if (S.ptr == nullptr) {  // once per device, with that device current: its own copy of the array
    unsigned char* p = nullptr;
    if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return SFI_ELAUNCH;
    }
    int n_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) {
      (void)hipGetLastError();
      return SFI_ELAUNCH;
    }
    S.n_cu = n_cu;
    S.counters_clean = false;
    S.ptr = p;
  }
  sfi_ctx x;  // a context for this call only: no workspace, no profiling, default launch policy
  memset(&x, 0, sizeof(x));
  x.cfg = *cfg;
  x.scale = cfg->scale > 0.f ? cfg->scale : 1.0f / sqrtf((float)cfg->head_dim);
  x.G = cfg->n_q_heads / cfg->n_kv_heads;
  x.alpha = cfg->alpha > 0.f ? cfg->alpha : 1.0f;
  x.n_cu = S.n_cu;
  x.tail_merge = 1;
  if ((rc = check_fast(&x, q, K, V, sel_idx, n_sel, sel_stride, recent_start, ctx_len, out)) != SFI_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  float* part = reinterpret_cast<float*>(S.ptr);
  uint32_t* arrive = reinterpret_cast<uint32_t*>(S.ptr + kStaticRecordBytes);
  const int32_t* one_word = reinterpret_cast<const int32_t*>(arrive + kStaticPairs);  // readable, never written
  const int max_splits = (int)(kStaticRecords / heads);  // >= 1
  if (!S.counters_clean) {  // first call on this device, or the call before did not get its launch out
    hipLaunchKernelGGL(clear_words_kernel, dim3((kStaticPairs + 255) / 256), dim3(256), 0, st, arrive, kStaticPairs);
    if (hipGetLastError() != hipSuccess) return SFI_ELAUNCH;
  }
  S.counters_clean = false;
  rc = fast_step_on(&x, q, K, V, sel_idx, n_sel, sel_stride, recent_start, ctx_len, (float*)out, st, part,
                    max_splits < kMaxSplits ? max_splits : kMaxSplits, arrive, nullptr, one_word, max_splits);
  S.counters_clean = rc == SFI_OK;
  return rc;
}

namespace {
// Compact-buffer geometry shared by sfi_reorg and sfi_fast_step_compact.
int check_compact(const sfi_ctx* x, const void* Kc, const void* Vc, int64_t c_stride_b, int64_t c_stride_h,
                  int32_t c_rows, int32_t sel_stride) {
  if (Kc == nullptr || Vc == nullptr) return SFI_EINVAL;
  if (misaligned(Kc, 16) || misaligned(Vc, 16)) return SFI_EALIGN;
  if (sel_stride < 0 || sel_stride > x->cfg.max_budget) return SFI_EINVAL;
  if (c_rows < x->cfg.n_sink + sel_stride || c_rows < 1) return SFI_EINVAL;
  if (c_stride_h < (int64_t)c_rows * kHeadDim || c_stride_b < c_stride_h * x->cfg.n_kv_heads) return SFI_EINVAL;
  if (c_stride_h % 8 != 0 || c_stride_b % 8 != 0) return SFI_EALIGN;
  if ((int64_t)c_rows * kHeadDim * 2 > 0xffffffffll) return SFI_EUNSUPPORTED;
  return SFI_OK;
}
}  // namespace

namespace {
int reorg_on(sfi_ctx* x, const void* K, const void* V, const int32_t* sel_idx, const int32_t* n_sel, int32_t sel_stride,
             const int32_t* ctx_len, const uint8_t* is_slow, void* Kc, void* Vc, int64_t c_stride_b, int64_t c_stride_h,
             hipStream_t st, int meta_stride = 1) {
  const sfi_config& c = x->cfg;
  ReorgArgs r;
  memset(&r, 0, sizeof(r));
  r.K = (const uint16_t*)K; r.V = (const uint16_t*)V;
  r.k_sb = c.k_stride_b; r.k_sh = c.k_stride_h; r.k_st = c.k_stride_t;
  r.v_sb = c.v_stride_b; r.v_sh = c.v_stride_h; r.v_st = c.v_stride_t;
  r.sel_idx = sel_idx; r.n_sel = n_sel; r.ctx_len = ctx_len; r.is_slow = is_slow; r.sel_stride = sel_stride;
  r.ms = meta_stride; r.fs = meta_stride == 1 ? 1 : 4 * meta_stride;
  r.Kc = (uint16_t*)Kc; r.Vc = (uint16_t*)Vc; r.c_sb = c_stride_b; r.c_sh = c_stride_h;
  r.Hkv = c.n_kv_heads; r.n_sink = c.n_sink;
  r.table = x->table; r.table_stride = x->table_stride; r.page_lg = x->page_lg; r.page_rpb = x->page_rpb;
  r.len_cap = c.max_ctx; r.n_blocks = x->n_blocks; r.guard = x->ws.guard;
  { StageTimer t(x, st, SFI_STAGE_REORG); SFI_TRY(launch_reorg(r, c.batch, c.n_sink + sel_stride, st)); if (!t.stop()) return SFI_ELAUNCH; }
  return SFI_OK;
}
}  // namespace

int sfi_reorg(sfi_ctx* x, const void* K, const void* V, const int32_t* sel_idx, const int32_t* n_sel,
              int32_t sel_stride, const int32_t* ctx_len, const uint8_t* is_slow, void* Kc, void* Vc,
              int64_t c_stride_b, int64_t c_stride_h, int32_t c_rows, void* stream) {
  if (x == nullptr || K == nullptr || V == nullptr || sel_idx == nullptr || n_sel == nullptr || ctx_len == nullptr)
    return SFI_EINVAL;
  if (misaligned(K, 16) || misaligned(V, 16) || misaligned(sel_idx, 4) || misaligned(n_sel, 4) || misaligned(ctx_len, 4))
    return SFI_EALIGN;
  if (x->cfg.page_size != 0 && x->table == nullptr) return SFI_EINVAL;
  int rc = check_compact(x, Kc, Vc, c_stride_b, c_stride_h, c_rows, sel_stride);
  if (rc != SFI_OK) return rc;
  CallRecord call_record(x);
  return reorg_on(x, K, V, sel_idx, n_sel, sel_stride, ctx_len, is_slow, Kc, Vc, c_stride_b, c_stride_h, (hipStream_t)stream);
}

int sfi_fast_step_compact(sfi_ctx* x, const void* q, const void* Kc, const void* Vc, int64_t c_stride_b,
                          int64_t c_stride_h, int32_t c_rows, const int32_t* n_sel, int32_t sel_stride,
                          const void* K, const void* V, const int32_t* recent_start, const int32_t* ctx_len,
                          void* out_, void* stream) {
  float* out = (float*)out_;
  int rc = check_common(x, q, K, V, ctx_len, out);
  if (rc != SFI_OK) return rc;
  if (n_sel == nullptr || recent_start == nullptr) return SFI_EINVAL;
  if (misaligned(n_sel, 4) || misaligned(recent_start, 4)) return SFI_EALIGN;
  if ((rc = check_compact(x, Kc, Vc, c_stride_b, c_stride_h, c_rows, sel_stride)) != SFI_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  CallRecord call_record(x);
  AttnArgs a;
  fill_attn(x, &a, q, K, V, ctx_len);
  a.recent_start = recent_start;
  a.n_sel = n_sel;
  a.sel_stride = sel_stride;
  a.Kc = (const uint16_t*)Kc; a.Vc = (const uint16_t*)Vc;
  a.c_sb = c_stride_b; a.c_sh = c_stride_h; a.c_rows = c_rows;
  a.n_split = compact_splits_for(x, sel_stride);
  x->last_fast_splits = a.n_split;
  if (a.n_split == 1) a.out_direct = out;
  else if (x->tail_merge) { a.out_merge = out; a.arrive = x->ws.arrive; }
  { StageTimer t(x, st, SFI_STAGE_ATTN); SFI_TRY(launch_attn_compact(a, x->cfg.batch, a.n_split, st)); if (!t.stop()) return SFI_ELAUNCH; }
  if (a.n_split == 1 || a.out_merge != nullptr) return SFI_OK;
  MergeArgs m{x->ws.part, out, nullptr, x->cfg.n_q_heads, 0, a.n_split, 1, nullptr, 0, x->G, ctx_len, nullptr, x->cfg.n_sink, x->cfg.recent, x->alpha, x->cfg.max_ctx, x->cfg.out_bf16};
  { StageTimer t(x, st, SFI_STAGE_MERGE); SFI_TRY(launch_merge(m, x->cfg.batch, st)); if (!t.stop()) return SFI_ELAUNCH; }
  return SFI_OK;
}

namespace {
struct CompactBuffers {
  void* Kc;
  void* Vc;
  int64_t stride_b, stride_h;
  int32_t rows;
};

// The ragged mix.  cb == nullptr: fast sequences gather their rows through sel_idx; else they read the two-segment
// layout (compact buffers + recent window in place) and the slow sequences' buffers are refilled after the Selector.
int mixed_step_on(sfi_ctx* x, const void* q, const void* K, const void* V, const uint8_t* is_slow, const int32_t* ctx_len,
                  const int32_t* recent_start, int32_t max_len, int32_t budget, float* out, int32_t* sel_idx,
                  int32_t* n_sel, const CompactBuffers* cb, hipStream_t st, int meta_stride = 1) {
  // meta_stride 4: ctx_len, recent_start, is_slow point at the fields of a packed sfi_step_desc array
  const int ms = meta_stride, fs = meta_stride == 1 ? 1 : 4 * meta_stride;
  int rc = check_common(x, q, K, V, ctx_len, out);
  if (rc != SFI_OK) return rc;
  if (is_slow == nullptr || sel_idx == nullptr || n_sel == nullptr || recent_start == nullptr) return SFI_EINVAL;
  if (budget < 0 || budget > x->cfg.max_budget) return SFI_EINVAL;
  if (misaligned(sel_idx, 4) || misaligned(n_sel, 4) || misaligned(recent_start, 4)) return SFI_EALIGN;
  if (cb != nullptr && (rc = check_compact(x, cb->Kc, cb->Vc, cb->stride_b, cb->stride_h, cb->rows, budget)) != SFI_OK) return rc;
  int ml;
  if ((rc = resolve_max_len(x, max_len, &ml)) != SFI_OK) return rc;
  CallRecord call_record(x);

  AttnArgs d;
  fill_attn(x, &d, q, K, V, ctx_len);
  d.is_slow = is_slow;
  d.ms = ms; d.fs = fs;
  d.n_split = dense_splits_for(x, ml, true);
  set_dense_bounds(x, &d, ml);
  d.logits = x->ws.logits;
  d.with_knorm = x->cfg.selector_mode == 1;
  d.hist1 = x->ws.hist1;
  d.state = x->ws.state;
  x->last_dense_splits = d.n_split;
  AttnArgs f;
  fill_attn(x, &f, q, K, V, ctx_len);
  f.is_slow = is_slow;
  f.ms = ms; f.fs = fs;
  f.recent_start = recent_start;
  f.sel_idx = budget > 0 ? sel_idx : x->ws.guard;  // as in sfi_fast_step
  f.n_sel = n_sel;
  f.sel_stride = budget;
  f.len_cap = ml;
  if (cb != nullptr) {
    f.Kc = (const uint16_t*)cb->Kc; f.Vc = (const uint16_t*)cb->Vc;
    f.c_sb = cb->stride_b; f.c_sh = cb->stride_h; f.c_rows = cb->rows;
    f.n_split = compact_splits_for(x, budget);
  } else {
    f.n_split = fast_splits_for(x, budget, &f.pipelined);
  }
  if (f.n_split == 1) f.out_direct = out;
  else if (x->tail_merge) { f.out_merge = out; f.arrive = x->ws.arrive; }  // slow sequences' workgroups never arrive
  x->last_fast_splits = f.n_split;
  // Fast sequences finish inside their launch unless their split records need the merge launch;
  // slow sequences are merged by the first scoring launch (as in sfi_slow_step).  The merge kernel only
  // runs when the in-kernel merge is switched off (for both kinds: it skips what is already done).
  const bool fast_done = f.n_split == 1 || f.out_merge != nullptr;
  const bool merge_in_score = fast_done;
  // The dense launch plans itself on the device (one workgroup per compute unit, splits per slow sequence in proportion to
  // its length: attn_dense_items_kernel) where its records are merged by the scoring launch, which reads the plan back.
  const bool planned = x->mixed_plan != 0 && merge_in_score && x->cfg.batch <= kListCap;
  if (planned) {
    d.item_batch = x->cfg.batch;
    d.item_wgs = x->n_cu;
    d.seq_splits = x->ws.seq_splits;
  }
  // the fast part reads last segment's sel rows (or compact rows) of fast sequences; the Selector and Reorg below
  // only rewrite rows of slow sequences, so the order of the two attention launches is free.
  {
    StageTimer t(x, st, SFI_STAGE_ATTN2);
    if (cb != nullptr) SFI_TRY(launch_attn_compact(f, x->cfg.batch, f.n_split, st));
    else SFI_TRY(launch_attn_gather(f, x->cfg.batch, f.n_split, st));
    if (!t.stop()) return SFI_ELAUNCH;
  }
  { StageTimer t(x, st, SFI_STAGE_ATTN); SFI_TRY(launch_attn_dense(d, x->cfg.batch, d.n_split, st)); if (!t.stop()) return SFI_ELAUNCH; }
  x->selector_ran = 0;
  if (!merge_in_score) {
    MergeArgs m{x->ws.part, out, is_slow, x->cfg.n_q_heads, d.n_split * kWaves, fast_done ? 0 : f.n_split, 2, x->ws.jstat, d.n_split * kWaves, x->G, ctx_len, nullptr, x->cfg.n_sink, x->cfg.recent, x->alpha, ml, x->cfg.out_bf16, ms, fs};
    StageTimer t(x, st, SFI_STAGE_MERGE);
    SFI_TRY(launch_merge(m, x->cfg.batch, st));
    if (!t.stop()) return SFI_ELAUNCH;
  }
  SelArgs sa;
  fill_sel(x, &sa, ctx_len, ml, is_slow, budget, d.n_split, sel_idx, n_sel);
  sa.ms = ms; sa.fs = fs;
  if (merge_in_score) {
    sa.part = x->ws.part;
    sa.merge_out = out;
  }
  if (planned) sa.seq_splits = x->ws.seq_splits;
  if ((rc = run_selector(x, sa, ml, st)) != SFI_OK) return rc;
  if (cb == nullptr) return SFI_OK;
  // Reorg_i for the sequences that were refreshed (Sel_i -> Reorg_i)
  return reorg_on(x, K, V, sel_idx, n_sel, budget, ctx_len, is_slow, cb->Kc, cb->Vc, cb->stride_b, cb->stride_h, st, meta_stride);
}
}  // namespace

int sfi_mixed_step(sfi_ctx* x, const void* q, const void* K, const void* V, const uint8_t* is_slow,
                   const int32_t* ctx_len, const int32_t* recent_start, int32_t max_len, int32_t budget,
                   void* out, int32_t* sel_idx, int32_t* n_sel, void* stream) {
  return mixed_step_on(x, q, K, V, is_slow, ctx_len, recent_start, max_len, budget, (float*)out, sel_idx, n_sel, nullptr,
                       (hipStream_t)stream);
}

int sfi_mixed_step_compact(sfi_ctx* x, const void* q, const void* K, const void* V, const uint8_t* is_slow,
                           const int32_t* ctx_len, const int32_t* recent_start, int32_t max_len, int32_t budget,
                           void* out, int32_t* sel_idx, int32_t* n_sel, void* Kc, void* Vc, int64_t c_stride_b,
                           int64_t c_stride_h, int32_t c_rows, void* stream) {
  const CompactBuffers cb{Kc, Vc, c_stride_b, c_stride_h, c_rows};
  return mixed_step_on(x, q, K, V, is_slow, ctx_len, recent_start, max_len, budget, (float*)out, sel_idx, n_sel, &cb,
                       (hipStream_t)stream);
}

int sfi_step_begin(sfi_ctx* x, sfi_step_desc* desc, const int32_t* last_token, const uint32_t* trigger_bitmap,
                   int32_t vocab_size, int32_t t_max, int32_t advance, void* stream) {
  if (x == nullptr || desc == nullptr || t_max < 0) return SFI_EINVAL;
  if (trigger_bitmap != nullptr && vocab_size < 1) return SFI_EINVAL;
  if (misaligned(desc, 16) || misaligned(last_token, 4) || misaligned(trigger_bitmap, 4)) return SFI_EALIGN;
  SFI_TRY(launch_step_begin(desc, last_token, trigger_bitmap, vocab_size, t_max, advance != 0, x->cfg.batch, x->cfg.n_sink,
                            x->cfg.recent, (hipStream_t)stream));
  return SFI_OK;
}

int sfi_mixed_step_desc(sfi_ctx* x, const void* q, const void* K, const void* V, const sfi_step_desc* desc,
                        int32_t max_len, int32_t budget, void* out, int32_t* sel_idx, int32_t* n_sel, void* stream) {
  if (desc == nullptr) return SFI_EINVAL;
  if (misaligned(desc, 16)) return SFI_EALIGN;
  static_assert(sizeof(sfi_step_desc) == 16, "four int32 per sequence");
  return mixed_step_on(x, q, K, V, reinterpret_cast<const uint8_t*>(&desc->is_slow), &desc->ctx_len, &desc->recent_start,
                       max_len, budget, (float*)out, sel_idx, n_sel, nullptr, (hipStream_t)stream, 4);
}

int sfi_trigger(sfi_ctx* x, const int32_t* last_token, const uint32_t* trigger_bitmap, int32_t vocab_size,
                int32_t t_max, int32_t* since_slow, uint8_t* is_slow, void* stream) {
  if (x == nullptr || last_token == nullptr || trigger_bitmap == nullptr || since_slow == nullptr || is_slow == nullptr)
    return SFI_EINVAL;
  if (vocab_size < 1 || t_max < 0) return SFI_EINVAL;
  if (misaligned(last_token, 4) || misaligned(trigger_bitmap, 4) || misaligned(since_slow, 4)) return SFI_EALIGN;
  SFI_TRY(launch_trigger(last_token, trigger_bitmap, vocab_size, t_max, since_slow, is_slow, x->cfg.batch,
                         (hipStream_t)stream));
  return SFI_OK;
}

int sfi_advance(sfi_ctx* x, int32_t* ctx_len, int32_t* recent_start, void* stream) {
  if (x == nullptr || ctx_len == nullptr || recent_start == nullptr) return SFI_EINVAL;
  SFI_TRY(launch_advance(ctx_len, recent_start, x->cfg.batch, x->cfg.n_sink, x->cfg.recent, (hipStream_t)stream));
  return SFI_OK;
}

int sfi_set_profiling(sfi_ctx* x, int max_calls) {
  if (x == nullptr || max_calls < 0 || max_calls > (1 << 16)) return SFI_EINVAL;
  if (max_calls > x->prof_cap) {  // (re)build the ring
    if (x->ev != nullptr) {
      for (size_t i = 0; i < (size_t)x->prof_cap * SFI_N_STAGES * 2; ++i) (void)hipEventDestroy(x->ev[i]);
      delete[] x->ev;
      delete[] x->ev_used;
      x->ev = nullptr;
      x->ev_used = nullptr;
      x->prof_cap = 0;
    }
    const size_t n = (size_t)max_calls * SFI_N_STAGES * 2;
    x->ev = new (std::nothrow) hipEvent_t[n];
    x->ev_used = new (std::nothrow) unsigned char[(size_t)max_calls * SFI_N_STAGES];
    size_t made = 0;
    int rc = (x->ev == nullptr || x->ev_used == nullptr) ? SFI_ENOMEM : SFI_OK;
    for (; rc == SFI_OK && made < n; ++made)
      if (hipEventCreate(&x->ev[made]) != hipSuccess) { rc = SFI_ELAUNCH; break; }
    if (rc != SFI_OK) {  // leave the context without a ring rather than with half of one
      (void)hipGetLastError();
      for (size_t i = 0; i < made; ++i) (void)hipEventDestroy(x->ev[i]);
      delete[] x->ev;
      delete[] x->ev_used;
      x->ev = nullptr;
      x->ev_used = nullptr;
      x->profiling = 0;
      return rc;
    }
    x->prof_cap = max_calls;
  }
  x->profiling = max_calls > 0 ? 1 : 0;
  x->prof_calls = 0;
  if (x->ev_used != nullptr) memset(x->ev_used, 0, (size_t)x->prof_cap * SFI_N_STAGES);
  return SFI_OK;
}

int sfi_stage_times(sfi_ctx* x, float* ms_sum, int32_t* count) {
  if (x == nullptr || ms_sum == nullptr || count == nullptr) return SFI_EINVAL;
  for (int i = 0; i < SFI_N_STAGES; ++i) {
    ms_sum[i] = 0.f;
    count[i] = 0;
  }
  for (int c = 0; c < x->prof_calls; ++c)
    for (int i = 0; i < SFI_N_STAGES; ++i) {
      if (!x->ev_used[(size_t)c * SFI_N_STAGES + i]) continue;
      hipEvent_t* e = x->ev + ((size_t)c * SFI_N_STAGES + i) * 2;
      float ms = 0.f;
      if (hipEventSynchronize(e[1]) != hipSuccess) return SFI_ELAUNCH;
      if (hipEventElapsedTime(&ms, e[0], e[1]) != hipSuccess) return SFI_ELAUNCH;
      ms_sum[i] += ms;
      ++count[i];
    }
  return SFI_OK;
}

int sfi_set_tuning(sfi_ctx* x, int32_t dense_target_wgs, int32_t fast_tiles_per_wave, int32_t fast_merge) {
  if (x == nullptr || fast_merge > 2) return SFI_EINVAL;
  if (dense_target_wgs != 0) x->dense_target_wgs = dense_target_wgs > 0 ? dense_target_wgs : 0;
  if (fast_tiles_per_wave != 0) x->fast_tiles_per_wave = fast_tiles_per_wave > 0 ? fast_tiles_per_wave : 0;
  if (fast_merge != 0) x->tail_merge = fast_merge != 2;
  return SFI_OK;
}

int sfi_set_mixed_plan(sfi_ctx* x, int32_t on) {
  if (x == nullptr || on < 0 || on > 1) return SFI_EINVAL;
  x->mixed_plan = on;
  return SFI_OK;
}

int sfi_set_dense_k_layout(sfi_ctx* x, int32_t whole_lines) {
  if (x == nullptr || whole_lines < 0 || whole_lines > 1) return SFI_EINVAL;
  x->dense_wide = whole_lines;
  return SFI_OK;
}

int sfi_plan_splits(const sfi_ctx* x, int32_t max_len, int32_t sel_stride, int32_t* dense_splits,
                    int32_t* fast_splits) {
  if (x == nullptr || sel_stride < 0 || sel_stride > x->cfg.max_budget) return SFI_EINVAL;
  int ml;
  const int rc = resolve_max_len(x, max_len, &ml);
  if (rc != SFI_OK) return rc;
  int pipelined;
  if (dense_splits) *dense_splits = dense_splits_for(x, ml, false);
  if (fast_splits) *fast_splits = fast_splits_for(x, sel_stride, &pipelined);
  return SFI_OK;
}

int sfi_device_status(sfi_ctx* x, int32_t* flags, int32_t clear, void* stream) {
  if (x == nullptr || flags == nullptr) return SFI_EINVAL;
  static_assert(kGuardCtxLen == SFI_GUARD_CTX_LEN && kGuardNSel == SFI_GUARD_N_SEL &&
                kGuardSelIdx == SFI_GUARD_SEL_IDX && kGuardBlock == SFI_GUARD_BLOCK, "guard bits");
  hipStream_t st = (hipStream_t)stream;
  int32_t v = 0;
  SFI_TRY(hipMemcpyAsync(&v, x->ws.guard, sizeof(v), hipMemcpyDeviceToHost, st));
  SFI_TRY(hipStreamSynchronize(st));
  if (clear != 0 && v != 0) {
    SFI_TRY(hipMemsetAsync(x->ws.guard, 0, sizeof(v), st));
    SFI_TRY(hipStreamSynchronize(st));
  }
  *flags = v;
  return SFI_OK;
}

int sfi_query_splits(const sfi_ctx* x, int32_t* dense_splits, int32_t* fast_splits) {
  if (x == nullptr) return SFI_EINVAL;
  if (dense_splits) *dense_splits = x->last_dense_splits;
  if (fast_splits) *fast_splits = x->last_fast_splits;
  return SFI_OK;
}

}  // extern "C"
