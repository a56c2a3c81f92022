// Host side of libmdi: the C ABI of include/mdi.h, arena carving, weight
// repacking, per-sample cache bookkeeping and the launch sequences of a first
// visit (prefill) and a later visit (decode step) of a sample (Alg. 1, Alg. 2).
#include <algorithm>
#include <cstdlib>
#include <atomic>
#include <mutex>
#include <new>
#include <vector>

#include "mdi_internal.h"

using namespace mdi;

namespace {

struct LayerPacked {
  const float *ln1_g = nullptr, *ln1_b = nullptr, *ln2_g = nullptr, *ln2_b = nullptr;
  const void *wqkv = nullptr, *wo = nullptr, *wup = nullptr, *wdown = nullptr;
  const float *bqkv = nullptr, *bo = nullptr, *bup = nullptr, *bdown = nullptr;
  char* kv = nullptr;  // this layer's pages: [page][K][2][pt][h]
};

// Walks the arena in a fixed order; with base == nullptr it only measures.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  void* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

}  // namespace

struct mdi_partition {
  mdi_config cfg;
  uint32_t lo, hi, flags;
  int n_local;
  int esz;            // bytes per stored element
  int pt, n_pages, pages_per_seq;
  int Tm;             // longest first visit
  hipStream_t stream;
  std::vector<LayerPacked> layers;
  const void *wte = nullptr, *wpe = nullptr, *lm_head = nullptr;
  const float *lnf_g = nullptr, *lnf_b = nullptr;
  float2* rope = nullptr;
  int32_t* tables = nullptr;
  // decode scratch
  float *xres = nullptr, *q = nullptr, *o = nullptr, *u = nullptr, *part = nullptr, *amax_val = nullptr;
  int* amax_idx = nullptr;
  float* logits = nullptr;       // [V] scratch of the stochastic sampler
  int head_nwg = 0, head_part_floats = 0;   // streaming launch of the output layers (0: per-operation GEMV)
  size_t head_lds = 0;
  // output layers of several samples per pass over the vocabulary matrix (bf16 + RMSNorm heads)
  int hb_nwg = 0; size_t hb_lds = 0;
  tagged_t* hb_cand = nullptr; tagged_t* cand = nullptr; int* herr = nullptr; float* hb_logits = nullptr;
  unsigned* counters = nullptr;  // [H] attention + [1] argmax
  // prefill scratch
  float *p_xres = nullptr, *p_qkv = nullptr, *p_q = nullptr;
  void *p_xn = nullptr, *p_o = nullptr, *p_u = nullptr;
  bf16_t *p_qb = nullptr, *p_kc = nullptr, *p_vt = nullptr;   // operands of the matrix-core attention of a first visit
  int Tp = 0;                                                 // longest first visit rounded up to whole query blocks
  // host bookkeeping
  std::vector<uint32_t> seq_len;
  std::vector<int32_t> host_tables;   // mirror of `tables`, source of the async page-table copies
  std::vector<int32_t> free_pages;
  size_t arena_bytes = 0;
  // persistent single-launch decode step
  bool use_step = false;
  int nwg = 0, G = 1, n_hg = 0, part_floats = 0;
  int group_ctx = 4096;   // context length from which a launch lets G query heads share a pass over the cache
  size_t step_lds = 0;
  std::vector<StepLayer> h_step_layers;
  StepLayer* d_step_layers = nullptr;
  unsigned *bar_flags = nullptr, *tickets = nullptr;
  tagged_t *t_xres = nullptr, *t_q = nullptr, *t_o = nullptr, *t_u = nullptr, *t_part = nullptr, *t_knew = nullptr;
  int* err = nullptr;
  unsigned epoch = 0;
  unsigned long long* trace = nullptr;
  // exchange buffers, flags and phase counter of each message a launch can carry (set 0 aliases the members above)
  struct StepScratch {
    tagged_t *xres = nullptr, *q = nullptr, *o = nullptr, *u = nullptr, *part = nullptr, *knew = nullptr;
    unsigned *flags = nullptr, *tickets = nullptr;
    unsigned epoch = 0;
  } sc[kMaxSlots];
  // decode of several queued messages with one pass over the weights (step_batch.h)
  bool batch_region = false;           // the arena holds the exchange region of that launch (bf16 storage, RMSNorm)
  bool use_batch = false;              // ... and the shape allows the launch on this device
  char* b_slot0 = nullptr; size_t b_stride = 0;
  size_t b_off_q = 0, b_off_part = 0, b_off_knew = 0, b_off_tickets = 0;
  tagged_t *b_xn = nullptr, *b_ob = nullptr, *b_ub = nullptr;   // [pair of columns][kMaxBatch messages]
  size_t b_vec_words = 0;
  tagged_t* b_ssq = nullptr;
  tagged_t* b_ssum = nullptr; float* b_nc = nullptr; size_t b_nc_stride = 0;   // LayerNorm in the batched pass (BatchArgs)
  tagged_t* b_ppart = nullptr; int b_S = 0, b_oct = 0;   // streamed products split among workgroups (plan_batch)
  unsigned* b_flags = nullptr;
  unsigned b_epoch = 0;
  int b_R[4] = {16, 16, 16, 16};
  int batch_group = 0;                 // MDI_BATCH_GROUP: query heads per attention work item of a batched pass (0: chosen per launch)
  int b_lds_xres = 0, b_lds_sq = 0, b_lds_part = 0;
  size_t b_lds = 0;
  int n_cu = 0;
  int device = 0;         // HIP device the partition was created on (index into the per-device launch chain)
};

namespace {

int act_kind(const mdi_config& c) { return c.dtype == MDI_BF16 ? IN_BF16 : IN_F32; }

mdi_status check_config(const mdi_config* c, uint32_t lo, uint32_t hi, uint32_t flags) {
  if (!c || c->abi_version != MDI_ABI_VERSION) return MDI_ERR_ARG;
  if (!c->n_layer || !c->d_model || !c->n_head || !c->n_kv_head || !c->head_dim || !c->d_ff || !c->vocab) return MDI_ERR_ARG;
  if (!c->max_ctx || !c->max_seqs) return MDI_ERR_ARG;
  if (c->d_model % 8 || c->d_ff % 8) return MDI_ERR_ARG;
  const uint32_t h = c->head_dim;
  if (h < 8 || h > 256 || (h & (h - 1))) return MDI_ERR_ARG;   // a token's head vector maps to 2^k lanes
  if (c->n_head % c->n_kv_head) return MDI_ERR_ARG;
  if (c->norm_kind > MDI_NORM_RMSNORM || c->mlp_kind > MDI_MLP_SWIGLU || c->pos_kind > MDI_POS_ROPE) return MDI_ERR_ARG;
  if (c->dtype > MDI_BF16) return MDI_ERR_ARG;
  if (!(c->norm_eps >= 0.f)) return MDI_ERR_ARG;
  if (c->pos_kind == MDI_POS_ROPE && !(c->rope_base > 0.f)) return MDI_ERR_ARG;
  if (c->max_prefill > c->max_ctx) return MDI_ERR_ARG;
  // the decode kernel divides a position by the page size with one multiplication, exact below this bound
  if ((uint64_t)c->max_ctx * (c->kv_page_tokens ? c->kv_page_tokens : 16) >= (1ull << 32)) return MDI_ERR_ARG;
  if (flags & ~(uint32_t)(MDI_HAS_EMBED | MDI_HAS_HEAD)) return MDI_ERR_ARG;
  if (hi > c->n_layer || lo > hi) return MDI_ERR_ARG;
  if (lo == hi && ((flags & MDI_HAS_EMBED) || !(flags & MDI_HAS_HEAD))) return MDI_ERR_ARG;
  if ((flags & MDI_HAS_EMBED) && lo != 0) return MDI_ERR_ARG;  // token ids enter at layer 0 only
  return MDI_OK;
}

// Lays the partition out in the arena.  Called with p->... unset pointers when measuring.
size_t carve(mdi_partition* p, void* arena) {
  const mdi_config& c = p->cfg;
  const size_t B = p->esz, d = c.d_model, H = c.n_head, K = c.n_kv_head, h = c.head_dim, F = c.d_ff, V = c.vocab;
  const bool ln = c.norm_kind == MDI_NORM_LAYERNORM, swiglu = c.mlp_kind == MDI_MLP_SWIGLU;
  const size_t nqkv = (H + 2 * K) * h, nup = swiglu ? 2 * F : F;
  Carver cv(arena);
  p->layers.assign(p->n_local, LayerPacked());
  for (auto& L : p->layers) {
    L.ln1_g = (float*)cv.take(d * 4);
    if (ln) L.ln1_b = (float*)cv.take(d * 4);
    L.wqkv = cv.take(nqkv * d * B);
    if (c.has_bias) L.bqkv = (float*)cv.take(nqkv * 4);
    L.wo = cv.take(d * H * h * B);
    if (c.has_bias) L.bo = (float*)cv.take(d * 4);
    L.ln2_g = (float*)cv.take(d * 4);
    if (ln) L.ln2_b = (float*)cv.take(d * 4);
    L.wup = cv.take(nup * d * B);
    if (c.has_bias && !swiglu) L.bup = (float*)cv.take(F * 4);
    L.wdown = cv.take(d * F * B);
    if (c.has_bias && !swiglu) L.bdown = (float*)cv.take(d * 4);
  }
  const bool embed = p->flags & MDI_HAS_EMBED, head = p->flags & MDI_HAS_HEAD;
  if (embed || (head && c.tie_embed)) p->wte = cv.take(V * d * B);
  if (embed && c.pos_kind == MDI_POS_LEARNED) p->wpe = cv.take((size_t)c.max_ctx * d * B);
  if (head) {
    p->lnf_g = (float*)cv.take(d * 4);
    if (ln) p->lnf_b = (float*)cv.take(d * 4);
    p->lm_head = c.tie_embed ? p->wte : cv.take(V * d * B);
    p->amax_val = (float*)cv.take(1024 * 4);
    p->amax_idx = (int*)cv.take(1024 * 4);
    p->logits = (float*)cv.take(V * 4);
    p->cand = (tagged_t*)cv.take(1024 * 2 * sizeof(tagged_t));
    p->herr = (int*)cv.take(256);
    if (c.dtype == MDI_BF16) {
      p->hb_cand = (tagged_t*)cv.take((size_t)kMaxBatch * 1024 * 2 * sizeof(tagged_t));
      p->hb_logits = (float*)cv.take((size_t)kMaxBatch * V * 4);
    }
  }
  p->counters = (unsigned*)cv.take((H + 2) * 4);
  if (p->n_local) {
    if (c.pos_kind == MDI_POS_ROPE) p->rope = (float2*)cv.take((size_t)c.max_ctx * (h / 2) * sizeof(float2));
    const size_t layer_pool = (size_t)p->n_pages * K * 2 * p->pt * h * B;
    for (auto& L : p->layers) L.kv = (char*)cv.take(layer_pool);
    p->tables = (int32_t*)cv.take((size_t)c.max_seqs * p->pages_per_seq * 4);
    p->xres = (float*)cv.take(d * 4);
    p->q = (float*)cv.take(H * h * 4);
    p->o = (float*)cv.take(H * h * 4);
    p->u = (float*)cv.take(F * 4);
    p->part = (float*)cv.take(H * kMaxSplits * (h + 2) * 4);
    p->d_step_layers = (StepLayer*)cv.take(p->n_local * sizeof(StepLayer));
    p->bar_flags = (unsigned*)cv.take(1024 * 4);
    p->tickets = (unsigned*)cv.take(H * 4);
    p->err = (int*)cv.take(256);
    p->t_xres = (tagged_t*)cv.take(d * 8);
    p->t_q = (tagged_t*)cv.take(H * h * 8);
    p->t_o = (tagged_t*)cv.take(H * h * 8);
    p->t_u = (tagged_t*)cv.take(F * 8);
    p->t_part = (tagged_t*)cv.take(H * kMaxSplits * (h + 2) * 8);
    p->t_knew = (tagged_t*)cv.take(2 * K * h * 8);
    p->sc[0].xres = p->t_xres; p->sc[0].q = p->t_q; p->sc[0].o = p->t_o; p->sc[0].u = p->t_u;
    p->sc[0].part = p->t_part; p->sc[0].knew = p->t_knew; p->sc[0].flags = p->bar_flags; p->sc[0].tickets = p->tickets;
    for (int m = 1; m < kMaxSlots; ++m) {
      auto& sc = p->sc[m];
      sc.flags = (unsigned*)cv.take(1024 * 4);
      sc.tickets = (unsigned*)cv.take(H * 4);
      sc.xres = (tagged_t*)cv.take(d * 8);
      sc.q = (tagged_t*)cv.take(H * h * 8);
      sc.o = (tagged_t*)cv.take(H * h * 8);
      sc.u = (tagged_t*)cv.take(F * 8);
      sc.part = (tagged_t*)cv.take(H * kMaxSplits * (h + 2) * 8);
      sc.knew = (tagged_t*)cv.take(2 * K * h * 8);
    }
    p->batch_region = c.dtype == MDI_BF16;
    if (p->batch_region) {
      // one block per message of a batched launch, all laid out alike, so that message j's vectors are message
      // 0's advanced by j strides
      size_t off = 0;
      auto sub = [&off](size_t bytes) { const size_t at = off; off = (off + bytes + 255) & ~(size_t)255; return at; };
      p->b_off_q = sub(H * h * 8);
      p->b_off_part = sub(H * kMaxSplits * (h + 2) * 8);
      p->b_off_knew = sub(2 * K * h * 8);
      p->b_off_tickets = sub(H * 4);
      p->b_stride = off;
      p->b_slot0 = (char*)cv.take(p->b_stride * kMaxBatch);
      p->b_vec_words = (d / 2 + H * h / 2 + F / 2) * (size_t)kMaxBatch;
      p->b_xn = (tagged_t*)cv.take(p->b_vec_words * 8);
      p->b_ob = p->b_xn ? p->b_xn + d / 2 * kMaxBatch : nullptr;
      p->b_ub = p->b_xn ? p->b_ob + H * h / 2 * kMaxBatch : nullptr;
      p->b_ssq = (tagged_t*)cv.take((size_t)kMaxBatch * 1024 * 8);
      if (ln) {
        p->b_ssum = (tagged_t*)cv.take((size_t)kMaxBatch * 1024 * 8);
        p->b_nc_stride = 2 * (nqkv + nup);
        p->b_nc = (float*)cv.take(p->n_local * p->b_nc_stride * 4);
      }
      p->b_ppart = (tagged_t*)cv.take((size_t)((d + 15) / 16) * 16 * 256 * 8);   // [block][up to 16 slices][256]
      p->b_flags = (unsigned*)cv.take((size_t)1024 * kFlagStride * 4);
    }
    const size_t T = p->Tm;
    p->p_xres = (float*)cv.take(T * d * 4);
    p->p_xn = cv.take(T * d * B);
    p->p_qkv = (float*)cv.take(T * nqkv * 4);
    p->p_q = (float*)cv.take(T * H * h * 4);
    p->p_o = cv.take(T * H * h * B);
    p->p_u = cv.take(T * F * B);
    if (flash_supported(c.dtype, (int)h)) {
      // keys and values^T of every position a first visit in pieces can reach: up to max_ctx, in blocks of 128
      p->Tp = (int)(((size_t)c.max_ctx + 127) / 128 * 128);
      p->p_qb = (bf16_t*)cv.take(T * H * h * 2);
      p->p_kc = (bf16_t*)cv.take((size_t)K * p->Tp * h * 2);
      p->p_vt = (bf16_t*)cv.take((size_t)K * h * p->Tp * 2);
    }
  }
  return (cv.off + 255) & ~(size_t)255;
}

void init_geometry(mdi_partition* p, const mdi_config* cfg, uint32_t lo, uint32_t hi, uint32_t flags) {
  p->cfg = *cfg;
  p->lo = lo; p->hi = hi; p->flags = flags;
  p->n_local = (int)(hi - lo);
  p->esz = cfg->dtype == MDI_BF16 ? 2 : 4;
  p->pt = cfg->kv_page_tokens ? (int)cfg->kv_page_tokens : 16;
  p->pages_per_seq = ((int)cfg->max_ctx + p->pt - 1) / p->pt;
  p->n_pages = cfg->kv_pages ? (int)cfg->kv_pages : (int)cfg->max_seqs * p->pages_per_seq;
  p->Tm = cfg->max_prefill ? (int)cfg->max_prefill : (int)cfg->max_ctx;
}

// Decides whether a decode step runs as one persistent launch and sizes its LDS.
void plan_step(mdi_partition* p, int n_cu) {
  const mdi_config& c = p->cfg;
  p->use_step = false;
  if (c.decode_path == 1 || !p->n_local || n_cu <= 0) return;
  const int H = c.n_head, K = c.n_kv_head, h = c.head_dim, d = c.d_model, F = c.d_ff;
  const int group = H / K;
  // Query heads that take one pass over their kv head's cache together.  Measured (heads of 128, groups of 4 and 8):
  // sharing the pass among a whole group leaves few, long work items (one per kv head and context split) with many
  // partials to fold, and loses to one head per item, whose repeated cache reads hit in L2 / the memory-side cache;
  // pairs of heads win once the cache is long (step_group picks per launch).  LDS is sized for pairs.
  p->G = group % 2 == 0 ? 2 : 1;
  p->group_ctx = 4096;
  if (const char* e = getenv("MDI_GROUP_CTX")) p->group_ctx = std::max(0, atoi(e));   // tuning / test knob, see mdi.h
  if (const char* e = getenv("MDI_BATCH_GROUP")) { const int v = atoi(e); p->batch_group = (v == 1 || v == 2 || v == 4) ? v : 0; }
  p->n_hg = H;                           // the most head groups a launch has (one head each)
  p->nwg = std::min(n_cu, 1024);
  if (p->n_hg > p->nwg) return;
  const int nup = c.mlp_kind == MDI_MLP_SWIGLU ? 2 * F : F;
  const int max_rows = std::max(std::max((H + 2 * K) * h, nup), d);
  const int max_pairs = ((max_rows + 1) / 2 + p->nwg - 1) / p->nwg + 1;
  p->part_floats = (max_pairs * 2 * kStepWavesMax + 3) & ~3;
  int xs = std::max(std::max(d, H * h), F);
  xs = (xs + 511) / 512 * 512;         // the kernel keeps zeros behind a vector up to a whole 64-lane chunk (64 x 8 values)
  xs = std::max(xs, kStepWavesMax * p->G * (h + 2));
  xs = (xs + 3) & ~3;
  p->step_lds = (size_t)(128 + p->part_floats + xs) * sizeof(float);
  if (p->step_lds > 64 * 1024) return;
  p->use_step = true;
}

// Decides whether several queued messages can share one pass over the weights (step_batch.h) and lays out its LDS.
void plan_batch(mdi_partition* p) {
  const mdi_config& c = p->cfg;
  p->use_batch = false;
  if (!p->use_step || !p->batch_region) return;
  const int H = c.n_head, K = c.n_kv_head, h = c.head_dim, d = c.d_model, F = c.d_ff, nwg = p->nwg;
  if (d % 32 || (H * h) % 32 || F % 32) return;                 // a column step of the matrix instruction is 32 wide
  if (((d / 32 + kStepWavesMax - 1) / kStepWavesMax) > 16) return;   // a wavefront keeps its slice of a d-sized vector in registers
  const int nup = c.mlp_kind == MDI_MLP_SWIGLU ? 2 * F : F;
  const int rows[4] = {(H + 2 * K) * h, d, nup, d};
  int nb_max = 1, nb_d = 1;
  for (int j = 0; j < 4; ++j) {
    // 16 rows per block when that gives every workgroup a block, else 8 (twice the blocks to spread).  Measured on
    // the 7B shape's gate/up product (1376 blocks of 16 over 256 workgroups: 5 or 6 each): blocks of 8 balance better
    // (10 or 11 each) but every load and matrix instruction then carries half the rows, and the phase took twice as long.
    int R = (rows[j] + 15) / 16 >= nwg ? 16 : 8;
    if (j == 0 && (h / 2) % (R / 2)) R = 8;                      // a block holds R/2 rows of a half head and their partners
    if (j == 0 && (h / 2) % (R / 2)) return;
    if (j == 2 && c.mlp_kind == MDI_MLP_SWIGLU && rows[j] % 4) return;
    p->b_R[j] = R;
    const int nb = ((rows[j] + R - 1) / R + nwg - 1) / nwg;
    nb_max = std::max(nb_max, nb);
    if (j == 1) nb_d = nb;
  }
  // The two residual products (output projection, MLP down) split their inner dimension among workgroups: groups
  // of S workgroups share eight 16-row blocks, one block per wavefront, one column slice per workgroup; the owner
  // of a block (workgroup = block index) adds the S partial results.
  int ks_floats = 0;
  {
    const int nblk = (d + 15) / 16, octets = (nblk + kStepWavesMax - 1) / kStepWavesMax;
    if (nblk > nwg) return;
    const int S = std::min(16, nwg / octets);
    const int c_max = (std::max(H * h, F) / 32 + S - 1) / S;     // column steps of the longest slice: 1 KiB of LDS each
    p->b_S = S; p->b_oct = octets;
    p->b_R[1] = p->b_R[3] = 16;
    nb_d = 1;
    ks_floats = S * 256 + c_max * 256;
  }
  p->b_lds_xres = 128;
  p->b_lds_sq = p->b_lds_xres + nb_d * 256;
  p->b_lds_part = p->b_lds_sq + std::max(nb_d * 128, 128);
  const int Gmax = (H / K) % 4 == 0 ? 4 : p->G;
  const int attn_floats = std::max(Gmax * h, kStepWavesMax * Gmax * (h + 2)) + 64;
  const int part_floats = std::max(std::max(nb_max * 2048, attn_floats), ks_floats);
  p->b_lds = (size_t)(p->b_lds_part + part_floats) * sizeof(float);
  if (p->b_lds > 160 * 1024) return;
  if (p->b_lds > 64 * 1024 && !step_batch_allow_lds(p->b_lds)) return;
  p->use_batch = true;
}

// The one piece of state that partitions share (see mdi.h, "Process-wide state").  A persistent launch needs
// every one of its workgroups resident at once; two such launches dispatched side by side from different
// streams could each be given a part of the compute units and wait for the rest for ever (their bounded
// waits would turn that into MDI_ERR_HIP).  So, per device, an event orders a partition's persistent launch
// after the previous one of any other partition.
constexpr int kMaxDevices = 64;
struct LaunchChain {
  std::mutex mutex;
  hipEvent_t event = nullptr;
  hipStream_t stream = nullptr;       // the stream of the launch `event` was recorded after
};
LaunchChain g_chain[kMaxDevices];

template <typename Launch>
mdi_status launch_step_serialised(mdi_partition* p, Launch&& launch) {
  LaunchChain& ch = g_chain[p->device];
  std::lock_guard<std::mutex> lock(ch.mutex);
  if (!ch.event) {
    if (hipEventCreateWithFlags(&ch.event, hipEventDisableTiming) != hipSuccess) return MDI_ERR_HIP;
  } else if (ch.stream != p->stream) {
    if (hipStreamWaitEvent(p->stream, ch.event, 0) != hipSuccess) return MDI_ERR_HIP;
  }
  launch();
  if (hipEventRecord(ch.event, p->stream) != hipSuccess) return MDI_ERR_HIP;
  ch.stream = p->stream;
  return MDI_OK;
}

// Scratch of mdi_sample_topk_static, the entry point for callers that cannot allocate: a [V] float logits buffer
// for vocabularies up to kStaticVocabMax, the per-workgroup argmax candidates (plain for the per-operation kernel,
// tagged for the streaming one), the arrival counter and an error word.  One copy
// per GPU, held until the process ends; its device address is taken once per device and kept.
constexpr size_t kStaticVocabMax = 262144;
constexpr size_t kStaticCand = 1024;                       // workgroups of the output-layer launch, at most
constexpr size_t kStaticLogitsOff = 0;
constexpr size_t kStaticValOff = kStaticVocabMax * 4;
constexpr size_t kStaticIdxOff = kStaticValOff + kStaticCand * 4;
constexpr size_t kStaticCandOff = kStaticIdxOff + kStaticCand * 4;        // tagged candidates of the streaming launch
constexpr size_t kStaticCounterOff = kStaticCandOff + kStaticCand * 2 * sizeof(tagged_t);
constexpr size_t kStaticErrOff = kStaticCounterOff + 128;
constexpr size_t kStaticScratchBytes = kStaticCounterOff + 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];                 // device address of `scratch` on each GPU (nullptr: not taken yet)

// `device` must be the current device: the symbol's address is that of the current device's copy.
mdi_status static_scratch(int device, unsigned char** out) {
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) return MDI_ERR_HIP;
    if (cur != device) return MDI_ERR_STATE;
    unsigned char* ptr = nullptr;
    if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MDI_ERR_HIP;
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return MDI_OK;
}

// device-to-device copy of a [rows, cols] matrix into rows r*mul + off of dst
void put_rows(mdi_partition* p, const void* src, const void* dst, size_t rows, size_t cols, int esz, long mul = 1, long off = 0) {
  if (!src || !dst) return;
  launch_copy_rows(p->stream, esz, src, const_cast<void*>(dst), (long)rows, (long)cols, mul, off);
}

mdi_status hip_status() { return hipGetLastError() == hipSuccess ? MDI_OK : MDI_ERR_HIP; }

}  // namespace

extern "C" {

mdi_status mdi_partition_bytes(const mdi_config* cfg, uint32_t layer_lo, uint32_t layer_hi, uint32_t flags, size_t* arena_bytes) {
  if (!arena_bytes) return MDI_ERR_ARG;
  const mdi_status st = check_config(cfg, layer_lo, layer_hi, flags);
  if (st != MDI_OK) return st;
  mdi_partition tmp;
  init_geometry(&tmp, cfg, layer_lo, layer_hi, flags);
  *arena_bytes = carve(&tmp, nullptr);
  return MDI_OK;
}

mdi_status mdi_partition_create(const mdi_config* cfg, uint32_t layer_lo, uint32_t layer_hi, const mdi_weights* w,
                                uint32_t flags, void* arena, size_t arena_bytes, void* hip_stream, mdi_partition** out) {
  if (!out) return MDI_ERR_ARG;
  *out = nullptr;
  mdi_status st = check_config(cfg, layer_lo, layer_hi, flags);
  if (st != MDI_OK) return st;
  if (!w || !arena || ((uintptr_t)arena & 255)) return MDI_ERR_ARG;
  const bool embed = flags & MDI_HAS_EMBED, head = flags & MDI_HAS_HEAD;
  const bool ln = cfg->norm_kind == MDI_NORM_LAYERNORM, swiglu = cfg->mlp_kind == MDI_MLP_SWIGLU;
  if (layer_hi > layer_lo && !w->layers) return MDI_ERR_ARG;
  if ((embed || (head && cfg->tie_embed)) && !w->wte) return MDI_ERR_ARG;
  if (embed && cfg->pos_kind == MDI_POS_LEARNED && !w->wpe) return MDI_ERR_ARG;
  if (head && (!w->lnf_g || (!cfg->tie_embed && !w->lm_head))) return MDI_ERR_ARG;
  for (uint32_t i = 0; i < layer_hi - layer_lo; ++i) {
    const mdi_layer_weights& s = w->layers[i];
    if (!s.ln1_g || !s.ln2_g || !s.wq || !s.wk || !s.wv || !s.wo || !s.w_up || !s.w_down) return MDI_ERR_ARG;
    if (swiglu && !s.w_gate) return MDI_ERR_ARG;
    if (swiglu && (s.b_up || s.b_down)) return MDI_ERR_ARG;   // a SwiGLU MLP carries no biases here: refuse rather than drop them
  }
  mdi_partition* p = new (std::nothrow) mdi_partition();
  if (!p) return MDI_ERR_NOMEM;
  init_geometry(p, cfg, layer_lo, layer_hi, flags);
  p->stream = (hipStream_t)hip_stream;
  const size_t need = carve(p, arena);
  if (need > arena_bytes) { delete p; return MDI_ERR_NOMEM; }
  p->arena_bytes = arena_bytes;

  const mdi_config& c = p->cfg;
  const size_t d = c.d_model, H = c.n_head, K = c.n_kv_head, h = c.head_dim, F = c.d_ff, V = c.vocab;
  const int B = p->esz;
  for (int i = 0; i < p->n_local; ++i) {
    const mdi_layer_weights& s = w->layers[i];
    LayerPacked& L = p->layers[i];
    put_rows(p, s.ln1_g, L.ln1_g, 1, d, 4);
    put_rows(p, s.ln2_g, L.ln2_g, 1, d, 4);
    if (ln) {
      if (s.ln1_b) put_rows(p, s.ln1_b, L.ln1_b, 1, d, 4); else launch_fill_f32(p->stream, (float*)L.ln1_b, d, 0.f);
      if (s.ln2_b) put_rows(p, s.ln2_b, L.ln2_b, 1, d, 4); else launch_fill_f32(p->stream, (float*)L.ln2_b, d, 0.f);
    }
    // fused QKV matrix: query rows, then key rows, then value rows
    char* wqkv = (char*)L.wqkv;
    put_rows(p, s.wq, wqkv, H * h, d, B);
    put_rows(p, s.wk, wqkv + H * h * d * B, K * h, d, B);
    put_rows(p, s.wv, wqkv + (H + K) * h * d * B, K * h, d, B);
    put_rows(p, s.wo, L.wo, d, H * h, B);
    if (swiglu) {   // gate and up rows interleaved: row 2f = gate_f, row 2f+1 = up_f
      put_rows(p, s.w_gate, L.wup, F, d, B, 2, 0);
      put_rows(p, s.w_up, L.wup, F, d, B, 2, 1);
    } else {
      put_rows(p, s.w_up, L.wup, F, d, B);
    }
    put_rows(p, s.w_down, L.wdown, d, F, B);
    if (c.has_bias) {
      float* bq = (float*)L.bqkv;
      launch_fill_f32(p->stream, bq, (H + 2 * K) * h, 0.f);
      put_rows(p, s.bq, bq, 1, H * h, 4);
      put_rows(p, s.bk, bq + H * h, 1, K * h, 4);
      put_rows(p, s.bv, bq + (H + K) * h, 1, K * h, 4);
      launch_fill_f32(p->stream, (float*)L.bo, d, 0.f);
      put_rows(p, s.bo, L.bo, 1, d, 4);
      if (!swiglu) {
        launch_fill_f32(p->stream, (float*)L.bup, F, 0.f);
        put_rows(p, s.b_up, L.bup, 1, F, 4);
        launch_fill_f32(p->stream, (float*)L.bdown, d, 0.f);
        put_rows(p, s.b_down, L.bdown, 1, d, 4);
      }
    }
  }
  if (p->wte) put_rows(p, w->wte, p->wte, V, d, B);
  if (p->wpe) put_rows(p, w->wpe, p->wpe, c.max_ctx, d, B);
  if (head) {
    put_rows(p, w->lnf_g, p->lnf_g, 1, d, 4);
    if (ln) { if (w->lnf_b) put_rows(p, w->lnf_b, p->lnf_b, 1, d, 4); else launch_fill_f32(p->stream, (float*)p->lnf_b, d, 0.f); }
    if (!c.tie_embed) put_rows(p, w->lm_head, p->lm_head, V, d, B);
  }
  launch_fill_u32(p->stream, p->counters, H + 2, 0u);
  if (p->cand) {
    launch_fill_u32(p->stream, (uint32_t*)p->cand, 1024 * 4, 0u);                          // tag 0 = no call's
    launch_fill_u32(p->stream, (uint32_t*)p->herr, 64, 0u);
  }
  if (p->hb_cand) launch_fill_u32(p->stream, (uint32_t*)p->hb_cand, (long)kMaxBatch * 1024 * 4, 0u);
  if (p->rope) launch_rope_table(p->stream, p->rope, (int)c.max_ctx, (int)h, (double)c.rope_base);

  if (p->n_local) {
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n_cu = 0;
    if (dev < 0 || dev >= kMaxDevices) { delete p; return MDI_ERR_ARG; }
    p->n_cu = n_cu;
    p->device = dev;
    plan_step(p, n_cu);
    plan_batch(p);
    if (p->batch_region) {
      launch_fill_u32(p->stream, (uint32_t*)p->b_slot0, (long)(p->b_stride * kMaxBatch / 4), 0u);
      launch_fill_u32(p->stream, (uint32_t*)p->b_xn, (long)p->b_vec_words * 2, 0u);
      launch_fill_u32(p->stream, (uint32_t*)p->b_ssq, (long)kMaxBatch * 1024 * 2, 0u);
      if (p->b_ssum) {
        launch_fill_u32(p->stream, (uint32_t*)p->b_ssum, (long)kMaxBatch * 1024 * 2, 0u);
        const int nq = (int)((H + 2 * K) * h), nu = (int)(c.mlp_kind == MDI_MLP_SWIGLU ? 2 * F : F);
        for (int i = 0; i < p->n_local; ++i) {       // what the mean and the norm's bias add to the two normed products
          const LayerPacked& L = p->layers[i];
          float* nc = p->b_nc + (size_t)i * p->b_nc_stride;
          launch_row_dots(p->stream, L.wqkv, nq, (int)d, L.ln1_g, L.ln1_b, nc, nc + nq);
          launch_row_dots(p->stream, L.wup, nu, (int)d, L.ln2_g, L.ln2_b, nc + 2 * nq, nc + 2 * nq + nu);
        }
      }
      launch_fill_u32(p->stream, (uint32_t*)p->b_ppart, (long)((d + 15) / 16) * 16 * 256 * 2, 0u);
      launch_fill_u32(p->stream, p->b_flags, 1024L * kFlagStride, 1u);
      p->b_epoch = 1;
    }
    launch_fill_u32(p->stream, p->bar_flags, 1024, 1u);     // phase counters start at 1: tag 0 marks "never written"
    p->epoch = 1;
    launch_fill_u32(p->stream, (uint32_t*)p->t_xres, 2 * d, 0u);
    launch_fill_u32(p->stream, (uint32_t*)p->t_q, 2 * H * h, 0u);
    launch_fill_u32(p->stream, (uint32_t*)p->t_o, 2 * H * h, 0u);
    launch_fill_u32(p->stream, (uint32_t*)p->t_u, 2 * F, 0u);
    launch_fill_u32(p->stream, (uint32_t*)p->t_part, 2 * H * kMaxSplits * (h + 2), 0u);
    launch_fill_u32(p->stream, (uint32_t*)p->t_knew, 4 * K * h, 0u);
    launch_fill_u32(p->stream, p->tickets, H, 0u);
    for (int m = 1; m < kMaxSlots; ++m) {
      auto& sc = p->sc[m];
      launch_fill_u32(p->stream, sc.flags, 1024, 1u);
      sc.epoch = 1;
      launch_fill_u32(p->stream, (uint32_t*)sc.xres, 2 * d, 0u);
      launch_fill_u32(p->stream, (uint32_t*)sc.q, 2 * H * h, 0u);
      launch_fill_u32(p->stream, (uint32_t*)sc.o, 2 * H * h, 0u);
      launch_fill_u32(p->stream, (uint32_t*)sc.u, 2 * F, 0u);
      launch_fill_u32(p->stream, (uint32_t*)sc.part, 2 * H * kMaxSplits * (h + 2), 0u);
      launch_fill_u32(p->stream, (uint32_t*)sc.knew, 4 * K * h, 0u);
      launch_fill_u32(p->stream, sc.tickets, H, 0u);
    }
    launch_fill_u32(p->stream, (uint32_t*)p->err, 64, 0u);
    p->h_step_layers.resize(p->n_local);
    for (int i = 0; i < p->n_local; ++i) {
      const LayerPacked& L = p->layers[i];
      p->h_step_layers[i] = StepLayer{L.wqkv, L.wo, L.wup, L.wdown, L.bqkv, L.bo, L.bup, L.bdown,
                                      L.ln1_g, L.ln1_b, L.ln2_g, L.ln2_b, L.kv};
    }
    if (hipMemcpyAsync(p->d_step_layers, p->h_step_layers.data(), p->n_local * sizeof(StepLayer), hipMemcpyHostToDevice, p->stream) != hipSuccess) {
      delete p;
      return MDI_ERR_HIP;
    }
  }
  if (head) {
    // the static scratch of mdi_sample_topk_static: its address on this device is taken here, once, so that the
    // entry point itself only reads it
    int dev = 0;
    unsigned char* unused = nullptr;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { delete p; return MDI_ERR_HIP; }
    p->device = dev;
    const mdi_status sst = static_scratch(dev, &unused);
    if (sst != MDI_OK) { delete p; return sst; }
  }
  if (head && c.decode_path != 1) {
    // the output layers as one streaming launch when the activation and the pair partials fit in LDS
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n_cu = 0;
    if (n_cu > 0) {
      const int nwg = std::min(n_cu, 1024);
      const int max_pairs = (((int)V + 1) / 2 + nwg - 1) / nwg + 8;
      const int part_floats = (max_pairs * 2 * kStepWavesMax + 3) & ~3;
      const size_t lds = (size_t)(128 + part_floats + ((d + 3) & ~(size_t)3)) * sizeof(float);
      if (lds <= 64 * 1024) { p->head_nwg = nwg; p->head_part_floats = part_floats; p->head_lds = lds; }
      // several samples per pass: all normalised activations in LDS as bf16 ([d / 8][16] units of 16 bytes)
      const size_t hb_lds = (size_t)d * kMaxBatch * 2;
      if (p->hb_cand && d % 32 == 0 && (uint64_t)V * d * 2 < (1ull << 32) && hb_lds <= 144 * 1024 &&
          (hb_lds <= 60 * 1024 || logits_batch_allow_lds(hb_lds))) {
        p->hb_nwg = nwg; p->hb_lds = hb_lds;
      }
    }
  }
  p->seq_len.assign(c.max_seqs, 0u);
  if (p->n_local) {
    p->host_tables.assign((size_t)c.max_seqs * p->pages_per_seq, 0);
    launch_fill_u32(p->stream, (uint32_t*)p->tables, (long)p->host_tables.size(), 0u);
    p->free_pages.resize(p->n_pages);
    for (int i = 0; i < p->n_pages; ++i) p->free_pages[i] = p->n_pages - 1 - i;   // page 0 is handed out first
  }
  st = hip_status();
  if (st != MDI_OK) { delete p; return st; }
  *out = p;
  return MDI_OK;
}

namespace {

// Forwards T positions of sample seq, starting at position pos0 = its current cache length (0: a first visit).
mdi_status prefill_rows(mdi_partition* p, uint32_t seq, const void* acts_in, uint32_t T, void* acts_out) {
  const mdi_config& c = p->cfg;
  const int pos0 = (int)p->seq_len[seq];
  if ((uint32_t)pos0 + T > c.max_ctx) return MDI_ERR_CTX;
  if (T > (uint32_t)p->Tm) return MDI_ERR_ARG;
  const int have = (pos0 + p->pt - 1) / p->pt;
  const int need = (pos0 + (int)T + p->pt - 1) / p->pt - have;
  if ((int)p->free_pages.size() < need) return MDI_ERR_NOMEM;
  int32_t* row = p->host_tables.data() + (size_t)seq * p->pages_per_seq;
  for (int i = 0; i < need; ++i) { row[have + i] = p->free_pages.back(); p->free_pages.pop_back(); }
  int32_t* drow = p->tables + (size_t)seq * p->pages_per_seq;
  if (need && hipMemcpyAsync(drow + have, row + have, (size_t)need * 4, hipMemcpyHostToDevice, p->stream) != hipSuccess) return MDI_ERR_HIP;

  hipStream_t s = p->stream;
  const int d = c.d_model, H = c.n_head, K = c.n_kv_head, h = c.head_dim, F = c.d_ff;
  const int ak = act_kind(c);
  const bool embed = p->flags & MDI_HAS_EMBED, swiglu = c.mlp_kind == MDI_MLP_SWIGLU;
  RowsInArgs ri{acts_in, embed ? IN_TOKEN : ak, p->wte, p->wpe, (int)c.dtype, (int)T, d, p->p_xres, (int)c.vocab, p->err, pos0};
  launch_rows_input(s, ri);
  for (int i = 0; i < p->n_local; ++i) {
    const LayerPacked& L = p->layers[i];
    NormRowsArgs n1{p->p_xres, (int)T, d, (int)c.norm_kind, L.ln1_g, L.ln1_b, c.norm_eps, p->p_xn, ak};
    launch_norm_rows(s, n1);
    GemmArgs g1{p->p_xn, L.wqkv, L.bqkv, (int)T, (H + 2 * K) * h, d, p->p_qkv, nullptr};
    launch_gemm(s, c.dtype, GEPI_F32_BIAS, g1);
    // Attention on the matrix cores over operand arrays that hold the keys and the transposed values of positions
    // 0 .. pos0 + T - 1: the new ones written by the scatter and the transpose below, the earlier ones (a later piece
    // of a first visit) brought from the cache pages first.  The arrays are packed to what this call needs.
    const bool flash = p->p_qb != nullptr;
    const int Tp = ((int)T + 127) / 128 * 128;
    const int Tk = (pos0 + (int)T + 127) / 128 * 128;      // keys, padded; at most p->Tp
    const float scale = 1.f / sqrtf((float)h);
    if (flash && pos0) launch_cache_gather(s, L.kv, drow, pos0, K, h, p->pt, Tk, p->p_kc, p->p_vt);
    RopeScatterArgs rs{p->p_qkv, (int)T, H, K, h, p->pt, p->rope, flash ? nullptr : p->p_q, L.kv, drow, (int)c.dtype,
                       flash ? p->p_qb : nullptr, flash ? p->p_kc : nullptr, Tk, Tk - pos0, scale, pos0};
    launch_rope_scatter(s, rs);
    if (flash) {
      launch_v_transpose(s, p->p_qkv, (int)T, Tk - pos0, pos0, Tk, H, K, h, p->p_vt);
      FlashArgs fa{p->p_qb, p->p_kc, p->p_vt, (bf16_t*)p->p_o, (int)T, Tp, H, K, h, pos0, Tk, Tk};
      launch_flash_prefill(s, fa);
    } else {
      AttnArgs at{};
      at.q = p->p_q; at.q_stride = (long)H * h; at.pool = L.kv; at.table = drow;
      at.ctx0 = pos0 + 1; at.n_q = (int)T; at.H = H; at.K = K; at.h = h; at.pt = p->pt;
      at.chunk = (int)c.max_ctx; at.n_splits = 1; at.scale = scale;
      at.part = p->part; at.counters = p->counters; at.out = p->p_o; at.out_stride = (long)H * h; at.out_kind = ak;
      launch_attn(s, c.dtype, at);
    }
    GemmArgs g2{p->p_o, L.wo, L.bo, (int)T, d, H * h, p->p_xres, nullptr};
    launch_gemm(s, c.dtype, GEPI_RESID, g2);
    NormRowsArgs n2{p->p_xres, (int)T, d, (int)c.norm_kind, L.ln2_g, L.ln2_b, c.norm_eps, p->p_xn, ak};
    launch_norm_rows(s, n2);
    GemmArgs g3{p->p_xn, L.wup, L.bup, (int)T, swiglu ? 2 * F : F, d, nullptr, p->p_u};
    launch_gemm(s, c.dtype, swiglu ? GEPI_SWIGLU : (c.mlp_kind == MDI_MLP_GELU_TANH ? GEPI_GELU_TANH : GEPI_GELU_ERF), g3);
    GemmArgs g4{p->p_u, L.wdown, L.bdown, (int)T, d, F, p->p_xres, i == p->n_local - 1 ? acts_out : nullptr};
    launch_gemm(s, c.dtype, GEPI_RESID, g4);
  }
  p->seq_len[seq] = (uint32_t)pos0 + T;
  return hip_status();
}

}  // namespace

mdi_status mdi_prefill(mdi_partition* p, uint32_t seq, const void* acts_in, uint32_t T, void* acts_out) {
  if (!p || !acts_in || !acts_out || !p->n_local) return MDI_ERR_ARG;
  if (seq >= p->cfg.max_seqs || T == 0) return MDI_ERR_ARG;
  if (p->seq_len[seq]) return MDI_ERR_STATE;
  return prefill_rows(p, seq, acts_in, T, acts_out);
}

mdi_status mdi_prefill_chunk(mdi_partition* p, uint32_t seq, const void* acts_in, uint32_t T, void* acts_out) {
  if (!p || !acts_in || !acts_out || !p->n_local) return MDI_ERR_ARG;
  if (seq >= p->cfg.max_seqs || T == 0) return MDI_ERR_ARG;
  return prefill_rows(p, seq, acts_in, T, acts_out);
}

namespace {

// Host bookkeeping of one decode message: the page and slot of the new position.
struct MessagePlan {
  int len, ctx, page, slot;
  int32_t* drow;        // the sequence's page table on the device
  int32_t* new_entry;   // table entry the launch has to fill (a page starts), or nullptr
};

mdi_status check_message(const mdi_partition* p, uint32_t seq) {
  const mdi_config& c = p->cfg;
  if (seq >= c.max_seqs) return MDI_ERR_ARG;
  const uint32_t len = p->seq_len[seq];
  if (!len) return MDI_ERR_STATE;
  if (len + 1 > c.max_ctx) return MDI_ERR_CTX;
  return MDI_OK;
}

mdi_status plan_message(mdi_partition* p, uint32_t seq, MessagePlan* m) {
  const mdi_status st = check_message(p, seq);
  if (st != MDI_OK) return st;
  m->len = (int)p->seq_len[seq];
  m->ctx = m->len + 1;
  int32_t* row = p->host_tables.data() + (size_t)seq * p->pages_per_seq;
  m->drow = p->tables + (size_t)seq * p->pages_per_seq;
  const int pidx = m->len / p->pt;
  m->slot = m->len % p->pt;
  m->new_entry = nullptr;
  if (m->slot == 0) {
    if (p->free_pages.empty()) return MDI_ERR_NOMEM;
    row[pidx] = p->free_pages.back();
    p->free_pages.pop_back();
    m->new_entry = m->drow + pidx;
  }
  m->page = row[pidx];
  return MDI_OK;
}

// Query heads per attention work item for a launch whose longest context is ctx (see plan_step).
int step_group(const mdi_partition* p, int ctx) { return ctx >= p->group_ctx ? p->G : 1; }

// Arguments of the persistent step kernel that do not depend on the message; G = query heads per attention work item.
void fill_step_shared(const mdi_partition* p, int G, StepArgs* a) {
  const mdi_config& c = p->cfg;
  a->l0 = p->h_step_layers[0];
  a->w_stride = p->n_local > 1 ? (const char*)p->h_step_layers[1].wqkv - (const char*)p->h_step_layers[0].wqkv : 0;
  a->kv_stride = p->n_local > 1 ? (const char*)p->h_step_layers[1].kv - (const char*)p->h_step_layers[0].kv : 0;
  a->n_layer = p->n_local;
  a->d = c.d_model; a->H = c.n_head; a->K = c.n_kv_head; a->h = c.head_dim; a->F = c.d_ff; a->pt = p->pt;
  a->pt_h = (long)p->pt * c.head_dim;
  a->norm_kind = c.norm_kind; a->mlp_kind = c.mlp_kind; a->eps = c.norm_eps;
  a->wte = p->wte; a->wpe = p->wpe; a->vocab = (int)c.vocab;
  a->err = p->err; a->spin_limit = 1 << 21;
  a->n_hg = (int)c.n_head / G;
  a->scale = 1.f / sqrtf((float)c.head_dim);
  a->act_kind = act_kind(c);
  a->part_floats = p->part_floats;
}

// One message's part of the arguments: message m of a launch whose sets have nwg workgroups each.
void fill_step_slot(const mdi_partition* p, int m, int nwg, int n_hg, const MessagePlan& mp, const void* act_in, void* act_out, StepSlot* s) {
  const mdi_config& c = p->cfg;
  const int h = c.head_dim, K = c.n_kv_head;
  const long pt_h = (long)p->pt * h;
  s->in = act_in; s->in_kind = (p->flags & MDI_HAS_EMBED) ? IN_TOKEN : act_kind(c);
  s->pos = mp.len; s->ctx = mp.ctx;
  s->rope = p->rope ? p->rope + (size_t)mp.len * (h / 2) : nullptr;
  s->table = mp.drow; s->table_entry = mp.new_entry; s->new_page = mp.page;
  s->kv_tok_off = (long)mp.page * K * 2 * pt_h + (long)mp.slot * h;
  const auto& sc = p->sc[m];
  s->xres = sc.xres; s->q = sc.q; s->o = sc.o; s->u = sc.u; s->part = sc.part; s->knew = sc.knew;
  s->tickets = sc.tickets; s->flags = sc.flags; s->epoch0 = m == 0 ? p->epoch : sc.epoch;
  // context splits: as many as there are workgroups per head group, but no split shorter than 128 positions -
  // the partials of a head group are folded by one workgroup, eight at a time, and every eight cost a round trip
  const int max_splits = std::max(1, std::min(kMaxSplits, nwg / n_hg));
  int chunk = std::max((mp.ctx + max_splits - 1) / max_splits, 128);
  chunk = (chunk + 15) / 16 * 16;
  s->chunk = chunk; s->n_splits = (mp.ctx + chunk - 1) / chunk;
  s->act_out = act_out;
  s->trace = nullptr;
}

// Launches the persistent kernel for n <= kMaxSlots planned messages.
mdi_status launch_messages(mdi_partition* p, int n, const uint32_t* seqs, const MessagePlan* mp, const void* const* ins, void* const* outs) {
  StepArgs a{};
  int ctx = 0;
  for (int m = 0; m < n; ++m) ctx = std::max(ctx, mp[m].ctx);
  const int G = step_group(p, ctx);
  fill_step_shared(p, G, &a);
  a.n_slots = n;
  a.n_sets = n >= 2 ? 2 : 1;             // two sets of 4-wavefront workgroups share the compute units
  a.nwg = p->nwg;
  a.set_lo[0] = 0; a.set_lo[1] = a.n_sets == 2 ? (n + 1) / 2 : n; a.set_lo[2] = n;
  for (int m = 0; m < n; ++m) fill_step_slot(p, m, a.nwg, a.n_hg, mp[m], ins[m], outs[m], &a.s[m]);
  if (p->trace) {                      // timeline of the first message of each set (of the first two messages with one set)
    const int second = a.n_sets == 2 ? a.set_lo[1] : 1;
    a.s[0].trace = p->trace;
    if (second < n) a.s[second].trace = p->trace + (size_t)a.nwg * p->n_local * 40;
  }
  const mdi_status st = launch_step_serialised(p, [&]() {
    if (n == 1) launch_step_w8(p->stream, p->cfg.dtype, G, a.nwg, p->step_lds, a);
    else launch_step_w4(p->stream, p->cfg.dtype, G, a.nwg, p->step_lds, a);
  });
  if (st != MDI_OK) return st;
  p->epoch += 5u * (unsigned)p->n_local;
  for (int m = 1; m < n; ++m) p->sc[m].epoch += 5u * (unsigned)p->n_local;
  for (int m = 0; m < n; ++m) p->seq_len[seqs[m]] = (uint32_t)mp[m].ctx;
  return MDI_OK;
}

}  // namespace

mdi_status mdi_decode_step(mdi_partition* p, uint32_t seq, const void* act_in, void* act_out) {
  if (!p || !act_in || !act_out || !p->n_local) return MDI_ERR_ARG;
  const mdi_config& c = p->cfg;
  MessagePlan mp;
  const mdi_status pst = plan_message(p, seq, &mp);
  if (pst != MDI_OK) return pst;
  const int len = mp.len, ctx = mp.ctx, page = mp.page, slot = mp.slot;
  int32_t* drow = mp.drow;
  int32_t* new_entry = mp.new_entry;

  hipStream_t s = p->stream;
  const int d = c.d_model, H = c.n_head, K = c.n_kv_head, h = c.head_dim, F = c.d_ff;
  const int ak = act_kind(c);
  const bool embed = p->flags & MDI_HAS_EMBED, swiglu = c.mlp_kind == MDI_MLP_SWIGLU;
  if (p->use_step) {
    const mdi_status st = launch_messages(p, 1, &seq, &mp, &act_in, &act_out);
    return st != MDI_OK ? st : hip_status();
  }
  InputArgs ia{act_in, embed ? IN_TOKEN : ak, p->wte, p->wpe, (int)c.dtype, len, d, p->xres, new_entry, page, (int)c.vocab, p->err};
  launch_input(s, ia);

  // context split: enough workgroups to cover the chip, at least 64 tokens each
  int want = 512 / H * (H / K);   // splits so that (H/G) * splits is about 512 workgroups
  want = std::max(1, std::min(want, kMaxSplits));
  int chunk = (ctx + want - 1) / want;
  chunk = std::max(64, (chunk + 63) / 64 * 64);
  const int n_splits = (ctx + chunk - 1) / chunk;
  const long pt_h = (long)p->pt * h;

  for (int i = 0; i < p->n_local; ++i) {
    const LayerPacked& L = p->layers[i];
    GemvArgs qa{};
    qa.W = L.wqkv; qa.bias = L.bqkv; qa.N = (H + 2 * K) * h; qa.Kd = d;
    qa.x = p->xres; qa.x_kind = IN_F32; qa.norm_kind = c.norm_kind; qa.g = L.ln1_g; qa.b = L.ln1_b; qa.eps = c.norm_eps;
    qa.out = p->q; qa.H = H; qa.K = K; qa.h = h;
    qa.rope = p->rope ? p->rope + (size_t)len * (h / 2) : nullptr;
    qa.kv_tok = L.kv + ((size_t)page * K * 2 * pt_h + (size_t)slot * h) * p->esz;
    qa.pt_h = pt_h;
    launch_gemv(s, c.dtype, PRO_NORM, EPI_QKV, qa);

    AttnArgs at{};
    at.q = p->q; at.q_stride = 0; at.pool = L.kv; at.table = drow;
    at.ctx0 = ctx; at.n_q = 1; at.H = H; at.K = K; at.h = h; at.pt = p->pt;
    at.chunk = chunk; at.n_splits = n_splits; at.scale = 1.f / sqrtf((float)h);
    at.part = p->part; at.counters = p->counters; at.out = p->o; at.out_stride = 0; at.out_kind = IN_F32;
    launch_attn(s, c.dtype, at);

    GemvArgs oa{};
    oa.W = L.wo; oa.bias = L.bo; oa.N = d; oa.Kd = H * h;
    oa.x = p->o; oa.x_kind = IN_F32;
    oa.out = p->xres; oa.resid = p->xres;
    launch_gemv(s, c.dtype, PRO_COPY, EPI_RESID, oa);

    GemvArgs ua{};
    ua.W = L.wup; ua.bias = L.bup; ua.N = swiglu ? 2 * F : F; ua.Kd = d;
    ua.x = p->xres; ua.x_kind = IN_F32; ua.norm_kind = c.norm_kind; ua.g = L.ln2_g; ua.b = L.ln2_b; ua.eps = c.norm_eps;
    ua.out = p->u;
    launch_gemv(s, c.dtype, PRO_NORM, swiglu ? EPI_SWIGLU : (c.mlp_kind == MDI_MLP_GELU_TANH ? EPI_GELU_TANH : EPI_GELU_ERF), ua);

    GemvArgs da{};
    da.W = L.wdown; da.bias = L.bdown; da.N = d; da.Kd = F;
    da.x = p->u; da.x_kind = IN_F32;
    da.out = p->xres; da.resid = p->xres;
    if (i == p->n_local - 1) { da.act_out = act_out; da.act_kind = ak; }
    launch_gemv(s, c.dtype, PRO_COPY, EPI_RESID, da);
  }
  p->seq_len[seq] = (uint32_t)ctx;
  return hip_status();
}

mdi_status mdi_decode_steps(mdi_partition* p, uint32_t n, const uint32_t* seqs, const void* const* acts_in, void* const* acts_out) {
  if (!p || !n || !seqs || !acts_in || !acts_out || !p->n_local) return MDI_ERR_ARG;
  // everything that can be refused is checked before the first message is taken, so a refusal leaves no message half done
  size_t new_pages = 0;
  for (uint32_t i = 0; i < n; ++i) {
    if (!acts_in[i] || !acts_out[i]) return MDI_ERR_ARG;
    const mdi_status st = check_message(p, seqs[i]);
    if (st != MDI_OK) return st;
    for (uint32_t k = 0; k < i; ++k)
      if (seqs[k] == seqs[i]) return MDI_ERR_ARG;            // a sequence has one message in flight
    if (p->seq_len[seqs[i]] % (uint32_t)p->pt == 0) ++new_pages;
  }
  if (new_pages > p->free_pages.size()) return MDI_ERR_NOMEM;
  uint32_t i = 0;
  if (p->use_step) {
    const uint32_t per_launch = kMaxSlots;
    while (n - i >= 2) {
      const uint32_t m = std::min(per_launch, n - i);
      if (m < 2) break;
      MessagePlan mp[kMaxSlots];
      for (uint32_t k = 0; k < m; ++k) {
        const mdi_status st = plan_message(p, seqs[i + k], &mp[k]);
        if (st != MDI_OK) return st;
      }
      const mdi_status st = launch_messages(p, (int)m, seqs + i, mp, acts_in + i, acts_out + i);
      if (st != MDI_OK) return st;
      i += m;
    }
  }
  for (; i < n; ++i) {
    const mdi_status st = mdi_decode_step(p, seqs[i], acts_in[i], acts_out[i]);
    if (st != MDI_OK) return st;
  }
  return hip_status();
}

namespace {

// Launches one pass over the weights for n (2 .. kMaxBatch) planned messages.
mdi_status launch_batch(mdi_partition* p, int n, const uint32_t* seqs, const MessagePlan* mp, const void* const* ins, void* const* outs) {
  const mdi_config& c = p->cfg;
  BatchArgs a{};
  int ctx_max = 0;
  long ctx_sum = 0;
  for (int j = 0; j < n; ++j) { ctx_max = std::max(ctx_max, mp[j].ctx); ctx_sum += mp[j].ctx; }
  // Query heads per attention work item: pairs also when one head per item would give more items than workgroups
  // (every message brings n_head of them), so that a workgroup has one item and a kv head's cache is read half as often.
  // With more items than workgroups even so, four heads take the pass together (one work item then serves a whole
  // group of the 8B shape; the context splits that fill the grid are folded by one workgroup per item group).
  const int group = (int)(c.n_head / c.n_kv_head);
  int G = (n * (int)c.n_head >= 2 * p->nwg && group % 4 == 0) ? 4 : (ctx_max >= p->group_ctx || n * (int)c.n_head > p->nwg) ? p->G : 1;
  if (p->batch_group && group % p->batch_group == 0) G = p->batch_group;   // test knob, see mdi.h
  a.l0 = p->h_step_layers[0];
  a.w_stride = p->n_local > 1 ? (const char*)p->h_step_layers[1].wqkv - (const char*)p->h_step_layers[0].wqkv : 0;
  a.kv_stride = p->n_local > 1 ? (const char*)p->h_step_layers[1].kv - (const char*)p->h_step_layers[0].kv : 0;
  a.n_layer = p->n_local;
  a.d = c.d_model; a.H = c.n_head; a.K = c.n_kv_head; a.h = c.head_dim; a.F = c.d_ff; a.pt = p->pt;
  a.pt_h = (long)p->pt * c.head_dim;
  a.mlp_kind = c.mlp_kind; a.eps = c.norm_eps;
  a.wte = p->wte; a.wpe = p->wpe; a.vocab = (int)c.vocab;
  a.in_kind = (p->flags & MDI_HAS_EMBED) ? IN_TOKEN : act_kind(c);
  a.act_kind = act_kind(c);
  a.err = p->err; a.spin_limit = 1 << 21;
  a.n_hg = (int)c.n_head / G;
  a.scale = 1.f / sqrtf((float)c.head_dim);
  a.nwg = p->nwg; a.m = n;
  a.epoch0 = p->b_epoch;
  a.xn = p->b_xn; a.ob = p->b_ob; a.ub = p->b_ub;
  a.slot0 = p->b_slot0; a.slot_stride = (long)p->b_stride;
  a.off_q = (long)p->b_off_q; a.off_part = (long)p->b_off_part; a.off_knew = (long)p->b_off_knew; a.off_tickets = (long)p->b_off_tickets;
  a.ssq = p->b_ssq; a.flags = p->b_flags;
  a.norm_kind = (int)c.norm_kind; a.ssum = p->b_ssum; a.nc0 = p->b_nc; a.nc_stride = (long)p->b_nc_stride;
  a.ppart = p->b_ppart; a.str_S = p->b_S; a.str_oct = p->b_oct;
  for (int j = 0; j < 4; ++j) a.R[j] = p->b_R[j];
  a.lds_xres = p->b_lds_xres; a.lds_sq = p->b_lds_sq; a.lds_part = p->b_lds_part;
  a.trace = p->trace;
  // Attention work items: (message, head group, context split).  Splits of about equal length over all messages,
  // as many items as there are workgroups when the contexts allow it, no split shorter than 128 positions.
  int chunk = (int)std::max<long>(128, (ctx_sum * a.n_hg + a.nwg - 1) / a.nwg);
  chunk = (chunk + 15) / 16 * 16;
  auto items_at = [&](int ch) { long t = 0; for (int j = 0; j < n; ++j) t += (long)a.n_hg * std::min(kMaxSplits, (mp[j].ctx + ch - 1) / ch); return t; };
  while (items_at(chunk) > a.nwg && chunk < ctx_max) chunk += 16;
  int item = 0;
  for (int j = 0; j < n; ++j) {
    BatchSlot& s = a.s[j];
    s.in = ins[j]; s.act_out = outs[j];
    s.pos = mp[j].len; s.ctx = mp[j].ctx;
    s.rope = p->rope ? p->rope + (size_t)mp[j].len * (c.head_dim / 2) : nullptr;
    s.table = mp[j].drow; s.table_entry = mp[j].new_entry; s.new_page = mp[j].page;
    s.kv_tok_off = (long)mp[j].page * c.n_kv_head * 2 * a.pt_h + (long)mp[j].slot * c.head_dim;
    int ch = chunk;
    if ((mp[j].ctx + ch - 1) / ch > kMaxSplits) ch = ((mp[j].ctx + kMaxSplits - 1) / kMaxSplits + 15) / 16 * 16;
    s.chunk = ch; s.n_splits = (mp[j].ctx + ch - 1) / ch;
    s.item_lo = item;
    item += a.n_hg * s.n_splits;
  }
  a.n_items = item;
  const mdi_status st = launch_step_serialised(p, [&]() { launch_step_batch(p->stream, G, p->b_lds, a); });
  if (st != MDI_OK) return st;
  p->b_epoch += 5u * (unsigned)p->n_local;
  for (int j = 0; j < n; ++j) p->seq_len[seqs[j]] = (uint32_t)mp[j].ctx;
  return MDI_OK;
}

}  // namespace

mdi_status mdi_decode_batch(mdi_partition* p, uint32_t n, const uint32_t* seqs, const void* const* acts_in, void* const* acts_out) {
  if (!p || !n || !seqs || !acts_in || !acts_out || !p->n_local) return MDI_ERR_ARG;
  if (!p->use_batch) return mdi_decode_steps(p, n, seqs, acts_in, acts_out);
  // everything that can be refused is checked before the first message is taken, so a refusal leaves no message half done
  size_t new_pages = 0;
  for (uint32_t i = 0; i < n; ++i) {
    if (!acts_in[i] || !acts_out[i]) return MDI_ERR_ARG;
    const mdi_status st = check_message(p, seqs[i]);
    if (st != MDI_OK) return st;
    for (uint32_t k = 0; k < i; ++k)
      if (seqs[k] == seqs[i]) return MDI_ERR_ARG;            // a sequence has one message in flight
    if (p->seq_len[seqs[i]] % (uint32_t)p->pt == 0) ++new_pages;
  }
  if (new_pages > p->free_pages.size()) return MDI_ERR_NOMEM;
  for (uint32_t i = 0; i < n;) {
    const uint32_t m = std::min<uint32_t>(kMaxBatch, n - i);
    if (m == 1) {
      const mdi_status st = mdi_decode_step(p, seqs[i], acts_in[i], acts_out[i]);
      if (st != MDI_OK) return st;
    } else {
      MessagePlan mp[kMaxBatch];
      for (uint32_t k = 0; k < m; ++k) {
        const mdi_status st = plan_message(p, seqs[i + k], &mp[k]);
        if (st != MDI_OK) return st;
      }
      const mdi_status st = launch_batch(p, (int)m, seqs + i, mp, acts_in + i, acts_out + i);
      if (st != MDI_OK) return st;
    }
    i += m;
  }
  return hip_status();
}

namespace {
// Scratch of the output layers' kernels: per-workgroup argmax candidates and the arrival counter.
struct HeadScratch { float* amax_val; int* amax_idx; tagged_t* cand; unsigned* counter; int* err; };

// Tag of an output-layer launch: unique in the process, so that no word an earlier launch (of any partition, in the
// arena or in the static array) left behind can pass for this launch's.  0 is what fresh scratch holds.
std::atomic<unsigned> g_head_tag{0};
unsigned next_head_tag() {
  unsigned t = ++g_head_tag;
  while (t == 0) t = ++g_head_tag;
  return t;
}

// final norm + vocabulary projection + greedy argmax; logits (optional) go to `logits`
void launch_head(mdi_partition* p, const void* act_in, int32_t* token_out, float* logits, const HeadScratch& hs) {
  const mdi_config& c = p->cfg;
  if (p->head_nwg) {
    LogitsArgs a{p->lm_head, (int)c.vocab, (int)c.d_model, act_in, act_kind(c), (int)c.norm_kind, p->lnf_g, p->lnf_b, c.norm_eps,
                 logits, hs.cand, next_head_tag(), hs.counter, token_out, p->head_part_floats, hs.err, 1 << 21};
    launch_logits(p->stream, c.dtype, p->head_nwg, p->head_lds, a);
    return;
  }
  GemvArgs a{};
  a.W = p->lm_head; a.N = (int)c.vocab; a.Kd = (int)c.d_model;
  a.x = act_in; a.x_kind = act_kind(c); a.norm_kind = c.norm_kind; a.g = p->lnf_g; a.b = p->lnf_b; a.eps = c.norm_eps;
  a.out = logits; a.amax_val = hs.amax_val; a.amax_idx = hs.amax_idx;
  a.counter = hs.counter; a.token_out = token_out;
  launch_gemv(p->stream, c.dtype, PRO_NORM, EPI_LOGITS, a);
}
HeadScratch arena_head_scratch(const mdi_partition* p) {
  return HeadScratch{p->amax_val, p->amax_idx, p->cand, p->counters + p->cfg.n_head, p->herr};
}
}  // namespace

mdi_status mdi_sample_greedy(mdi_partition* p, uint32_t seq, const void* act_in, int32_t* token_out, float* logits_out) {
  if (!p || !act_in || !token_out) return MDI_ERR_ARG;
  if (!(p->flags & MDI_HAS_HEAD)) return MDI_ERR_STATE;
  const mdi_config& c = p->cfg;
  if (seq >= c.max_seqs) return MDI_ERR_ARG;
  launch_head(p, act_in, token_out, logits_out, arena_head_scratch(p));
  return hip_status();
}

mdi_status mdi_sample_topk(mdi_partition* p, uint32_t seq, const void* act_in, float temperature, uint32_t top_k,
                           uint64_t seed, uint32_t step, int32_t* token_out, float* logits_out) {
  if (!p || !act_in || !token_out) return MDI_ERR_ARG;
  if (!(p->flags & MDI_HAS_HEAD)) return MDI_ERR_STATE;
  const mdi_config& c = p->cfg;
  if (seq >= c.max_seqs || !(temperature > 0.f) || !top_k || top_k > (uint32_t)kMaxTopK) return MDI_ERR_ARG;
  launch_head(p, act_in, token_out, p->logits, arena_head_scratch(p));
  if (logits_out && hipMemcpyAsync(logits_out, p->logits, (size_t)c.vocab * 4, hipMemcpyDeviceToDevice, p->stream) != hipSuccess)
    return MDI_ERR_HIP;
  SampleArgs sa{p->logits, (int)c.vocab, (int)std::min<uint32_t>(top_k, c.vocab), 1.f / temperature, seq, step,
                (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32), token_out};
  launch_sample_topk(p->stream, sa);
  return hip_status();
}

mdi_status mdi_sample_topk_static(mdi_partition* p, uint32_t seq, const void* act_in, float temperature, uint32_t top_k,
                                  uint64_t seed, uint32_t step, int32_t* token_out, float* logits_out) {
  if (!p || !act_in || !token_out) return MDI_ERR_ARG;
  if (!(p->flags & MDI_HAS_HEAD)) return MDI_ERR_STATE;
  const mdi_config& c = p->cfg;
  if (seq >= c.max_seqs || !(temperature > 0.f) || !top_k || top_k > (uint32_t)kMaxTopK) return MDI_ERR_ARG;
  if ((size_t)c.vocab > kStaticVocabMax) return MDI_ERR_LIMIT;
  const int nwg = p->head_nwg ? p->head_nwg : gemv_grid((int)c.vocab);
  if ((size_t)nwg > kStaticCand) return MDI_ERR_LIMIT;
  unsigned char* base = nullptr;
  const mdi_status sst = static_scratch(p->device, &base);   // taken at create; here only read
  if (sst != MDI_OK) return sst;
  float* logits = (float*)(base + kStaticLogitsOff);
  const HeadScratch hs{(float*)(base + kStaticValOff), (int*)(base + kStaticIdxOff), (tagged_t*)(base + kStaticCandOff),
                       (unsigned*)(base + kStaticCounterOff), (int*)(base + kStaticErrOff)};
  // the array keeps the last call's contents: the arrival counter must start at zero (a fill kernel, not a
  // memset node, so that the call can be captured into a graph); everything else is written before it is read
  launch_fill_u32(p->stream, hs.counter, 1, 0u);
  launch_head(p, act_in, token_out, logits, hs);
  if (logits_out) launch_copy_rows(p->stream, 4, logits, logits_out, 1, (long)c.vocab, 1, 0);
  SampleArgs sa{logits, (int)c.vocab, (int)std::min<uint32_t>(top_k, c.vocab), 1.f / temperature, seq, step,
                (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32), token_out};
  launch_sample_topk(p->stream, sa);
  return hip_status();
}

mdi_status mdi_sample_batch(mdi_partition* p, uint32_t n, const uint32_t* seqs, const void* const* acts_in, float temperature,
                            uint32_t top_k, uint64_t seed, const uint32_t* steps, int32_t* tokens_out, float* logits_out) {
  if (!p) return MDI_ERR_ARG;
  if (!(p->flags & MDI_HAS_HEAD)) return MDI_ERR_STATE;
  if (n == 0) return MDI_OK;
  if (!acts_in || !tokens_out || !seqs) return MDI_ERR_ARG;
  const mdi_config& c = p->cfg;
  if (!top_k || top_k > (uint32_t)kMaxTopK || (top_k > 1 && (!(temperature > 0.f) || !steps))) return MDI_ERR_ARG;
  bool aligned = true;
  for (uint32_t i = 0; i < n; ++i) {
    if (seqs[i] >= c.max_seqs || !acts_in[i]) return MDI_ERR_ARG;
    aligned = aligned && ((uintptr_t)acts_in[i] & 15u) == 0;
  }
  const size_t V = c.vocab;
  if (!p->hb_nwg || !aligned || n == 1) {
    // one sample, or a head the shared pass does not cover: the output layers once per sample
    for (uint32_t i = 0; i < n; ++i) {
      float* lg = logits_out ? logits_out + (size_t)i * V : nullptr;
      const mdi_status st = top_k == 1 ? mdi_sample_greedy(p, seqs[i], acts_in[i], tokens_out + i, lg)
                                       : mdi_sample_topk(p, seqs[i], acts_in[i], temperature, top_k, seed, steps[i], tokens_out + i, lg);
      if (st != MDI_OK) return st;
    }
    return hip_status();
  }
  for (uint32_t i = 0; i < n; i += kMaxBatch) {
    const int m = (int)std::min<uint32_t>(kMaxBatch, n - i);
    float* user = logits_out ? logits_out + (size_t)i * V : nullptr;
    // the draw overwrites the logits it picks from: with top_k > 1 the pass writes the library's rows
    float* rows = top_k > 1 ? p->hb_logits : user;
    LogitsBatchArgs a{};
    a.W = p->lm_head; a.N = (int)V; a.Kd = (int)c.d_model;
    for (int j = 0; j < m; ++j) a.x[j] = acts_in[i + j];
    a.m = m; a.g = p->lnf_g; a.b = p->lnf_b; a.norm_kind = (int)c.norm_kind; a.eps = c.norm_eps;
    a.out = rows; a.out_stride = (long)V;
    a.cand = p->hb_cand; a.tag = next_head_tag(); a.counter = p->counters + c.n_head + 1;
    a.err = p->herr; a.spin_limit = 1 << 21;
    a.token_out = tokens_out + i;
    launch_logits_batch(p->stream, p->hb_nwg, p->hb_lds, a);
    if (top_k > 1) {
      if (user && hipMemcpyAsync(user, rows, (size_t)m * V * 4, hipMemcpyDeviceToDevice, p->stream) != hipSuccess) return MDI_ERR_HIP;
      SampleBatchArgs sb{};
      sb.logits = rows; sb.stride = (long)V; sb.V = (int)V; sb.k = (int)std::min<uint32_t>(top_k, c.vocab);
      sb.inv_t = 1.f / temperature; sb.key0 = (uint32_t)(seed & 0xFFFFFFFFu); sb.key1 = (uint32_t)(seed >> 32);
      sb.token_out = tokens_out + i;
      for (int j = 0; j < m; ++j) { sb.ctr0[j] = seqs[i + j]; sb.ctr1[j] = steps[i + j]; }
      launch_sample_topk_batch(p->stream, m, sb);
    }
  }
  return hip_status();
}

mdi_status mdi_partition_sync(mdi_partition* p) {
  if (!p) return MDI_ERR_ARG;
  if (hipStreamSynchronize(p->stream) != hipSuccess) return MDI_ERR_HIP;
  if (p->herr) {                         // output layers: a candidate never showed its launch's tag
    int e = 0;
    if (hipMemcpy(&e, p->herr, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return MDI_ERR_HIP;
    if (e) return MDI_ERR_HIP;
    unsigned char* base = nullptr;       // the same word of the static scratch, if this device's was ever used
    { std::lock_guard<std::mutex> lock(g_scratch_mutex); base = g_scratch_ptr[p->device]; }
    if (base && hipMemcpy(&e, base + kStaticErrOff, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return MDI_ERR_HIP;
    if (e) return MDI_ERR_HIP;
  }
  if (p->err) {
    int e = 0;
    if (hipMemcpy(&e, p->err, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return MDI_ERR_HIP;
    if (e == 2) return MDI_ERR_ARG;      // a token id outside [0, vocab) reached a kernel
    if (e) return MDI_ERR_HIP;
  }
  return hip_status();
}

mdi_status mdi_seq_reset(mdi_partition* p, uint32_t seq) {
  if (!p || seq >= p->cfg.max_seqs) return MDI_ERR_ARG;
  const int len = (int)p->seq_len[seq];
  if (len && p->n_local) {
    const int used = (len + p->pt - 1) / p->pt;
    const int32_t* row = p->host_tables.data() + (size_t)seq * p->pages_per_seq;
    for (int i = used - 1; i >= 0; --i) p->free_pages.push_back(row[i]);
  }
  p->seq_len[seq] = 0;
  return MDI_OK;
}

mdi_status mdi_seq_len(const mdi_partition* p, uint32_t seq, uint32_t* len) {
  if (!p || !len || seq >= p->cfg.max_seqs) return MDI_ERR_ARG;
  *len = p->seq_len[seq];
  return MDI_OK;
}

mdi_status mdi_step_bytes(const mdi_partition* p, uint32_t ctx, int head, uint64_t* bytes) {
  if (!p || !bytes) return MDI_ERR_ARG;
  const mdi_config& c = p->cfg;
  const uint64_t B = p->esz, d = c.d_model, H = c.n_head, K = c.n_kv_head, h = c.head_dim, F = c.d_ff, V = c.vocab;
  if (head) {
    if (!(p->flags & MDI_HAS_HEAD)) return MDI_ERR_STATE;
    *bytes = V * d * B + d * B + 4;
    return MDI_OK;
  }
  const uint64_t mlp = (c.mlp_kind == MDI_MLP_SWIGLU ? 3 : 2) * d * F;
  const uint64_t layer = ((H + 2 * K) * h * d + d * H * h + mlp) * B;
  const uint64_t kv_tok = 2 * K * h * B;
  *bytes = (uint64_t)p->n_local * (layer + kv_tok * ctx + kv_tok) + 2 * d * B;
  return MDI_OK;
}

mdi_status mdi_time_kernel(mdi_partition* p, int which, uint32_t reps, float* avg_us, uint64_t* bytes_per_launch) {
  if (!p || !avg_us || !bytes_per_launch || !p->n_local || !reps || which < 1 || which > 3) return MDI_ERR_ARG;
  const mdi_config& c = p->cfg;
  const int d = c.d_model, H = c.n_head, h = c.head_dim, F = c.d_ff;
  const bool swiglu = c.mlp_kind == MDI_MLP_SWIGLU;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return MDI_ERR_HIP;
  auto once = [&]() {
    for (int i = 0; i < p->n_local; ++i) {
      const LayerPacked& L = p->layers[i];
      GemvArgs a{};
      if (which == 1) {
        a.W = L.wo; a.bias = L.bo; a.N = d; a.Kd = H * h; a.x = p->o; a.x_kind = IN_F32; a.out = p->xres; a.resid = p->xres;
        launch_gemv(p->stream, c.dtype, PRO_COPY, EPI_RESID, a);
      } else if (which == 2) {
        a.W = L.wup; a.bias = L.bup; a.N = swiglu ? 2 * F : F; a.Kd = d; a.x = p->xres; a.x_kind = IN_F32;
        a.norm_kind = c.norm_kind; a.g = L.ln2_g; a.b = L.ln2_b; a.eps = c.norm_eps; a.out = p->u;
        launch_gemv(p->stream, c.dtype, PRO_NORM, swiglu ? EPI_SWIGLU : (c.mlp_kind == MDI_MLP_GELU_TANH ? EPI_GELU_TANH : EPI_GELU_ERF), a);
      } else {
        a.W = L.wdown; a.bias = L.bdown; a.N = d; a.Kd = F; a.x = p->u; a.x_kind = IN_F32; a.out = p->xres; a.resid = p->xres;
        launch_gemv(p->stream, c.dtype, PRO_COPY, EPI_RESID, a);
      }
    }
  };
  once();   // warm-up
  bool ok = hipEventRecord(e0, p->stream) == hipSuccess;
  for (uint32_t r = 0; r < reps; ++r) once();
  ok = ok && hipEventRecord(e1, p->stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
  float ms = 0.f;
  ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok) return MDI_ERR_HIP;
  *avg_us = ms * 1000.f / ((float)reps * (float)p->n_local);
  const uint64_t B = p->esz;
  *bytes_per_launch = which == 1 ? (uint64_t)d * H * h * B : which == 2 ? (uint64_t)(swiglu ? 2 : 1) * F * d * B : (uint64_t)d * F * B;
  return hip_status();
}

mdi_status mdi_partition_info(const mdi_partition* p, uint32_t what, uint64_t* value) {
  if (!p || !value) return MDI_ERR_ARG;
  switch (what) {
    case 0: *value = p->use_step ? 2 : 1; return MDI_OK;
    case 1: *value = p->use_step ? (uint64_t)p->nwg : 0; return MDI_OK;
    case 2: *value = p->use_step ? (uint64_t)p->step_lds : 0; return MDI_OK;
    case 3: *value = p->arena_bytes; return MDI_OK;
    case 4: *value = p->use_batch ? (uint64_t)kMaxBatch : 0; return MDI_OK;
    case 6: *value = p->hb_nwg ? (uint64_t)kMaxBatch : 0; return MDI_OK;
    case 5: {
      const mdi_config& c = p->cfg;
      const uint64_t B = p->esz, d = c.d_model, H = c.n_head, K = c.n_kv_head, h = c.head_dim, F = c.d_ff;
      *value = (uint64_t)p->n_local * ((H + 2 * K) * h * d + d * H * h + (c.mlp_kind == MDI_MLP_SWIGLU ? 3 : 2) * d * F) * B;
      return MDI_OK;
    }
    default: return MDI_ERR_ARG;
  }
}

mdi_status mdi_partition_trace(mdi_partition* p, void* trace) {
  if (!p) return MDI_ERR_ARG;
  p->trace = (unsigned long long*)trace;
  return MDI_OK;
}

void mdi_partition_destroy(mdi_partition* p) { delete p; }

const char* mdi_strerror(mdi_status st) {
  switch (st) {
    case MDI_OK: return "ok";
    case MDI_ERR_ARG: return "invalid argument";
    case MDI_ERR_STATE: return "call not valid in the sequence's or partition's state";
    case MDI_ERR_CTX: return "context length exceeded";
    case MDI_ERR_NOMEM: return "arena too small or KV page pool exhausted";
    case MDI_ERR_HIP: return "HIP runtime error";
    case MDI_ERR_LIMIT: return "size beyond the fixed scratch of the entry point that allocates nothing";
  }
  return "unknown status";
}

}  // extern "C"
