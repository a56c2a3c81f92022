// Internal declarations shared by the translation units of libmdi.
// Each .hip file owns its kernels and exposes host-side launchers declared here.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mdi.h"

namespace mdi {

constexpr int kBlock = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int kWave = 64;
constexpr int kMaxSplits = 64;       // context splits of single-query attention

typedef uint16_t bf16_t;             // bfloat16 bit pattern

// ---- input of a step ------------------------------------------------------
enum InKind { IN_TOKEN = 0, IN_F32 = 1, IN_BF16 = 2 };

// ---- weight-streaming GEMV family (decode; Sec. III-D: one position per visit)
enum Prologue { PRO_COPY = 0, PRO_NORM = 1 };
enum Epilogue { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_GELU_TANH = 3, EPI_GELU_ERF = 4, EPI_LOGITS = 5 };

struct GemvArgs {
  const void* W;        // [N, Kd] row-major, storage dtype
  const float* bias;    // [N] or nullptr
  int N, Kd;
  // prologue: vector of Kd values, fp32 or bf16, optionally normalised
  const void* x;
  int x_kind;           // IN_F32 | IN_BF16
  int norm_kind;        // MDI_NORM_*, used when the kernel's prologue is PRO_NORM
  const float* g;       // norm gain [Kd]
  const float* b;       // norm bias [Kd] or nullptr
  float eps;
  // epilogue
  float* out;           // EPI_QKV: q[H*h]; EPI_RESID: x (updated in place); SWIGLU/GELU: u[F]; LOGITS: logits or nullptr
  const float* resid;   // EPI_RESID: residual input [N]
  void* act_out;        // EPI_RESID: optional copy in storage dtype [N] (hand-off to the next stage)
  int act_kind;         // IN_F32 | IN_BF16
  // EPI_QKV
  int H, K, h;
  const float2* rope;   // (cos, sin)[h/2] of the current position, or nullptr
  void* kv_tok;         // address of K[kv head 0][slot][0] for this layer/page; V follows at +pt_h elements
  long pt_h;            // page_tokens * head_dim
  // EPI_LOGITS
  float* amax_val;      // [gridDim.x] per-workgroup best
  int* amax_idx;
  unsigned* counter;    // arrival counter, zero between calls
  int32_t* token_out;
};

void launch_gemv(hipStream_t s, int dtype, int pro, int epi, const GemvArgs& a);
int gemv_grid(int N);   // workgroups launch_gemv uses for N rows (sizes the argmax partials)

struct InputArgs {
  const void* in; int in_kind;       // token id / fp32 / bf16 vector
  const void* wte; const void* wpe;  // storage dtype
  int dtype; int pos; int d;
  float* xres;                       // [d] fp32 residual stream
  int32_t* table_entry; int new_page; // page-table slot to fill before attention (or nullptr)
  int vocab; int* err;               // a token id outside [0, vocab) sets *err = 2 and is read as token 0
};
void launch_input(hipStream_t s, const InputArgs& a);

struct AttnArgs {
  const float* q;          // [n_q][H*h] fp32, rotated
  long q_stride;
  const void* pool;        // this layer's pages: [page][K][2][pt][h], storage dtype
  const int32_t* table;    // this sequence's page ids
  int ctx0;                // keys visible to query row 0 (query row y sees ctx0 + y)
  int n_q;                 // query rows (1 for decode)
  int H, K, h, pt;
  int chunk, n_splits;     // context split (n_splits == 1 when n_q > 1)
  float scale;
  float* part;             // [H][kMaxSplits][h + 2] split partials
  unsigned* counters;      // [H] arrival counters, zero between calls
  void* out;               // [n_q][H*h]
  long out_stride;
  int out_kind;            // IN_F32 | IN_BF16
};
void launch_attn(hipStream_t s, int dtype, const AttnArgs& a);

// ---- stochastic sampling of the output pmf (Alg. 1) -----------------------
constexpr int kMaxTopK = 64;
struct SampleArgs {
  float* logits;        // [V] fp32; destroyed (the chosen candidates are overwritten)
  int V, k;             // k <= kMaxTopK and k <= V
  float inv_t;          // 1 / temperature
  uint32_t ctr0, ctr1;  // counter of the generator: (sample, step)
  uint32_t key0, key1;  // its key: the two halves of the seed
  int32_t* token_out;
};
void launch_sample_topk(hipStream_t s, const SampleArgs& a);
void launch_row_dots(hipStream_t s, const void* W, int N, int Kd, const float* g, const float* b, float* c1, float* c2);
struct SampleBatchArgs {              // the same draw for up to 16 samples, one workgroup each
  float* logits; long stride;         // row j = sample j's logits [V]; destroyed like SampleArgs::logits
  int V, k; float inv_t;
  uint32_t key0, key1;
  int32_t* token_out;                 // [m]
  uint32_t ctr0[16], ctr1[16];        // (sample, step) per sample
};
void launch_sample_topk_batch(hipStream_t s, int m, const SampleBatchArgs& a);

// ---- prefill (first visit: T positions at once; Alg. 2) -------------------
struct RowsInArgs {
  const void* in; int in_kind; const void* wte; const void* wpe; int dtype;
  int T, d; float* xres;
  int vocab; int* err;               // a token id outside [0, vocab) sets *err = 2 and is read as token 0
  int pos0;                          // position of row 0 (a first visit in several chunks continues at the cache length)
};
void launch_rows_input(hipStream_t s, const RowsInArgs& a);

struct NormRowsArgs {
  const float* x; int T, d; int norm_kind; const float* g; const float* b; float eps;
  void* out; int out_kind;
};
void launch_norm_rows(hipStream_t s, const NormRowsArgs& a);

enum GemmEpi { GEPI_F32_BIAS = 0, GEPI_RESID = 1, GEPI_SWIGLU = 2, GEPI_GELU_TANH = 3, GEPI_GELU_ERF = 4 };
struct GemmArgs {
  const void* A;     // [T, Kd] storage dtype
  const void* W;     // [N, Kd] storage dtype
  const float* bias; // [N] or nullptr
  int T, N, Kd;
  float* out_f32;    // GEPI_F32_BIAS: [T, N]; GEPI_RESID: residual stream [T, N], updated in place
  void* out_act;     // SWIGLU: [T, N/2]; GELU: [T, N]; RESID: optional hand-off copy [T, N]; storage dtype
};
void launch_gemm(hipStream_t s, int dtype, int epi, const GemmArgs& a);

struct RopeScatterArgs {
  const float* qkv;  // [T, (H+2K)h] fp32
  int T, H, K, h, pt;
  const float2* rope;     // [max_ctx][h/2] or nullptr
  float* q_out;           // [T, H*h] fp32, or nullptr
  void* pool;             // this layer's pages
  const int32_t* table;
  int dtype;
  // operands of the matrix-core attention of the first visit (bf16), or nullptr
  bf16_t* q_bf;           // [T][H*h], rotated and scaled by `scale`
  bf16_t* k_bf;           // [K][ldk][h], rotated; row pos0 + t holds position pos0 + t, rows up to pos0 + n_rows - 1 are zero-filled
  int ldk; int n_rows;    // positions the operand arrays have room for per kv head; rows to write or clear (>= T)
  float scale;
  int pos0;               // position of row 0
};
void launch_rope_scatter(hipStream_t s, const RopeScatterArgs& a);

// Causal attention of a first visit on the matrix cores (bf16 operands, fp32 accumulation and softmax).
struct FlashArgs {
  const bf16_t* q;        // [T][H*h] rotated, scaled: the queries of positions p0 .. p0 + T - 1
  const bf16_t* k;        // [K][ldk][h]: keys of positions 0 .. p0 + T - 1, finite up to Tk - 1
  const bf16_t* vt;       // [K][h][ldk]: values transposed, so that the contraction index (position) is contiguous
  bf16_t* out;            // [T][H*h]
  int T, Tp, H, K, h;     // Tp: T rounded up to 128 (the query grid)
  int p0, Tk, ldk;        // Tk: p0 + T rounded up to 64 (at most ldk)
};
bool flash_supported(int dtype, int h);
// values of T new positions (fp32 rows of the fused QKV product) -> vt[.][pos0 + t], zeros up to column pos0 + n_cols - 1
void launch_v_transpose(hipStream_t s, const float* qkv, int T, int n_cols, int pos0, int ldk, int H, int K, int h, bf16_t* vt);
// keys and values of positions 0 .. n_pos - 1 from a layer's cache pages (bf16) into the attention operand arrays
void launch_cache_gather(hipStream_t s, const void* pool, const int32_t* table, int n_pos, int K, int h, int pt, int ldk,
                         bf16_t* k_bf, bf16_t* vt);
void launch_flash_prefill(hipStream_t s, const FlashArgs& a);

// ---- whole decode step as one persistent launch ------------------------------
constexpr int kStepWavesMax = 8;     // wavefronts per workgroup: 8 (one workgroup per compute unit) or 4 (two)
constexpr int kMaxSlots = 8;         // messages one launch can carry
constexpr int kFlagStride = 32;      // batched pass: a workgroup's phase counter has a 128-byte line to itself (in 4-byte words);
                                     // measured on the one-message kernels as well: no gain there, their counters stay packed

typedef unsigned long long tagged_t;  // low half: the value's bits, high half: the phase counter it was written in

struct StepLayer {                   // device-resident, one per local layer
  const void *wqkv, *wo, *wup, *wdown;
  const float *bqkv, *bo, *bup, *bdown, *ln1_g, *ln1_b, *ln2_g, *ln2_b;
  void* kv;                          // this layer's pages
};

// What belongs to one message (one sequence's new token) inside a launch.  A launch carries one or two messages:
// with two, every phase runs for message 0 and then for message 1, so that the exchange between workgroups that
// ends one message's phase is covered by the other message's weight streaming.  Each message has its own exchange
// buffers, flags and counters.
struct StepSlot {
  const void* in; int in_kind;
  int pos, ctx;                      // position of the new token, context length including it
  const float2* rope;                // (cos, sin)[h/2] of `pos`, or nullptr
  const int32_t* table; int32_t* table_entry; int new_page;
  long kv_tok_off;                   // element offset of K[kv head 0][slot] of the new token inside a layer's pool
  // vectors exchanged between workgroups inside the launch: every element is (float bits, tag) in 8 bytes
  tagged_t *xres, *q, *o, *u, *part, *knew;   // [d], [H*h], [H*h], [F], [H][kMaxSplits][h+2], [2][K*h]
  unsigned *tickets, *flags; unsigned epoch0;
  int n_splits, chunk;
  void* act_out;
  unsigned long long* trace;         // optional [workgroup][n_layer * 5 phases][4] timestamps (100 MHz ticks), or nullptr
};
struct StepArgs {
  StepLayer l0;                      // first local layer; layer i's pointers are these advanced by i strides
  long w_stride, kv_stride;          // bytes between consecutive layers' packed weights / page pools
  int n_layer;
  int d, H, K, h, F, pt; long pt_h;
  int norm_kind, mlp_kind; float eps;
  const void* wte; const void* wpe; int vocab;
  int* err; int spin_limit;          // *err: 1 = a bounded wait expired, 2 = a token id outside [0, vocab) (read as token 0)
  int n_hg; float scale;
  int act_kind;
  int part_floats;                   // LDS floats reserved for GEMV pair partials (multiple of 4)
  int nwg;                           // workgroups in a set
  int n_slots;                       // messages in this launch, 1 .. kMaxSlots
  int n_sets;                        // sets of workgroups, 1 or 2 (grid = n_sets * nwg): set i takes messages
  int set_lo[3];                     // [set_lo[i], set_lo[i + 1]), alternating between them inside every phase
  StepSlot s[kMaxSlots];
};
// workgroups of 8 wavefronts (n_sets must be 1) / of 4 wavefronts
void launch_step_w8(hipStream_t s, int dtype, int G, int nwg, size_t lds_bytes, const StepArgs& a);
void launch_step_w4(hipStream_t s, int dtype, int G, int nwg, size_t lds_bytes, const StepArgs& a);


// Output layers as one streaming launch (step_w8.hip): final norm, vocabulary projection, greedy argmax.
struct LogitsArgs {
  const void* W; int N, Kd;          // vocabulary matrix [N, Kd], storage dtype
  const void* x; int x_kind;         // activation [Kd]
  int norm_kind; const float* g; const float* b; float eps;
  float* out;                        // logits [N] or nullptr
  tagged_t* cand; unsigned tag;      // per-workgroup candidates [workgroups][2] as (value | tag), (index | tag); tag = this call's
  unsigned* counter;                 // arrival counter, zero between calls
  int32_t* token_out;
  int part_floats;                   // LDS floats reserved for pair partials (multiple of 4)
  int* err; int spin_limit;          // error word, set when a candidate never shows this call's tag
};
void launch_logits(hipStream_t s, int dtype, int nwg, size_t lds_bytes, const LogitsArgs& a);

// ---- decode step of several queued messages with ONE pass over the weights (step_w8.hip) ----------------
// The messages waiting in the node's input queue (Sec. III-A; several samples are in flight, Sec. III-C) are
// taken through every layer together: a weight tile is fetched once and multiplied with all their vectors on the
// matrix cores (the messages are the second operand's columns), attention stays per sample.
constexpr int kMaxBatch = 16;        // messages one pass can carry: the matrix instruction's column count

struct BatchSlot {                   // what belongs to one message of the launch
  const void* in;                    // token id (int32) or activation [d] in storage dtype
  const float2* rope;                // (cos, sin)[h/2] of its position, or nullptr
  const int32_t* table; int32_t* table_entry;
  void* act_out;
  long kv_tok_off;                   // element offset of K[kv head 0][slot] of the new token inside a layer's pool
  int pos, ctx, new_page;
  int n_splits, chunk;               // context splits of its attention
  int item_lo;                       // its attention work items are item_lo .. item_lo + n_hg * n_splits - 1
};
struct BatchArgs {
  StepLayer l0; long w_stride, kv_stride; int n_layer;
  int d, H, K, h, F, pt; long pt_h;
  int mlp_kind; float eps;
  const void* wte; const void* wpe; int vocab;
  int in_kind, act_kind;
  int* err; int spin_limit;          // as in StepArgs
  int n_hg; float scale;
  int nwg, m;                        // workgroups (one set), messages
  unsigned epoch0;
  // Exchange buffers.  Vectors that feed a matrix product travel as pairs of bf16 with the writing phase's counter
  // in one 8-byte word, one array [pair of columns][kMaxBatch messages] per kind for the whole launch (xn: the
  // residual stream times the gain of the norm that follows; ob: attention output; ub: MLP hidden).  What attention
  // needs per message - q, the newest K/V row, split partials as (float, counter) like in StepSlot, tickets - sits
  // in one block per message: message j's are message 0's advanced by j * slot_stride bytes.
  tagged_t *xn, *ob, *ub;
  char* slot0; long slot_stride;
  long off_q, off_part, off_knew, off_tickets;
  tagged_t* ssq;                     // [kMaxBatch][nwg] per-workgroup sums of squares of the residual rows they own
  // LayerNorm (norm_kind = MDI_NORM_LAYERNORM): the sums of those rows travel too, and the products of a normalised
  // vector are corrected in the epilogue, y = rstd (W (x g)) - rstd mean (W g) + W b: per layer the four vectors
  // [W_qkv g1 | W_qkv b1 | W_up g2 | W_up b2] (float), layer l's at nc0 + l * nc_stride floats
  int norm_kind; tagged_t* ssum; const float* nc0; long nc_stride;
  tagged_t* ppart; int str_S, str_oct; // products split among workgroups along the inner dimension: partials [block][S][256], slices per block, block octets
  unsigned* flags;                   // [nwg] phase counters of the workgroups
  int R[4];                          // rows per matrix-instruction block in the QKV / output / up / down products (8 or 16)
  int lds_xres, lds_sq, lds_part;    // LDS layout in floats
  int n_items;                       // attention work items of the launch
  unsigned long long* trace;         // optional [workgroup][n_layer][5][8] timestamps (100 MHz ticks), or nullptr
  BatchSlot s[kMaxBatch];
};
// Output layers of up to kMaxBatch samples with one pass over the vocabulary matrix (step_w8.hip; bf16).
struct LogitsBatchArgs {
  const void* W; int N, Kd;          // vocabulary matrix [N, Kd] bf16; Kd a multiple of 32, N * Kd * 2 < 2^32
  const void* x[kMaxBatch]; int m;   // activations [Kd] bf16, 16-byte aligned, one per sample
  const float* g; const float* b; int norm_kind; float eps;   // the final norm: gain, bias (LayerNorm; may be nullptr), kind
  float* out; long out_stride;       // logits: row j = sample j, [N] floats each, rows out_stride floats apart; or nullptr
  tagged_t* cand; unsigned tag;      // candidates [kMaxBatch][workgroups][2] as (value | tag), (index | tag); tag = this call's
  unsigned* counter;                 // arrival counter, zero between calls
  int32_t* token_out;                // [m]
  int* err; int spin_limit;          // error word, set when a candidate never shows this call's tag
};
bool logits_batch_allow_lds(size_t lds_bytes);
void launch_logits_batch(hipStream_t s, int nwg, size_t lds_bytes, const LogitsBatchArgs& a);

void launch_step_batch(hipStream_t s, int G, size_t lds_bytes, const BatchArgs& a);
bool step_batch_allow_lds(size_t lds_bytes);

// ---- set-up ---------------------------------------------------------------
void launch_rope_table(hipStream_t s, float2* table, int max_ctx, int h, double base);
// dst[r*dst_stride_rows + ...]: copy `rows` rows of `cols` elements, dst row = r*row_mul + row_off
void launch_copy_rows(hipStream_t s, int elem_bytes, const void* src, void* dst, long rows, long cols, long row_mul, long row_off);
void launch_fill_f32(hipStream_t s, float* dst, long n, float v);
void launch_fill_u32(hipStream_t s, uint32_t* dst, long n, uint32_t v);

}  // namespace mdi
