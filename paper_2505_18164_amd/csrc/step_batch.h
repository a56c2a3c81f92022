// Decode step of SEVERAL queued messages with ONE pass over the partition's weights.
//
// The paper's node takes the messages of its input queue one at a time (Sec. III-A), so every later visit of a
// sample (Sec. III-D) streams all local weights again.  With several samples in flight (Sec. III-C) their messages
// wait in the queue together; here up to 16 of them go through every layer together: a 16-byte piece of a weight
// row is fetched once and multiplied with all the messages' vectors by one matrix instruction
// (v_mfma_f32_16x16x32_bf16: 16 weight rows x 32 columns times 32 x 16 messages), attention stays per sample over
// each sample's own cache.  The kernel is still bound by HBM: the matrix cores only take over the multiply-adds
// that the vector ALUs could not do for 16 messages at the rate the weights arrive.
//
// Same skeleton as k_step (one persistent launch, five phases per layer, a grid-wide barrier of per-workgroup
// phase counters, self-validating tagged exchange), with these differences:
//   * One set of 8-wavefront workgroups, all messages in lockstep.
//   * Work unit of a product = a block of R (16 or 8) weight rows; blocks are dealt round-robin to workgroups; the
//     eight wavefronts of a workgroup split the block's columns among them and their partial 16 x 16 results are
//     added in LDS in wavefront order (deterministic, no float atomics).  RoPE partners (i, i + h/2) and SwiGLU
//     partners (gate_f, up_f) sit in the same block, so the epilogue of a row pair needs no other workgroup.
//   * Vectors that feed a product cross workgroups as bf16 PAIRS with the writing phase's counter in one 8-byte
//     word, already multiplied by the gain of the RMSNorm that follows (1/rms is applied to the finished products;
//     the sum of squares travels as one partial per workgroup and message).  Bytes exchanged per message are half
//     those of k_step's (float, counter) words, which matters now that 16 messages share a pass.  A vector kind is
//     ONE array [pair of columns][16 messages] for the whole launch: the 16 lanes that hold the same columns of the
//     16 messages read 128 consecutive bytes.
//   * The residual stream never leaves the workgroup that owns its rows: it stays in LDS for the whole launch.
//   * Products whose input is the d-sized normalised vector (QKV, MLP up) keep each wavefront's column slice of all
//     messages in registers for all the blocks of the phase; the others (output projection, MLP down: one block per
//     workgroup at the benchmark shapes, a long inner dimension) split the inner dimension among workgroups, so
//     that a workgroup reads a fraction of the vectors, and exchange 16 x 16 partial results (see KsGeo).
// Needs bf16 storage and widths that are multiples of 32; other shapes keep one pass per message.  With LayerNorm the vectors still travel as x * gain: the mean and the norm's bias enter the finished
// products through two precomputed vectors per matrix (W g and W b), see BatchArgs.
//
// Included by step_w8.hip after step_impl.h (shares its exchange, attention and barrier helpers).
namespace mdi {
namespace step_w8 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}
__device__ __forceinline__ void st_pair(tagged_t* p, uint32_t bits, unsigned tag) {
  __hip_atomic_store(p, ((tagged_t)tag << 32) | (tagged_t)bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The low word of *p once its counter is `tag` (see settle in step_impl.h).
__device__ __forceinline__ uint32_t settle_bits(const tagged_t* p, tagged_t u, unsigned tag, int spin_limit, int* err) {
  int it = 0;
  while ((uint32_t)(u >> 32) != tag) {
    if (++it > spin_limit) { __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
    __builtin_amdgcn_s_sleep(1);
    u = ld_raw(p);
  }
  return (uint32_t)u;
}

// A word of an exchanged vector: loaded at agent scope, i.e. from memory, not from a die's L2, which may hold an
// older copy.  (Measured: ordinary loads that L2 may answer - with one address per (layer, phase) instance of every
// vector so that no older copy can exist, and a coherent second look for words that were fetched too early - move
// 32 times less over the fabric and are not faster: the phases that stream these vectors are bound by what a
// compute unit's memory pipeline passes per unit of time, whichever cache answers.)
__device__ __forceinline__ tagged_t ld_word(const MDI_GLOBAL tagged_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// What the attention helpers of step_impl.h read of a message.
struct BatchView {
  const tagged_t *q, *knew;
  tagged_t *part, *ob;             // ob: the launch's [pair][16 messages] array of attention outputs
  unsigned* tickets;
  const int32_t* table;
  int ctx, n_splits, chunk, msg;
};
__device__ __forceinline__ BatchView view_of(const BatchArgs& a, int j, tagged_t* ob) {
  char* base = a.slot0 + (long)j * a.slot_stride;
  BatchView v;
  v.q = (const tagged_t*)(base + a.off_q); v.knew = (const tagged_t*)(base + a.off_knew);
  v.part = (tagged_t*)(base + a.off_part); v.ob = ob; v.msg = j;
  v.tickets = (unsigned*)(base + a.off_tickets);
  v.table = a.s[j].table; v.ctx = a.s[j].ctx; v.n_splits = a.s[j].n_splits; v.chunk = a.s[j].chunk;
  return v;
}


// ---------------------------------------------------------------------------
// geometry of a product (all values uniform across the wavefront)
struct BGeo {
  const char* W;        // matrix [N, Kd] bf16, row-major
  long row_bytes;
  int N, R;             // rows; rows per block (16 or 8)
  int rope_sh;          // >= 0: rows pair as RoPE partners (i, i + h/2), h = 2 << rope_sh; -1: rows (2p, 2p + 1)
  int nb_local;         // this workgroup's blocks: its block lb is block lb * nwg + wg of the matrix
  int ks0, nks;         // this wavefront's column steps [ks0, ks0 + nks), 32 columns each (products with a resident operand)
};
__device__ __forceinline__ BGeo make_bgeo(const void* W, int N, int Kd, int R, int rope_h, int wg, int nwg, int wave) {
  BGeo g;
  g.W = (const char*)W; g.row_bytes = 2L * Kd; g.N = N; g.R = R;
  g.rope_sh = rope_h ? 31 - __builtin_clz(rope_h >> 1) : -1;
  const int nblk = (N + R - 1) / R;
  g.nb_local = nblk > wg ? (nblk - wg + nwg - 1) / nwg : 0;
  // The columns are cut into one slice per wavefront; which wavefront takes which slice rotates with the workgroup,
  // so that at any moment the workgroups read different parts of the messages' vectors (every workgroup walks the
  // same vectors: in step they would all queue up at the same few memory channels).
  const int total = Kd >> 5, c = (total + kStepWaves - 1) / kStepWaves;
  g.ks0 = ((wave + wg) & (kStepWaves - 1)) * c;
  g.nks = max(0, min(c, total - g.ks0));
  if (g.nks == 0) g.ks0 = 0;          // a wavefront without columns still issues its (unused) loads inside the matrix
  return g;
}
// Row of the matrix that row i (< R) of block `block` stands for.  With RoPE pairing a block is R/2 consecutive
// rows of a head's first half followed by their partners in the second half.
__device__ __forceinline__ int block_row(const BGeo& g, int block, int i) {
  if (g.rope_sh < 0) return block * g.R + i;
  const int hsh = 31 - __builtin_clz(g.R >> 1);            // log2 of the rows a block takes of a half head
  const int bsh = g.rope_sh - hsh;                           // log2 of the blocks per head
  const int head = block >> bsh, off = (block & ((1 << bsh) - 1)) << hsh;
  return (head << (g.rope_sh + 1)) + off + (i & ((g.R >> 1) - 1)) + ((i >> hsh) << g.rope_sh);
}
// ---------------------------------------------------------------------------
// products whose second operand stays in registers (QKV, MLP up): Bv[ks] = this wavefront's column step ks of all
// messages.  A tile is 8 column steps of a block; with more than 8 steps per wavefront a block is two tiles.
constexpr int kResSteps = 16;          // column steps a wavefront can keep: widths up to 8 * 16 * 32 = 4096
template <int HALF>
__device__ __forceinline__ void res_issue(Tile& t, const BGeo& g, int lb, int wg, int nwg, int lane) {
  const int i = lane & (g.R - 1) & 15, kg = lane >> 4;
  const int row = min(block_row(g, min(lb, max(g.nb_local - 1, 0)) * nwg + wg, i), g.N - 1);
  const uint32_t woff = (uint32_t)row * (uint32_t)g.row_bytes + (uint32_t)(kg << 4);
  const MDI_GLOBAL char* base = (const MDI_GLOBAL char*)g.W + ((long)g.ks0 << 6);
  const int last = max(g.nks - 1 - HALF * 8, 0);
#pragma unroll
  for (int s = 0; s < 8; ++s)
    t.r[s] = *reinterpret_cast<const MDI_GLOBAL u32x4*>(base + ((long)(HALF * 8 + min(s, last)) << 6) + woff);
}
template <int HALF, bool LAST_HALF>
__device__ __forceinline__ void res_compute(const Tile& t, const BGeo& g, int lb, const bf16x8 (&Bv)[kResSteps], f32x4& acc,
                                            float* part, int wave, int lane) {
  if (lb >= g.nb_local) return;                                  // uniform
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const int ks = HALF * 8 + s;
    if (ks < g.nks)                                              // uniform
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t.r[s]), Bv[ks], acc, 0, 0, 0);
  }
  if (LAST_HALF) {
    *reinterpret_cast<f32x4*>(part + (((lb * kStepWaves + wave) << 6) + lane) * 4) = acc;
    acc = f32x4{0.f, 0.f, 0.f, 0.f};
  }
}

// Four tagged words -> the matrix instruction's second operand; `bad` collects whether any of them does not carry the
// counter `tag` (a store not yet visible on this die: the rare case).  No load is retried here; the caller repeats
// its loads the slow, sure way instead.
__device__ __forceinline__ bf16x8 take4(tagged_t r0, tagged_t r1, tagged_t r2, tagged_t r3, unsigned tag, uint32_t& bad) {
  bad |= (((uint32_t)(r0 >> 32) ^ tag) | ((uint32_t)(r1 >> 32) ^ tag)) | (((uint32_t)(r2 >> 32) ^ tag) | ((uint32_t)(r3 >> 32) ^ tag));
  return __builtin_bit_cast(bf16x8, u32x4{(uint32_t)r0, (uint32_t)r1, (uint32_t)r2, (uint32_t)r3});
}

// ---------------------------------------------------------------------------
// Streamed products with the inner dimension split among workgroups.  Every workgroup used to read the whole
// vector of all messages for its one block of rows: 256 copies of it through the dies' L2s, twice the bytes of
// the matrix itself in the MLP down projection.  Here workgroup (q, s) takes column slice s of the eight row
// blocks 8 q .. 8 q + 7, one block per wavefront: it reads 1 / S of the vector - once, validated, into LDS, from
// where its eight wavefronts take the matrix instruction's second operand - and hands the 16 x 16 partial result
// of every block, as tagged words, to the workgroup that owns the block's residual rows, which adds the S partials
// in slice order.
struct KsGeo {
  int S, q, s;          // slices per block; this workgroup's block octet and slice (q >= octets: no work)
  int k0, nk;           // the slice: column steps [k0, k0 + nk)
  int blk, nblk;        // this wavefront's block; blocks of the product
  bool live;            // this wavefront has columns and a block
};
__device__ __forceinline__ KsGeo make_ksgeo(int N, int Kd, int S, int octets, int wg, int wave) {
  KsGeo g;
  g.S = S; g.q = wg / S; g.s = wg - g.q * S;
  const int ktot = Kd >> 5, c = (ktot + S - 1) / S;
  g.k0 = min(g.s * c, ktot);
  g.nk = g.q < octets ? max(0, min(c, ktot - g.s * c)) : 0;
  g.nblk = (N + 15) >> 4;
  g.blk = g.q * kStepWaves + wave;
  g.live = g.nk > 0 && g.blk < g.nblk;
  return g;
}
// column steps 8 t .. 8 t + 7 of the slice (steps past its end repeat its last one)
__device__ __forceinline__ void ks_issue(Tile& t, const KsGeo& g, const char* W, uint32_t woff, int ti) {
  const MDI_GLOBAL char* base = (const MDI_GLOBAL char*)W + ((long)g.k0 << 6);
  const int last = max(g.nk - 1, 0);
#pragma unroll
  for (int s = 0; s < 8; ++s)
    t.r[s] = *reinterpret_cast<const MDI_GLOBAL u32x4*>(base + ((long)min(ti * 8 + s, last) << 6) + woff);
}
__device__ __forceinline__ void ks_compute(const Tile& t, const KsGeo& g, const u32x4* Bs, int ti, int lane, f32x4& acc) {
  const int n = lane & 15, kg = lane >> 4;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const int ks = ti * 8 + s;
    if (ks < g.nk) {                                             // uniform
      const int gi = ks * 4 + kg;
      const u32x4 b = Bs[gi * 16 + (n ^ (gi & 15))];
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t.r[s]), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    }
  }
}
// Sum over n partials of element (row i, message j): partial w at part + 256 w, element order as the matrix
// instruction leaves it (lane = 16 (i / 4) + j, register i % 4).
__device__ __forceinline__ float part_sum_n(const float* part, int i, int j, int n) {
  const float* p = part + ((((i >> 2) << 4) + j) << 2) + (i & 3);
  float v = 0.f;
  for (int w = 0; w < n; ++w) v += p[w << 8];
  return v;
}

// Sum over the wavefronts of element (row i, message j) of local block lb.
__device__ __forceinline__ float part_sum(const float* part, int lb, int i, int j) {
  const float* p = part + ((lb * kStepWaves) << 8) + ((((i >> 2) << 4) + j) << 2) + (i & 3);
  float v = 0.f;
#pragma unroll
  for (int w = 0; w < kStepWaves; ++w) v += p[w << 8];
  return v;
}

// Wavefront records -> split partial, or the finished output when there is one split; the last workgroup of a head
// group to arrive folds the splits in split order (as attn_finish in step_impl.h).  The output leaves as bf16 pairs.
template <int G>
__device__ __forceinline__ void attn_finish_pairs(const AttnGeo& g, const BatchArgs& a, const BatchView& S, const float* sm, int* s_flag, unsigned epoch) {
  const unsigned wtag = epoch + 1;
  const int h = a.h, rec = h + 2, hp = h >> 1;
  const bool single = S.n_splits == 1;
  for (int idx = threadIdx.x; idx < G * hp; idx += kStepThreads) {
    const int gi = idx / hp, e = (idx - gi * hp) * 2;
    float m = -1e30f;
    for (int w = 0; w < kStepWaves; ++w) m = fmaxf(m, sm[(w * G + gi) * rec + h]);
    float l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int w = 0; w < kStepWaves; ++w) {
      const float* r = sm + (w * G + gi) * rec;
      const float sc = __expf(r[h] - m);
      l += r[h + 1] * sc; o0 += r[e] * sc; o1 += r[e + 1] * sc;
    }
    const int head = g.hg * G + gi;
    if (single) {
      st_pair(S.ob + ((((long)head * h + e) >> 1) << 4) + S.msg, pack_bf16x2(o0 / l, o1 / l), wtag);
    } else {
      tagged_t* pr = S.part + ((long)head * kMaxSplits + g.split) * rec;
      st_tag(pr + e, o0, wtag); st_tag(pr + e + 1, o1, wtag);
      if (e == 0) { st_tag(pr + h, m, wtag); st_tag(pr + h + 1, l, wtag); }
    }
  }
  if (single) return;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned ticket = __hip_atomic_fetch_add(S.tickets + g.hg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_flag[1] = ticket == (unsigned)S.n_splits - 1;
  }
  __syncthreads();
  if (!s_flag[1]) return;
  for (int idx = threadIdx.x; idx < G * hp; idx += kStepThreads) {
    const int gi = idx / hp, e = (idx - gi * hp) * 2;
    const int head = g.hg * G + gi;
    const tagged_t* pr = S.part + (long)head * kMaxSplits * rec;
    float m = -1e30f, l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int sp0 = 0; sp0 < S.n_splits; sp0 += 4) {                // four splits' loads in flight together
      tagged_t rm[4], rl[4], ra[4], rb[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool ok = sp0 + k < S.n_splits;
        const tagged_t* r = pr + (sp0 + k) * rec;
        rm[k] = ok ? ld_raw(r + h) : 0ull; rl[k] = ok ? ld_raw(r + h + 1) : 0ull;
        ra[k] = ok ? ld_raw(r + e) : 0ull; rb[k] = ok ? ld_raw(r + e + 1) : 0ull;
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (sp0 + k < S.n_splits) {
          const tagged_t* r = pr + (sp0 + k) * rec;
          const float mk = settle(r + h, rm[k], wtag, a.spin_limit, a.err);
          const float lk = settle(r + h + 1, rl[k], wtag, a.spin_limit, a.err);
          const float ak = settle(r + e, ra[k], wtag, a.spin_limit, a.err);
          const float bk = settle(r + e + 1, rb[k], wtag, a.spin_limit, a.err);
          const float mn = fmaxf(m, mk);
          const float sa = __expf(m - mn), sb = __expf(mk - mn);
          l = l * sa + lk * sb;
          o0 = o0 * sa + ak * sb; o1 = o1 * sa + bk * sb;
          m = mn;
        }
      }
    }
    st_pair(S.ob + ((((long)head * h + e) >> 1) << 4) + S.msg, pack_bf16x2(o0 / l, o1 / l), wtag);
  }
  if (threadIdx.x == 0) __hip_atomic_store(S.tickets + g.hg, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void bstamp(const BatchArgs& a, int layer, int ph, int k) {
  if (a.trace && threadIdx.x == 0)
    a.trace[(((long)blockIdx.x * a.n_layer + layer) * 5 + ph) * 8 + k] = wall_clock64();
}

// Per-message values that a thread needs for a message index of its own (a kernel argument cannot be indexed per lane).
struct BatchLds {
  const float2* rope[kMaxBatch];
  const void* in[kMaxBatch];
  void* out[kMaxBatch];
  long kv_off[kMaxBatch];
  long tok[kMaxBatch];
  int pos[kMaxBatch];
};

// Element `row` of message j's input vector (the token's embedding plus learned position, or the previous stage's activation).
__device__ __forceinline__ float batch_input(const BatchArgs& a, const BatchLds& sl, int j, int row) {
  if (a.in_kind == IN_TOKEN) {
    float v = bf16_to_f32(((const bf16_t*)a.wte)[sl.tok[j] * a.d + row]);
    if (a.wpe) v += bf16_to_f32(((const bf16_t*)a.wpe)[(long)sl.pos[j] * a.d + row]);
    return v;
  }
  return bf16_to_f32(((const bf16_t*)sl.in[j])[row]);
}

template <int G>
__global__ __launch_bounds__(kStepThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_step_batch(BatchArgs a) {
  typedef bf16_t WT;
  extern __shared__ float smem[];
  __shared__ BatchLds sl;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wg = blockIdx.x, nwg = a.nwg, m = a.m;
  int* s_flag = lds_flag();
  float* rscale = smem + 32;                     // [16] 1/rms (LayerNorm: 1/std) of every message's vector in the normed products
  float* rshift = smem + 64;                     // [16] LayerNorm: (mean - centre) / std of every message's vector
  float* rcen = smem + 80;                       // [16] LayerNorm: the centre the vectors are published around (see below)
  const bool ln = a.norm_kind == MDI_NORM_LAYERNORM;
  float* xres = smem + a.lds_xres;               // residual rows this workgroup owns: [block][16 rows][16 messages]
  float* sq = smem + a.lds_sq;                   // squares of those rows per epilogue item; cross-wavefront sums of the first product
  float* part = smem + a.lds_part;               // the wavefronts' partial products [block][wavefront][lane][4]; attention scratch
  const int kg = lane >> 4;
  const int nmsg = min(lane & 15, m - 1);        // the message this lane's column stands for (columns past m repeat the last)

  if (threadIdx.x == 0) {
    for (int j = 0; j < m; ++j) {
      const BatchSlot& S = a.s[j];
      sl.rope[j] = S.rope; sl.in[j] = S.in; sl.out[j] = S.act_out; sl.kv_off[j] = S.kv_tok_off; sl.pos[j] = S.pos;
      sl.tok[j] = a.in_kind == IN_TOKEN ? checked_token(S.in, 0, a.vocab, a.err) : 0;
      if (wg == 0 && S.table_entry) *S.table_entry = S.new_page;    // for later launches: no position before the newest lies on a page that starts now
    }
  }
  __syncthreads();

  // Residual rows of this workgroup (the output projection's and the down projection's rows: same geometry) start
  // as the launch's inputs.  They are also published exactly as a down projection publishes its result - pairs of
  // x times the first layer's gain, this workgroup's share of the sums of squares, both with the counter the
  // first phase expects - so that the first layer's QKV product is like any other.
  // LayerNorm: a vector travels as (x - c) g in bf16, c a number per message that every workgroup knows: rounding
  // x g itself would cost accuracy whenever |mean| >> std.  c is the mean of the message's vector at the previous
  // norm of the launch (every workgroup computes it, from the same sums in the same order), for the first norm the
  // mean of the input vector, which every workgroup forms here for itself.
  if (!ln) {
    if (threadIdx.x < kMaxBatch) rcen[threadIdx.x] = 0.f;
  } else {
    for (int j = wave; j < m; j += kStepWaves) {
      float u = 0.f;
      for (int r = lane; r < a.d; r += 64) u += batch_input(a, sl, j, r);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) u += __shfl_xor(u, off, 64);
      if (lane == 0) rcen[j] = u / (float)a.d;
    }
  }
  __syncthreads();
  {
    const int Rd = a.R[1], half = Rd >> 1;
    const BGeo gd = make_bgeo(nullptr, a.d, a.H * a.h, Rd, 0, wg, nwg, wave);
    const int n_items = gd.nb_local * half * m;
    for (int e = threadIdx.x; e < n_items; e += kStepThreads) {
      const int j = e % m, p = (e / m) % half, lb = e / (m * half);
      const int r0 = (lb * nwg + wg) * Rd + 2 * p;
      float s2 = 0.f;
      if (r0 < a.d) {
        const float x0 = batch_input(a, sl, j, r0), x1 = batch_input(a, sl, j, r0 + 1);
        float* xr = xres + ((lb << 4) + 2 * p) * 16 + j;
        xr[0] = x0; xr[16] = x1;
        st_pair(a.xn + ((r0 >> 1) << 4) + j, pack_bf16x2((x0 - rcen[j]) * a.l0.ln1_g[r0], (x1 - rcen[j]) * a.l0.ln1_g[r0 + 1]), a.epoch0);
        s2 = x0 * x0 + x1 * x1;
      }
      sq[e] = s2;
    }
    __syncthreads();
    if ((int)threadIdx.x < m) {
      float t = 0.f;
      for (int e = threadIdx.x; e < n_items; e += m) t += sq[e];
      st_tag(a.ssq + (long)threadIdx.x * nwg + wg, t, a.epoch0);
      if (ln) {                                  // the rows' sum as well (from the rows kept in LDS)
        float u = 0.f;
        for (int e = threadIdx.x; e < n_items; e += m) {
          const int p = (e / m) % half, lb = e / (m * half);
          if ((lb * nwg + wg) * Rd + 2 * p < a.d) { const float* xr = xres + ((lb << 4) + 2 * p) * 16 + threadIdx.x; u += xr[0] + xr[16]; }
        }
        st_tag(a.ssum + (long)threadIdx.x * nwg + wg, u, a.epoch0);
      }
    }
  }
  __syncthreads();

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};

  // Wait until every workgroup has finished the previous phase (its counter has reached `epoch`).
  auto barrier = [&](unsigned epoch) __attribute__((always_inline)) -> bool {
    if (threadIdx.x < 64) {
      bool ok = true;
      int it = 0;
      while (true) {
        bool all = true;
        for (int i = threadIdx.x; i < nwg; i += 64) {
          const unsigned v = __hip_atomic_load(a.flags + i * kFlagStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          all = all && ((int)(v - epoch) >= 0);
        }
        if (__all(all)) break;
        if (++it > a.spin_limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      if (threadIdx.x == 0) {
        s_flag[0] = ok;
        if (!ok) __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return s_flag[0] != 0;
  };

#pragma nounroll
  for (int layer = 0; layer < a.n_layer; ++layer) {
    const StepLayer Lv = layer_at(a, layer);
#pragma nounroll
    for (int ph = 0; ph < 5; ++ph) {
      const unsigned epoch = a.epoch0 + (unsigned)(layer * 5 + ph);
      const unsigned wtag = epoch + 1;
      const int jm = gemv_index(ph);
      const int N = jm == 0 ? (a.H + 2 * a.K) * a.h : jm == 2 ? (a.mlp_kind == MDI_MLP_SWIGLU ? 2 * a.F : a.F) : a.d;
      const int Kd = jm == 1 ? a.H * a.h : jm == 3 ? a.F : a.d;
      const BGeo g = make_bgeo(layer_matrix(Lv, jm), N, Kd, a.R[jm], jm == 0 ? a.h : 0, wg, nwg, wave);
      // LayerNorm corrections of this phase's product: [W g | W b], N floats each (QKV's first, then the up product's)
      const float* nc = ln ? a.nc0 + (long)layer * a.nc_stride + (jm == 2 ? 2L * (a.H + 2 * a.K) * a.h : 0L) : nullptr;
      // The per-lane addresses of the exchange vectors do not change from phase to phase; computed once outside
      // the loops they would occupy dozens of registers for the whole launch, so they are derived from a value
      // the compiler cannot see through and are recomputed where they are used.
      int lane_msg = nmsg;
      asm volatile("" : "+v"(lane_msg));
      const tagged_t* xn_in = a.xn;
      tagged_t* xn_out = a.xn;
      tagged_t* ob_l = a.ob;
      tagged_t* ub_l = a.ub;
      bstamp(a, layer, ph, 0);

      // Every kind of phase keeps its registers to itself (tiles in flight, the second operand, attention state are
      // declared inside its branch and given a value on every path), so that the compiler sees them dead elsewhere.
      // Each branch first issues the requests that depend on nothing another workgroup writes - they are in flight
      // while the barrier completes - and then waits for the barrier.
      if (ph == PH_ATTN) {
        // ---- attention: one work item = (message, head group, context split); items dealt round-robin
        AttnState<WT, G> st;
        AttnGeo ga{};
        Tile A, B;
        int pgA[kTile], pgB[kTile];
        BatchView V{};
        int item = wg, slot = 0;
        if (item < a.n_items) {
          while (slot + 1 < m && item >= a.s[slot + 1].item_lo) ++slot;
          V = view_of(a, slot, ob_l);
          ga = make_attn_geo<WT, G>(a, V, item - a.s[slot].item_lo, wave, lane);
          attn_pages(pgA, ga, a, V, 0, wave); attn_pages(pgB, ga, a, V, 1, wave);
          attn_issue<WT>(A, pgA, ga, a, V, Lv.kv, 0, wave); attn_issue<WT>(B, pgB, ga, a, V, Lv.kv, 1, wave);
          if (!barrier(epoch)) return;
          bstamp(a, layer, ph, 1);
          while (true) {
            attn_begin<WT, G>(st, ga, a, V, part, epoch);
            const int nte = ((ga.n_k + kTile - 1) / kTile + 1) & ~1;
            attn_stream<WT, G>(st, A, B, pgA, pgB, ga, a, V, Lv.kv, nte, wave, part);
            attn_to_lds<WT, G>(st, ga, a.h, part, wave);
            attn_finish_pairs<G>(ga, a, V, part, s_flag, epoch);
            item += nwg;
            if (item >= a.n_items) break;
            __syncthreads();                                       // the records in LDS have been read
            while (slot + 1 < m && item >= a.s[slot + 1].item_lo) ++slot;
            V = view_of(a, slot, ob_l);
            ga = make_attn_geo<WT, G>(a, V, item - a.s[slot].item_lo, wave, lane);
            attn_pages(pgA, ga, a, V, 0, wave); attn_pages(pgB, ga, a, V, 1, wave);
            attn_issue<WT>(A, pgA, ga, a, V, Lv.kv, 0, wave); attn_issue<WT>(B, pgB, ga, a, V, Lv.kv, 1, wave);
          }
        } else {
          if (!barrier(epoch)) return;                             // a workgroup without an item still takes part in the barrier
        }
        bstamp(a, layer, ph, 3);
      } else {
        if (ph == PH_QKV || ph == PH_UP) {
          // ---- a product whose second operand stays in registers
          Tile A, B;
          bf16x8 Bv[kResSteps];
          if (g.nks > 8) { res_issue<0>(A, g, 0, wg, nwg, lane); res_issue<1>(B, g, 0, wg, nwg, lane); }
          else { res_issue<0>(A, g, 0, wg, nwg, lane); res_issue<0>(B, g, 1, wg, nwg, lane); }
          if (!barrier(epoch)) return;
          bstamp(a, layer, ph, 1);
          // second operand: this wavefront's column slice of every message, and the messages' 1/rms
          {
            // 1/rms: every workgroup published the sum of squares of the rows it owns, per message
            {
              const int j = threadIdx.x >> 5, c = threadIdx.x & 31;
              float t = 0.f;
              if (j < m) {
                const tagged_t* src = a.ssq + (long)j * nwg;
                for (int w0 = c; w0 < nwg; w0 += 256) {
                  tagged_t raw[8];
#pragma unroll
                  for (int k = 0; k < 8; ++k) raw[k] = w0 + 32 * k < nwg ? ld_raw(src + w0 + 32 * k) : 0ull;
#pragma unroll
                  for (int k = 0; k < 8; ++k)
                    if (w0 + 32 * k < nwg) t += settle(src + w0 + 32 * k, raw[k], epoch, a.spin_limit, a.err);
                }
              }
#pragma unroll
              for (int off = 16; off >= 1; off >>= 1) t += __shfl_xor(t, off, 64);
              if (!ln) {
                if (j < m && c == 0) rscale[j] = 1.f / sqrtf(t / (float)a.d + a.eps);
              } else {
                // LayerNorm: the sums the same way, then 1/std and mean/std
                float u = 0.f;
                if (j < m) {
                  const tagged_t* src = a.ssum + (long)j * nwg;
                  for (int w0 = c; w0 < nwg; w0 += 32) u += settle(src + w0, ld_raw(src + w0), epoch, a.spin_limit, a.err);
                }
#pragma unroll
                for (int off = 16; off >= 1; off >>= 1) u += __shfl_xor(u, off, 64);
                if (j < m && c == 0) {
                  const float mean = u / (float)a.d;
                  const float rstd = 1.f / sqrtf(fmaxf(t / (float)a.d - mean * mean, 0.f) + a.eps);
                  rscale[j] = rstd; rshift[j] = rstd * (mean - rcen[j]);
                  rcen[j] = mean;                      // what the next norm's vector is published around
                }
              }
            }
            // the slice, as published: bf16 pairs of x * gain
            const MDI_GLOBAL tagged_t* bbase = (const MDI_GLOBAL tagged_t*)xn_in + ((long)g.ks0 << 8);
            const uint32_t boff = (uint32_t)((kg << 6) + lane_msg);
            const int last = max(g.nks - 1, 0);
            uint32_t bad = 0u;
#pragma unroll
            for (int h0 = 0; h0 < kResSteps; h0 += 4) {
              if (h0 == 0 || h0 < g.nks) {           // uniform: a batch of steps that lies past the slice costs no round trip
                tagged_t raw[4][4];
#pragma unroll
                for (int s = 0; s < 4; ++s) {        // steps past the slice repeat its last one: every register gets a value
                  const MDI_GLOBAL tagged_t* p = bbase + ((long)min(h0 + s, last) << 8) + boff;
#pragma unroll
                  for (int e = 0; e < 4; ++e) raw[s][e] = ld_word(p + (e << 4));
                }
#pragma unroll
                for (int s = 0; s < 4; ++s) Bv[h0 + s] = take4(raw[s][0], raw[s][1], raw[s][2], raw[s][3], epoch, bad);
              } else {
#pragma unroll
                for (int s = 0; s < 4; ++s) Bv[h0 + s] = Bv[0];
              }
            }
            if (__any(bad != 0u)) {                  // rare: every step again at agent scope, until its words carry the counter
#pragma unroll
              for (int ks = 0; ks < kResSteps; ++ks) {
                const tagged_t* p = xn_in + ((long)(g.ks0 + min(ks, last)) << 8) + boff;
                u32x4 bw;
                bw.x = settle_bits(p, ld_raw(p), epoch, a.spin_limit, a.err); bw.y = settle_bits(p + 16, ld_raw(p + 16), epoch, a.spin_limit, a.err);
                bw.z = settle_bits(p + 32, ld_raw(p + 32), epoch, a.spin_limit, a.err); bw.w = settle_bits(p + 48, ld_raw(p + 48), epoch, a.spin_limit, a.err);
                Bv[ks] = __builtin_bit_cast(bf16x8, bw);
              }
            }
          }
          bstamp(a, layer, ph, 2);
          // the stream: two tiles in flight, each multiplied while the other's rows arrive
          if (g.nks > 8) {
#pragma nounroll
            for (int lb = 0; lb < g.nb_local; ++lb) {
              res_compute<0, false>(A, g, lb, Bv, acc, part, wave, lane);
              res_issue<0>(A, g, lb + 1, wg, nwg, lane);
              res_compute<1, true>(B, g, lb, Bv, acc, part, wave, lane);
              res_issue<1>(B, g, lb + 1, wg, nwg, lane);
            }
          } else {
#pragma nounroll
            for (int lb = 0; lb < g.nb_local; lb += 2) {
              res_compute<0, true>(A, g, lb, Bv, acc, part, wave, lane);
              res_issue<0>(A, g, lb + 2, wg, nwg, lane);
              res_compute<0, true>(B, g, lb + 1, Bv, acc, part, wave, lane);
              res_issue<0>(B, g, lb + 3, wg, nwg, lane);
            }
          }
        } else {
          {
            // ---- a product whose inner dimension is split among workgroups (see KsGeo)
            const KsGeo kq = make_ksgeo(N, Kd, a.str_S, a.str_oct, wg, wave);
            Tile A, B;
            const uint32_t woff = (uint32_t)min(kq.blk * 16 + (lane & 15), N - 1) * (uint32_t)g.row_bytes + (uint32_t)(kg << 4);
            ks_issue(A, kq, g.W, woff, 0);
            ks_issue(B, kq, g.W, woff, 1);
            if (!barrier(epoch)) return;
            bstamp(a, layer, ph, 1);
            // the slice of every message's vector, validated word by word, to LDS as [group of 8 columns][message]
            u32x4* Bs = reinterpret_cast<u32x4*>(part + (a.str_S << 8));
            {
              const tagged_t* bvec = ph == PH_OPROJ ? ob_l : ub_l;
              for (int u0 = threadIdx.x; u0 < kq.nk * 64; u0 += 2 * kStepThreads) {
                tagged_t raw[2][4];
                const tagged_t* src[2];
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                  const int u = min(u0 + r * kStepThreads, kq.nk * 64 - 1);
                  const int gi = u >> 4, n = min(u & 15, m - 1);
                  src[r] = bvec + ((long)(kq.k0 * 4 + gi) << 6) + n;       // pairs 4 (4 k0 + gi) .. + 3, 16 words apart
#pragma unroll
                  for (int e = 0; e < 4; ++e) raw[r][e] = ld_raw(src[r] + (e << 4));
                }
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                  const int u = u0 + r * kStepThreads;
                  u32x4 v;
#pragma unroll
                  for (int e = 0; e < 4; ++e) v[e] = settle_bits(src[r] + (e << 4), raw[r][e], epoch, a.spin_limit, a.err);
                  if (u < kq.nk * 64) { const int gi = u >> 4; Bs[gi * 16 + ((u & 15) ^ (gi & 15))] = v; }
                }
              }
            }
            __syncthreads();
            bstamp(a, layer, ph, 2);
            acc = f32x4{0.f, 0.f, 0.f, 0.f};
            if (kq.live) {                                             // uniform per wavefront
              const int nt = ((kq.nk + 7) >> 3) + 1 & ~1;
#pragma nounroll
              for (int t = 0; t < nt; t += 2) {
                ks_compute(A, kq, Bs, t, lane, acc);
                ks_issue(A, kq, g.W, woff, t + 2);
                ks_compute(B, kq, Bs, t + 1, lane, acc);
                ks_issue(B, kq, g.W, woff, t + 3);
              }
            }
            // the partial of (block, slice), zeros from a slice without columns, to the block's owner
            if (kq.q < a.str_oct && kq.blk < kq.nblk) {
              tagged_t* dst = a.ppart + (((long)kq.blk * kq.S + kq.s) << 8) + (lane << 2);
#pragma unroll
              for (int r = 0; r < 4; ++r) st_tag(dst + r, acc[r], wtag);
            }
            acc = f32x4{0.f, 0.f, 0.f, 0.f};
            bstamp(a, layer, ph, 7);
            // the owner of block wg collects its S partials into the slots the epilogue adds up
            if (wg < kq.nblk) {
              const tagged_t* srcp = a.ppart + ((long)wg * kq.S << 8);
              for (int u0 = threadIdx.x; u0 < (kq.S << 8); u0 += 4 * kStepThreads) {
                tagged_t raw[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) raw[r] = ld_raw(srcp + min(u0 + r * kStepThreads, (kq.S << 8) - 1));
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                  const int u = u0 + r * kStepThreads;
                  const float v = settle(srcp + min(u, (kq.S << 8) - 1), raw[r], wtag, a.spin_limit, a.err);
                  if (u < (kq.S << 8)) part[u] = v;
                }
              }
            }
          }
        }
        bstamp(a, layer, ph, 3);
        __syncthreads();                                             // every wavefront's partial products are in LDS
        bstamp(a, layer, ph, 4);

        // ---- epilogue: one thread per (block, row pair, message)
        const int R = g.R, half = R >> 1;
        if (ph == PH_QKV) {
          for (int e = threadIdx.x; e < g.nb_local * half * m; e += kStepThreads) {
            const int j = e % m, p = (e / m) % half, lb = e / (m * half);
            const int r0 = block_row(g, lb * nwg + wg, p), r1 = r0 + (a.h >> 1);
            float v0 = part_sum(part, lb, p, j) * rscale[j], v1 = part_sum(part, lb, p + half, j) * rscale[j];
            if (ln) { v0 += nc[N + r0] - rshift[j] * nc[r0]; v1 += nc[N + r1] - rshift[j] * nc[r1]; }
            if (Lv.bqkv) { v0 += Lv.bqkv[r0]; v1 += Lv.bqkv[r1]; }
            const int head = r0 / a.h, i = r0 - head * a.h;
            const float2* rope = sl.rope[j];
            if (rope && head < a.H + a.K) {
              const float2 cs = rope[i];
              const float t0 = v0 * cs.x - v1 * cs.y, t1 = v0 * cs.y + v1 * cs.x;
              v0 = t0; v1 = t1;
            }
            char* base = a.slot0 + (long)j * a.slot_stride;
            if (head < a.H) {
              tagged_t* q = (tagged_t*)(base + a.off_q);
              st_tag(q + r0, v0, wtag); st_tag(q + r1, v1, wtag);
            } else {
              // the cache row is for later launches (plain stores); this launch's attention takes the same
              // rounded values from the tagged copy
              const bool is_v = head >= a.H + a.K;
              const int kvh = head - a.H - (is_v ? a.K : 0);
              WT* dst = (WT*)Lv.kv + sl.kv_off[j] + (long)(kvh * 2 + (is_v ? 1 : 0)) * a.pt_h + i;
              Storage<WT>::put(dst, v0); Storage<WT>::put(dst + (a.h >> 1), v1);
              tagged_t* kn = (tagged_t*)(base + a.off_knew) + (long)(is_v ? a.K * a.h : 0) + kvh * a.h + i;
              st_tag(kn, Storage<WT>::get(dst), wtag); st_tag(kn + (a.h >> 1), Storage<WT>::get(dst + (a.h >> 1)), wtag);
            }
          }
        } else if (ph == PH_UP) {
          if (a.mlp_kind == MDI_MLP_SWIGLU) {
            // rows (4q .. 4q + 3) = (gate_f, up_f, gate_f+1, up_f+1): one lane of every wavefront's result holds all four
            const int quads = R >> 2;
            for (int e = threadIdx.x; e < g.nb_local * quads * m; e += kStepThreads) {
              const int j = e % m, qd = (e / m) % quads, lb = e / (m * quads);
              const int r0 = (lb * nwg + wg) * R + 4 * qd;
              if (r0 < g.N) {
                const float* pp = part + ((lb * kStepWaves) << 8) + (((qd << 4) + j) << 2);
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int w = 0; w < kStepWaves; ++w) { const f32x4 t = *reinterpret_cast<const f32x4*>(pp + (w << 8)); v += t; }
                const float rs = rscale[j];
                v *= rs;
                if (ln) {
                  const float sh = rshift[j];
                  v.x += nc[N + r0] - sh * nc[r0]; v.y += nc[N + r0 + 1] - sh * nc[r0 + 1];
                  v.z += nc[N + r0 + 2] - sh * nc[r0 + 2]; v.w += nc[N + r0 + 3] - sh * nc[r0 + 3];
                }
                const float u0 = silu_f(v.x) * v.y, u1 = silu_f(v.z) * v.w;
                st_pair(ub_l + ((r0 >> 2) << 4) + j, pack_bf16x2(u0, u1), wtag);
              }
            }
          } else {
            const bool tanh_form = a.mlp_kind == MDI_MLP_GELU_TANH;
            for (int e = threadIdx.x; e < g.nb_local * half * m; e += kStepThreads) {
              const int j = e % m, p = (e / m) % half, lb = e / (m * half);
              const int r0 = (lb * nwg + wg) * R + 2 * p;
              if (r0 < g.N) {
                float v0 = part_sum(part, lb, 2 * p, j) * rscale[j], v1 = part_sum(part, lb, 2 * p + 1, j) * rscale[j];
                if (ln) { v0 += nc[N + r0] - rshift[j] * nc[r0]; v1 += nc[N + r0 + 1] - rshift[j] * nc[r0 + 1]; }
                if (Lv.bup) { v0 += Lv.bup[r0]; v1 += Lv.bup[r0 + 1]; }
                st_pair(ub_l + ((r0 >> 1) << 4) + j, pack_bf16x2(tanh_form ? gelu_tanh_f(v0) : gelu_erf_f(v0), tanh_form ? gelu_tanh_f(v1) : gelu_erf_f(v1)), wtag);
              }
            }
          }
        } else {
          // residual products: x += W v (+ bias) on the rows this workgroup owns; what leaves is x times the gain of the
          // norm that follows, as bf16 pairs, and this workgroup's share of every message's sum of squares
          const float* bias = ph == PH_OPROJ ? Lv.bo : Lv.bdown;
          const bool last = ph == PH_DOWN && layer == a.n_layer - 1;
          const float* gain = ph == PH_OPROJ ? Lv.ln2_g : advance(Lv.ln1_g, a.w_stride);
          const int n_items = g.nb_local * half * m;
          for (int e = threadIdx.x; e < n_items; e += kStepThreads) {
            const int j = e % m, p = (e / m) % half, lb = e / (m * half);
            const int r0 = (lb * nwg + wg) * R + 2 * p;
            float s2 = 0.f;
            if (r0 < g.N) {
              float* xr = xres + ((lb << 4) + 2 * p) * 16 + j;
              const float d0 = part_sum_n(part, 2 * p, j, a.str_S), d1 = part_sum_n(part, 2 * p + 1, j, a.str_S);
              const float x0 = xr[0] + d0 + (bias ? bias[r0] : 0.f);
              const float x1 = xr[16] + d1 + (bias ? bias[r0 + 1] : 0.f);
              xr[0] = x0; xr[16] = x1;
              if (last) {
                store_kind(sl.out[j], a.act_kind, r0, x0); store_kind(sl.out[j], a.act_kind, r0 + 1, x1);
              } else {
                st_pair(xn_out + ((r0 >> 1) << 4) + j, pack_bf16x2((x0 - rcen[j]) * gain[r0], (x1 - rcen[j]) * gain[r0 + 1]), wtag);
                s2 = x0 * x0 + x1 * x1;
              }
            }
            sq[e] = s2;
          }
          if (!last) {
            __syncthreads();
            if ((int)threadIdx.x < m) {
              float t = 0.f;
              for (int e = threadIdx.x; e < n_items; e += m) t += sq[e];
              st_tag(a.ssq + (long)threadIdx.x * nwg + wg, t, wtag);
              if (ln) {
                float u = 0.f;
                for (int e = threadIdx.x; e < n_items; e += m) {
                  const int p = (e / m) % half, lb = e / (m * half);
                  if ((lb * nwg + wg) * R + 2 * p < g.N) { const float* xr = xres + ((lb << 4) + 2 * p) * 16 + threadIdx.x; u += xr[0] + xr[16]; }
                }
                st_tag(a.ssum + (long)threadIdx.x * nwg + wg, u, wtag);
              }
            }
          }
        }
      }

      // ---- publish: this workgroup is done with the phase
      bstamp(a, layer, ph, 5);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
      bstamp(a, layer, ph, 6);
      if (threadIdx.x == 0) __hip_atomic_store(a.flags + wg * kFlagStride, epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace step_w8

bool step_batch_allow_lds(size_t lds) {
  using namespace step_w8;
  return hipFuncSetAttribute((const void*)k_step_batch<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
         hipFuncSetAttribute((const void*)k_step_batch<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
         hipFuncSetAttribute((const void*)k_step_batch<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
}

void launch_step_batch(hipStream_t s, int G, size_t lds, const BatchArgs& a) {
  using namespace step_w8;
  const dim3 grid(a.nwg), block(kStepThreads);
  if (G == 4) hipLaunchKernelGGL((k_step_batch<4>), grid, block, lds, s, a);
  else if (G == 2) hipLaunchKernelGGL((k_step_batch<2>), grid, block, lds, s, a);
  else hipLaunchKernelGGL((k_step_batch<1>), grid, block, lds, s, a);
}

}  // namespace mdi
