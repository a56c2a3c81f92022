// Decode steps of a whole partition as ONE persistent kernel launch.
//
// A later visit of a sample (Sec. III-D) pushes a single position through every
// local layer; each layer is five dependent matrix-vector / attention phases whose
// inputs are full vectors produced by the previous phase.  Launching them as
// separate kernels leaves the memory system idle at every boundary (drain, launch,
// ramp-up).  Here workgroups stay resident for the whole launch - one of eight
// wavefronts per compute unit for a launch that carries one message, two of four
// wavefronts for a launch that carries the queued messages of several samples
// (Sec. III-A: the input queue; Sec. III-C: several samples in flight).  In the
// latter a set of workgroups takes its messages in turn inside every phase and
// two sets share each compute unit, so that the serial part of one message's
// phase boundary (flags, vector staging, cross-wavefront sums, epilogue) runs
// under other messages' weight streams; every message still makes its own pass
// over the weights.
//
//   * phases are separated by a grid-wide barrier built from per-workgroup epoch
//     flags.  Everything that crosses workgroups (x, q, o, u, attention partials,
//     the newest K/V row, the flags) is written and read with cache-coherent
//     (sc1, agent scope) stores and loads, so the barrier needs no L2
//     write-back/invalidate.  Because such a store can be acknowledged before
//     every compute die sees it, each exchanged value carries the counter of the
//     phase that wrote it in the same 8-byte word and readers reload until the
//     counter is the expected one; the flags only guard against overwriting.
//   * weight and KV-cache addresses do not depend on activations, so every
//     wavefront keeps two register tiles of 16-byte loads in flight and, while it
//     finishes a phase, already issues the first two tiles of the NEXT phase; the
//     barrier latency and the vector staging after it are covered by those loads.
//   * the rows a workgroup owns in a phase form one flat sequence of (row pair,
//     1-KiB chunk) items dealt round-robin to its wavefronts.  At any moment the
//     workgroup therefore reads consecutive KiB of a row pair (DRAM sees a few
//     wide sequential streams instead of thousands of narrow ones), and the
//     wavefronts stay balanced whatever the shape.  A wavefront's share of a pair
//     goes to an LDS slot of its own; slots are summed in wavefront order
//     (deterministic, no float atomics; the order depends on the number of
//     wavefronts, which is why launches of one and of several messages may differ
//     in the last bits).
//   * in a launch with two sets of workgroups, each workgroup compares once per
//     phase the work it has left with that of the other set and takes the higher
//     wave priority when it has more: left alone, the set that was dispatched
//     first is served first by a compute unit's memory pipeline and finishes a
//     fifth earlier.
//
// Every spin is bounded: a workgroup that waits longer than `spin_limit` polls
// raises the partition's error flag and leaves, and so does every other one.
//
// This file is the kernel's body; step_w4.hip and step_w8.hip compile it for workgroups of four and of
// eight wavefronts (MDI_STEP_WAVES), each in a namespace of its own with a launcher of its own.
#include "device_utils.h"

#ifndef MDI_STEP_WAVES
#error "include from step_w4.hip / step_w8.hip, which define MDI_STEP_WAVES"
#endif
#define MDI_STEP_CAT2(a, b) a##b
#define MDI_STEP_CAT(a, b) MDI_STEP_CAT2(a, b)

namespace mdi {
namespace MDI_STEP_CAT(step_w, MDI_STEP_WAVES) {

constexpr int kStepWaves = MDI_STEP_WAVES;       // wavefronts per workgroup
constexpr int kStepThreads = 64 * kStepWaves;

#define MDI_GLOBAL __attribute__((address_space(1)))

constexpr int kTile = 4;                 // items per register tile (two 16-byte loads each)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
struct Tile { u32x4 r[2 * kTile]; };

// Tagged exchange.  A workgroup that has seen every flag of a barrier may still be ahead of the data
// another compute die wrote before raising its flag (a store is acknowledged before every die can
// read it back), so the data validates itself: value and the writing phase's counter travel in one
// 8-byte store, and a reader that finds another counter simply loads again.  Flags then only protect
// buffers from being overwritten while still in use, which needs no ordering between stores.
__device__ __forceinline__ void st_tag(tagged_t* p, float v, unsigned tag) {
  __hip_atomic_store(p, ((tagged_t)tag << 32) | (tagged_t)__float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ tagged_t ld_raw(const tagged_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float tag_value(tagged_t u) { return __uint_as_float((uint32_t)u); }
// Returns the value once its tag is `tag`; gives up (error flag) after spin_limit reloads.
__device__ __forceinline__ float settle(const tagged_t* p, tagged_t u, unsigned tag, int spin_limit, int* err) {
  int it = 0;
  while ((uint32_t)(u >> 32) != tag) {
    if (++it > spin_limit) { __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
    __builtin_amdgcn_s_sleep(1);
    u = ld_raw(p);
  }
  return tag_value(u);
}
__device__ __forceinline__ float ld_tag(const tagged_t* p, unsigned tag, int spin_limit, int* err) {
  return settle(p, ld_raw(p), tag, spin_limit, err);
}

template <typename T> struct Unpack;
template <> struct Unpack<float> {
  __device__ static __forceinline__ void go(const u32x4& t, float (&v)[4]) {
    v[0] = __uint_as_float(t.x); v[1] = __uint_as_float(t.y); v[2] = __uint_as_float(t.z); v[3] = __uint_as_float(t.w);
  }
};
template <> struct Unpack<bf16_t> {
  __device__ static __forceinline__ void go(const u32x4& t, float (&v)[8]) {
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
    v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xFFFF0000u);
    v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xFFFF0000u);
  }
};

enum StepPhase { PH_QKV = 0, PH_ATTN = 1, PH_OPROJ = 2, PH_UP = 3, PH_DOWN = 4 };

// optional timeline for profiling: thread 0 of every workgroup records a 100 MHz timestamp
__device__ __forceinline__ void stamp(const StepArgs& a, const StepSlot& S, int layer, int ph, int k) {
  if (S.trace && threadIdx.x == 0)
    S.trace[(((long)(blockIdx.x % a.nwg) * a.n_layer + layer) * 5 + ph) * 8 + k] = wall_clock64();
}


// LDS map (floats): [0,16) reduction scratch, [16,20) flags, [20,56) phase geometry,
// [128, 128+part_floats) pair partials, then the vector.
constexpr int kLdsPart = 128;
__device__ __forceinline__ float* lds_red() { extern __shared__ float smem[]; return smem; }
__device__ __forceinline__ int* lds_flag() { extern __shared__ float smem[]; return (int*)(smem + 16); }
__device__ __forceinline__ float* lds_part() { extern __shared__ float smem[]; return smem + kLdsPart; }
__device__ __forceinline__ float* lds_vec(int part_floats) { extern __shared__ float smem[]; return smem + kLdsPart + part_floats; }

// ---------------------------------------------------------------------------
// vector staging: n floats written earlier in this launch by other workgroups -> LDS
// With gain != nullptr (RMSNorm) the staged values are x[i] * gain[i] and the return value is this
// thread's share of sum(x^2); the common factor 1/rms is applied to the finished dot products.
// The first batch of eight values per thread (and their gains) may have been requested earlier, while the
// workgroup was finishing its previous phase (`pre`); values that were not there yet carry another tag and are
// simply loaded again.
__device__ __forceinline__ float stage_coherent(const tagged_t* src, int n, float* xs, const float* gain, unsigned tag,
                                                int spin_limit, int* err, bool pre, const tagged_t (&praw)[8],
                                                const float (&pgain)[8]) {
  float ss = 0.f;
  for (int i0 = threadIdx.x; i0 < n; i0 += 8 * kStepThreads) {
    const bool early = pre && i0 == (int)threadIdx.x;
    tagged_t raw[8];
    float gv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {                      // eight loads in flight per thread
      const int i = i0 + j * kStepThreads;
      raw[j] = early ? praw[j] : (i < n ? ld_raw(src + i) : 0ull);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = i0 + j * kStepThreads;
      gv[j] = early ? pgain[j] : ((gain && i < n) ? gain[i] : 1.f);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = i0 + j * kStepThreads;
      if (i < n) {
        const float x = settle(src + i, raw[j], tag, spin_limit, err);
        ss += x * x;
        xs[i] = gain ? x * gv[j] : x;
      }
    }
  }
  return ss;
}

__device__ __forceinline__ void normalise(float* xs, int n, int norm_kind, float eps, const float* g, const float* b, float* red) {
  if (norm_kind == MDI_NORM_LAYERNORM) {
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += kStepThreads) s += xs[i];
    const float mean = block_sum(s, red) / (float)n;
    float s2 = 0.f;
    for (int i = threadIdx.x; i < n; i += kStepThreads) { const float c = xs[i] - mean; s2 += c * c; }
    const float rstd = 1.f / sqrtf(block_sum(s2, red) / (float)n + eps);
    for (int i = threadIdx.x; i < n; i += kStepThreads) xs[i] = (xs[i] - mean) * rstd * g[i] + (b ? b[i] : 0.f);
  } else {
    float s2 = 0.f;
    for (int i = threadIdx.x; i < n; i += kStepThreads) s2 += xs[i] * xs[i];
    const float rstd = 1.f / sqrtf(block_sum(s2, red) / (float)n + eps);
    for (int i = threadIdx.x; i < n; i += kStepThreads) xs[i] = xs[i] * rstd * g[i];
  }
}

// ---------------------------------------------------------------------------
// GEMV phase geometry (all values uniform across the wavefront)
struct Geo {
  const void* W;
  int N, units, cpp;     // rows, 16-byte units per row, 64-lane chunks per row
  int rope_h;            // > 0: pair (i, i + h/2) inside heads of size h; 0: rows (2p, 2p + 1)
  int p_lo, n_pl;        // this workgroup owns n_pl pairs: blocks of 2^bshift consecutive pairs, block b of the
  int bshift, nwg;       // matrix going to workgroup b % nwg (p_lo = workgroup index).  At any moment the grid
                         // reads one contiguous window of the matrix, and a workgroup stays >= 64 KiB in place.
  int n_k;               // this wavefront's items: item k is flat index wave + 8k, flat = pair * cpp + chunk
  int dq, dr;            // 8 / cpp and 8 % cpp: how (pair, chunk) moves from one item to the next
  int rsh, rmask, rmul, rstep;   // first row of pair p = (p >> rsh) * rmul + (p & rmask); its partner rstep rows on
};
// The two pairings as one branch-free formula (head sizes are powers of two): rows (2p, 2p + 1), or RoPE partners
// (i, i + h/2) inside heads of h rows.
__device__ __forceinline__ void geo_rows(Geo& g) {
  if (g.rope_h) {
    const int half = g.rope_h >> 1;
    g.rsh = 31 - __builtin_clz(half); g.rmask = half - 1; g.rmul = g.rope_h; g.rstep = half;
  } else {
    g.rsh = 0; g.rmask = 0; g.rmul = 2; g.rstep = 1;
  }
}

template <typename WT>
__device__ __forceinline__ Geo make_geo(const void* W, int N, int Kd, int rope_h, int wg, int nwg, int wave) {
  constexpr int V = Storage<WT>::kVec;
  Geo g;
  g.W = W; g.N = N; g.units = Kd / V; g.cpp = (g.units + 63) >> 6; g.rope_h = rope_h;
  const int pairs = (N + 1) >> 1;
  g.p_lo = wg; g.nwg = nwg;
  g.bshift = 0;
  const long pair_bytes = 2L * Kd * (long)sizeof(WT);
  // larger blocks only while they still divide evenly among the workgroups (balance comes first)
  while (g.bshift < 3 && (pair_bytes << g.bshift) < 65536 && pairs % (nwg << (g.bshift + 1)) == 0) ++g.bshift;
  const int B = 1 << g.bshift, nblk = (pairs + B - 1) >> g.bshift;
  const int own = nblk > wg ? (nblk - wg + nwg - 1) / nwg : 0;
  g.n_pl = own * B;
  if (own > 0 && wg + (own - 1) * nwg == nblk - 1) g.n_pl -= nblk * B - pairs;   // the matrix's last block may be short
  const int flat = g.n_pl * g.cpp;
  g.n_k = flat > wave ? (flat - wave + kStepWaves - 1) / kStepWaves : 0;
  g.dq = kStepWaves / g.cpp; g.dr = kStepWaves - g.dq * g.cpp;
  geo_rows(g);
  return g;
}
__device__ __forceinline__ void geo_next(const Geo& g, int& pl, int& c) {
  c += g.dr; pl += g.dq;
  if (c >= g.cpp) { c -= g.cpp; ++pl; }
}
__device__ __forceinline__ int geo_pair(const Geo& g, int pl) {     // local pair index -> pair index in the matrix
  return ((((pl >> g.bshift) * g.nwg) + g.p_lo) << g.bshift) + (pl & ((1 << g.bshift) - 1));
}
__device__ __forceinline__ int geo_row(const Geo& g, int p, int j) {
  return (p >> g.rsh) * g.rmul + (p & g.rmask) + j * g.rstep;
}

// the step's own input (token embedding + learned position, or the previous stage's activation)
template <typename WT>
__device__ __forceinline__ void stage_input(const StepArgs& a, const StepSlot& S, float* xs, const Geo& gres, unsigned tag) {
  const int n = a.d;
  if (S.in_kind == IN_TOKEN) {
    const long tok = checked_token(S.in, 0, a.vocab, a.err);
    for (int i = threadIdx.x; i < n; i += kStepThreads) {
      float v = Storage<WT>::get((const WT*)a.wte + tok * n + i);
      if (a.wpe) v += Storage<WT>::get((const WT*)a.wpe + (long)S.pos * n + i);
      xs[i] = v;
    }
  } else {
    for (int i = threadIdx.x; i < n; i += kStepThreads) xs[i] = load_kind(S.in, S.in_kind, i);
  }
  __syncthreads();
  // rows this workgroup owns in the residual phases get their starting value
  for (int pl = threadIdx.x; pl < gres.n_pl; pl += kStepThreads) {
    const int r = 2 * geo_pair(gres, pl);
    st_tag(S.xres + r, xs[r], tag);
    if (r + 1 < n) st_tag(S.xres + r + 1, xs[r + 1], tag);
  }
}

// Where a wavefront stands in its items (local pair, chunk of the row): tiles are issued, and multiplied, in order, so
// each side keeps a cursor and moves it item by item instead of dividing the item index again for every tile.
struct Cursor {
  int pl, c;
  int row_pl;                          // the local pair whose row addresses b0, b1 hold (-1: none yet)
  const MDI_GLOBAL u32x4 *b0, *b1;     // (issue side only) a pair's rows stay the same over its chunks
};
__device__ __forceinline__ Cursor cursor_start(const Geo& g, int wave) {
  Cursor cur;
  cur.pl = wave / g.cpp; cur.c = wave - cur.pl * g.cpp;
  cur.row_pl = -1; cur.b0 = nullptr; cur.b1 = nullptr;
  return cur;
}

// Every call issues exactly 2 * kTile loads, whatever the geometry: a fixed number of loads per tile is what lets
// the compiler wait for one tile while the next stays in flight (its counters cannot follow conditional loads).
// Items past the end of the wavefront's share need no case of their own: their pair index lies past the matrix and
// is clamped to its last row, lanes past the end of a row read the row's first bytes; gemv_compute skips the former
// and masks the latter or multiplies them by zeros.  All of this is scalar arithmetic, which the wavefronts of a
// compute unit share one unit for, on the critical path of a phase's start: it is kept short.
__device__ __forceinline__ void gemv_issue(Tile& t, const Geo& g, Cursor& cur, int lane) {
  const MDI_GLOBAL u32x4* W = (const MDI_GLOBAL u32x4*)g.W;
  int pl = cur.pl, c = cur.c;
#pragma unroll
  for (int s = 0; s < kTile; ++s) {
    if (pl != cur.row_pl) {                                     // uniform; long rows keep a pair for several items
      const int r0 = min(geo_row(g, geo_pair(g, pl), 0), g.N - 1), r1 = min(r0 + g.rstep, g.N - 1);
      cur.b0 = W + (long)r0 * g.units;
      cur.b1 = W + (long)r1 * g.units;
      cur.row_pl = pl;
    }
    const int off = c * 64 + (c * 64 + lane < g.units ? lane : 0);   // unit 0 of the chunk always exists
    t.r[2 * s] = cur.b0[off];
    t.r[2 * s + 1] = cur.b1[off];
    geo_next(g, pl, c);
  }
  cur.pl = pl; cur.c = c;
}

// kPadded: the caller has zeros in xs behind the vector, up to a whole number of 64-lane chunks, so the lanes past the
// end of a row (which hold the row's first bytes) multiply by zero and need no case of their own.
template <typename WT, bool kPadded>
__device__ __forceinline__ void gemv_compute(const Tile& t, const Geo& g, int ti, Cursor& cur, int wave, int lane, const float* xs,
                                             float* part, float& acc0, float& acc1) {
  constexpr int V = Storage<WT>::kVec;
  int pl = cur.pl, c = cur.c;
#pragma unroll
  for (int s = 0; s < kTile; ++s) {
    int npl = pl, nc = c;
    geo_next(g, npl, nc);
    const int k = ti * kTile + s;
    if (k < g.n_k) {                                         // uniform
      const int unit = c * 64 + lane;
      if (kPadded || unit < g.units) {
        float w0[V], w1[V], xv[V];
        Unpack<WT>::go(t.r[2 * s], w0);
        Unpack<WT>::go(t.r[2 * s + 1], w1);
#pragma unroll
        for (int e = 0; e < V; e += 4) {
          const float4 q4 = *reinterpret_cast<const float4*>(xs + unit * V + e);
          xv[e] = q4.x; xv[e + 1] = q4.y; xv[e + 2] = q4.z; xv[e + 3] = q4.w;
        }
#pragma unroll
        for (int e = 0; e < V; ++e) { acc0 = fmaf(w0[e], xv[e], acc0); acc1 = fmaf(w1[e], xv[e], acc1); }
      }
      if (npl != pl || k == g.n_k - 1) {                     // this wavefront's share of the pair is complete
        const float r0 = wave_sum_to_lane63(acc0), r1 = wave_sum_to_lane63(acc1);
        if (lane == 63) { part[(pl * 2) * kStepWaves + wave] = r0; part[(pl * 2 + 1) * kStepWaves + wave] = r1; }
        acc0 = 0.f; acc1 = 0.f;
      }
    }
    pl = npl; c = nc;
  }
  cur.pl = pl; cur.c = c;
}

// Sums the wavefront slots of every pair and applies the phase's epilogue.
template <typename WT>
__device__ __forceinline__ void gemv_finish(int ph, const Geo& g, const StepLayer* Lp, int layer, const StepArgs& a, const StepSlot& S, const float* part,
                                            float row_scale, tagged_t x0_pre, tagged_t x1_pre, unsigned epoch) {
  const unsigned wtag = epoch + 1;                            // what this phase writes carries the next counter
  const StepLayer& L = *Lp;
  __syncthreads();                                           // all wavefronts' partials are in LDS
  stamp(a, S, layer, ph, 4);
  for (int pl = threadIdx.x; pl < g.n_pl; pl += kStepThreads) {
    float v0 = 0.f, v1 = 0.f;
#pragma unroll
    for (int w = 0; w < kStepWaves; ++w) { v0 += part[(pl * 2) * kStepWaves + w]; v1 += part[(pl * 2 + 1) * kStepWaves + w]; }
    v0 *= row_scale; v1 *= row_scale;
    const int p = geo_pair(g, pl);
    const int r0 = geo_row(g, p, 0), r1 = geo_row(g, p, 1);
    if (ph == PH_QKV) {
      if (L.bqkv) { v0 += L.bqkv[r0]; v1 += L.bqkv[r1]; }
      const int head = r0 / a.h, i = r0 - head * a.h;
      if (S.rope && head < a.H + a.K) {
        const float2 cs = S.rope[i];
        const float t0 = v0 * cs.x - v1 * cs.y, t1 = v0 * cs.y + v1 * cs.x;
        v0 = t0; v1 = t1;
      }
      if (head < a.H) {
        st_tag(S.q + r0, v0, wtag); st_tag(S.q + r1, v1, wtag);
      } else {
        // the cache row is for later launches (plain stores); this launch's attention takes the same
        // rounded values from the tagged copy
        const bool is_v = head >= a.H + a.K;
        const int kvh = head - a.H - (is_v ? a.K : 0);
        WT* dst = (WT*)L.kv + S.kv_tok_off + (long)(kvh * 2 + (is_v ? 1 : 0)) * a.pt_h + i;
        Storage<WT>::put(dst, v0); Storage<WT>::put(dst + (a.h >> 1), v1);
        tagged_t* kn = S.knew + (long)(is_v ? a.K * a.h : 0) + kvh * a.h + i;
        st_tag(kn, Storage<WT>::get(dst), wtag); st_tag(kn + (a.h >> 1), Storage<WT>::get(dst + (a.h >> 1)), wtag);
      }
    } else if (ph == PH_UP) {
      if (a.mlp_kind == MDI_MLP_SWIGLU) {
        st_tag(S.u + p, silu_f(v0) * v1, wtag);              // rows (2f, 2f+1) = (gate_f, up_f)
      } else {
        if (L.bup) { v0 += L.bup[r0]; if (r1 < g.N) v1 += L.bup[r1]; }
        const bool tanh_form = a.mlp_kind == MDI_MLP_GELU_TANH;
        st_tag(S.u + r0, tanh_form ? gelu_tanh_f(v0) : gelu_erf_f(v0), wtag);
        if (r1 < g.N) st_tag(S.u + r1, tanh_form ? gelu_tanh_f(v1) : gelu_erf_f(v1), wtag);
      }
    } else {                                                  // residual phases
      const float* bias = ph == PH_OPROJ ? L.bo : L.bdown;
      const bool last = ph == PH_DOWN && layer == a.n_layer - 1;
      const bool two = r1 < g.N;
      // rows of the first kStepThreads pairs were fetched before the stream
      const bool pre = pl == (int)threadIdx.x;
      // this workgroup wrote these rows itself: two phases ago (output projection) or one (down projection)
      const unsigned rtag = ph == PH_OPROJ ? epoch - 2 : epoch - 1;
      const float x0 = settle(S.xres + r0, pre ? x0_pre : ld_raw(S.xres + r0), rtag, a.spin_limit, a.err);
      const float x1 = two ? settle(S.xres + r1, pre ? x1_pre : ld_raw(S.xres + r1), rtag, a.spin_limit, a.err) : 0.f;
      v0 += x0 + (bias ? bias[r0] : 0.f);
      st_tag(S.xres + r0, v0, wtag);
      if (last) store_kind(S.act_out, a.act_kind, r0, v0);
      if (two) {
        v1 += x1 + (bias ? bias[r1] : 0.f);
        st_tag(S.xres + r1, v1, wtag);
        if (last) store_kind(S.act_out, a.act_kind, r1, v1);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// attention phase geometry
struct AttnGeo {
  bool active;
  int hg, split, kvh, s0, s1, s1p;
  int L, tpw, sub, hoff;
  int n_k;                // this wavefront's steps: step k covers tokens s0 + (8k + wave) * tpw ..
  float f2, f4, f8, f16;  // 1 when a position's values are spread over at least that many lanes, else 0
  int pt_sh;              // log2(tokens per page) when that is a power of two, else -1 ...
  unsigned pt_magic;      // ... and then position / page size = high word of position * pt_magic (exact while
                          // position * page size < 2^32, which creating the partition checks)
};
// Sum over the g.L lanes that share a position, in every one of them.  Inside a row of 16 lanes every step is taken,
// multiplied by the step's flag: no branch on the (run-time) lane count in the streaming loop.  Same order of
// additions as group_sum.
template <int CTRL>
__device__ __forceinline__ float dpp_add_if(float v, float flag) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false);
  return fmaf(__int_as_float(moved), flag, v);
}
__device__ __forceinline__ float group_sum_lanes(float v, const AttnGeo& g) {
  v = dpp_add_if<kDppXor1>(v, g.f2);
  v = dpp_add_if<kDppXor2>(v, g.f4);
  v = dpp_add_if<kDppHalfMirror>(v, g.f8);
  v = dpp_add_if<kDppMirror>(v, g.f16);
  if (g.L >= 32) v += __shfl_xor(v, 16, 64);
  if (g.L >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}
__device__ __forceinline__ int page_of(const AttnGeo& g, int tok) {
  return g.pt_sh >= 0 ? tok >> g.pt_sh : (int)__umulhi((unsigned)tok, g.pt_magic);
}

template <typename WT, int G, typename AR, typename SL>
__device__ __forceinline__ AttnGeo make_attn_geo(const AR& a, const SL& S, int wg, int wave, int lane) {
  constexpr int V = Storage<WT>::kVec;
  AttnGeo g;
  g.L = a.h / V; g.tpw = 64 / g.L; g.sub = lane / g.L; g.hoff = (lane % g.L) * V;
  g.active = wg < a.n_hg * S.n_splits;
  g.hg = g.active ? wg % a.n_hg : 0;
  g.split = g.active ? wg / a.n_hg : 0;
  g.kvh = (g.hg * G) / (a.H / a.K);
  g.s0 = g.split * S.chunk;
  g.s1 = min(S.ctx, g.s0 + S.chunk);
  g.s1p = min(g.s1, S.ctx - 1);                               // the newest row is written in this launch
  const int steps = g.active && g.s1p > g.s0 ? (g.s1p - g.s0 + g.tpw - 1) / g.tpw : 0;
  g.n_k = steps > wave ? (steps - wave + kStepWaves - 1) / kStepWaves : 0;
  g.f2 = g.L >= 2 ? 1.f : 0.f; g.f4 = g.L >= 4 ? 1.f : 0.f; g.f8 = g.L >= 8 ? 1.f : 0.f; g.f16 = g.L >= 16 ? 1.f : 0.f;
  g.pt_sh = (a.pt & (a.pt - 1)) == 0 ? __builtin_ctz(a.pt) : -1;
  g.pt_magic = g.pt_sh >= 0 ? 0u : 0xFFFFFFFFu / (unsigned)a.pt + 1u;
  return g;
}

// Page numbers of the tokens of tile ti (slots without a token take token 0's).  The table entries of every position
// before the newest were written by earlier launches, so they are fetched a tile pair ahead of the rows they locate:
// a row's address then never waits for a table look-up.
template <typename AR, typename SL>
__device__ __forceinline__ void attn_pages(int (&pg)[kTile], const AttnGeo& g, const AR& a, const SL& S, int ti, int wave) {
  const MDI_GLOBAL int32_t* table = (const MDI_GLOBAL int32_t*)S.table;
#pragma unroll
  for (int s = 0; s < kTile; ++s) {
    const int k = ti * kTile + s;
    int tok = g.s0 + (k * kStepWaves + wave) * g.tpw + g.sub;
    if (!(k < g.n_k && tok < g.s1p)) tok = 0;
    pg[s] = __hip_atomic_load(table + page_of(g, tok), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// Issues exactly 2 * kTile row loads (see gemv_issue) for tile ti, whose page numbers are in pg, then asks for the
// page numbers of the tile that goes into the same registers next; slots without a token re-read token 0.
template <typename WT, typename AR, typename SL>
__device__ __forceinline__ void attn_issue(Tile& t, int (&pg)[kTile], const AttnGeo& g, const AR& a, const SL& S, const void* pool_,
                                           int ti, int wave) {
  const MDI_GLOBAL WT* pool = (const MDI_GLOBAL WT*)pool_;
#pragma unroll
  for (int s = 0; s < kTile; ++s) {
    const int k = ti * kTile + s;
    int tok = g.s0 + (k * kStepWaves + wave) * g.tpw + g.sub;
    if (!(k < g.n_k && tok < g.s1p)) tok = 0;
    const int in_page = tok - page_of(g, tok) * a.pt;
    const MDI_GLOBAL WT* kp = pool + ((long)pg[s] * a.K + g.kvh) * 2 * a.pt_h + (long)in_page * a.h + g.hoff;
    t.r[2 * s] = *reinterpret_cast<const MDI_GLOBAL u32x4*>(kp);
    t.r[2 * s + 1] = *reinterpret_cast<const MDI_GLOBAL u32x4*>(kp + a.pt_h);
  }
  attn_pages(pg, g, a, S, ti + 2, wave);
}

template <typename WT, int G>
struct AttnState {
  float m[G], l[G], o[G][Storage<WT>::kVec];
};

template <typename WT, int G>
__device__ __forceinline__ void attn_update_f(AttnState<WT, G>& st, const AttnGeo& g, int h, const float (&kf)[Storage<WT>::kVec],
                                              const float (&vf)[Storage<WT>::kVec], bool valid, const float* qs) {
  constexpr int V = Storage<WT>::kVec;
#pragma unroll
  for (int gi = 0; gi < G; ++gi) {
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < V; e += 4) {
      const float4 q4 = *reinterpret_cast<const float4*>(qs + gi * h + g.hoff + e);
      s = fmaf(q4.x, kf[e], s); s = fmaf(q4.y, kf[e + 1], s); s = fmaf(q4.z, kf[e + 2], s); s = fmaf(q4.w, kf[e + 3], s);
    }
    s = group_sum_lanes(s, g);
    if (valid) {
      const float mn = fmaxf(st.m[gi], s);
      const float alpha = __expf(st.m[gi] - mn), p = __expf(s - mn);
      st.m[gi] = mn;
      st.l[gi] = st.l[gi] * alpha + p;
#pragma unroll
      for (int e = 0; e < V; ++e) st.o[gi][e] = st.o[gi][e] * alpha + p * vf[e];
    }
  }
}

template <typename WT, int G>
__device__ __forceinline__ void attn_update(AttnState<WT, G>& st, const AttnGeo& g, int h, const u32x4& kq, const u32x4& vq,
                                            bool valid, const float* qs) {
  float kf[Storage<WT>::kVec], vf[Storage<WT>::kVec];
  Unpack<WT>::go(kq, kf);
  Unpack<WT>::go(vq, vf);
  attn_update_f<WT, G>(st, g, h, kf, vf, valid, qs);
}

// One tile = kTile cached positions per lane group.  The scores of all of them first, then ONE rescaling of the running
// sums to the new maximum, then the weighted values: a rescaling per position (as attn_update_f does for the single
// newest row) costs as many multiplications as the values themselves.
template <typename WT, int G>
__device__ __forceinline__ void attn_compute(AttnState<WT, G>& st, const Tile& t, const AttnGeo& g, int h, int ti, int wave,
                                             const float* qs) {
  constexpr int V = Storage<WT>::kVec;
  float sc[kTile][G];
  bool ok[kTile];
#pragma unroll
  for (int s = 0; s < kTile; ++s) {
    const int k = ti * kTile + s;
    const int tok = g.s0 + (k * kStepWaves + wave) * g.tpw + g.sub;
    ok[s] = k < g.n_k && tok < g.s1p;
    if (k < g.n_k) {                                     // uniform
      float kf[V];
      Unpack<WT>::go(t.r[2 * s], kf);
#pragma unroll
      for (int gi = 0; gi < G; ++gi) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < V; e += 4) {
          const float4 q4 = *reinterpret_cast<const float4*>(qs + gi * h + g.hoff + e);
          d = fmaf(q4.x, kf[e], d); d = fmaf(q4.y, kf[e + 1], d); d = fmaf(q4.z, kf[e + 2], d); d = fmaf(q4.w, kf[e + 3], d);
        }
        sc[s][gi] = group_sum_lanes(d, g);
      }
    } else {
#pragma unroll
      for (int gi = 0; gi < G; ++gi) sc[s][gi] = -1e30f;
    }
  }
#pragma unroll
  for (int gi = 0; gi < G; ++gi) {
    float mn = st.m[gi];
#pragma unroll
    for (int s = 0; s < kTile; ++s) mn = ok[s] ? fmaxf(mn, sc[s][gi]) : mn;
    const float alpha = __expf(st.m[gi] - mn);
    st.m[gi] = mn;
    st.l[gi] *= alpha;
#pragma unroll
    for (int e = 0; e < V; ++e) st.o[gi][e] *= alpha;
  }
#pragma unroll
  for (int s = 0; s < kTile; ++s) {
    if (ti * kTile + s < g.n_k) {                        // uniform
      float vf[V];
      Unpack<WT>::go(t.r[2 * s + 1], vf);
#pragma unroll
      for (int gi = 0; gi < G; ++gi) {
        const float p = ok[s] ? __expf(sc[s][gi] - st.m[gi]) : 0.f;
        st.l[gi] += p;
#pragma unroll
        for (int e = 0; e < V; ++e) st.o[gi][e] = fmaf(p, vf[e], st.o[gi][e]);
      }
    }
  }
}

// The streaming loop of the attention phase: two tiles in flight, each multiplied while the other's rows arrive.
template <typename WT, int G, typename AR, typename SL>
__device__ __forceinline__ void attn_stream(AttnState<WT, G>& st, Tile& A, Tile& B, int (&pgA)[kTile], int (&pgB)[kTile], const AttnGeo& ga,
                                            const AR& a, const SL& S, const void* kv, int nte, int wave, const float* xs) {
#pragma nounroll
  for (int t = 0; t < nte; t += 2) {
    attn_compute<WT, G>(st, A, ga, a.h, t, wave, xs);
    attn_issue<WT>(A, pgA, ga, a, S, kv, t + 2, wave);
    attn_compute<WT, G>(st, B, ga, a.h, t + 1, wave, xs);
    attn_issue<WT>(B, pgB, ga, a, S, kv, t + 3, wave);
  }
}

// queries into LDS (pre-scaled); the newest position through coherent loads
template <typename WT, int G, typename AR, typename SL>
__device__ __forceinline__ void attn_begin(AttnState<WT, G>& st, const AttnGeo& g, const AR& a, const SL& S, float* qs, unsigned epoch) {
  constexpr int V = Storage<WT>::kVec;
#pragma unroll
  for (int gi = 0; gi < G; ++gi) {
    st.m[gi] = -1e30f; st.l[gi] = 0.f;
#pragma unroll
    for (int e = 0; e < V; ++e) st.o[gi][e] = 0.f;
  }
  if (g.active)
    for (int i = threadIdx.x; i < G * a.h; i += kStepThreads)
      qs[i] = ld_tag(S.q + (long)g.hg * G * a.h + i, epoch, a.spin_limit, a.err) * a.scale;
  __syncthreads();
  if (g.active && g.s1 == S.ctx && threadIdx.x < 64) {
    // the newest position: its K/V row (already rounded to the storage type) from the tagged copy
    float kf[V], vf[V];
#pragma unroll
    for (int e = 0; e < V; ++e) { kf[e] = 0.f; vf[e] = 0.f; }
    if (g.sub == 0) {
      const tagged_t* kn = S.knew + g.kvh * a.h + g.hoff;
      const tagged_t* vn = kn + (long)a.K * a.h;
#pragma unroll
      for (int e = 0; e < V; ++e) { kf[e] = ld_tag(kn + e, epoch, a.spin_limit, a.err); vf[e] = ld_tag(vn + e, epoch, a.spin_limit, a.err); }
    }
    attn_update_f<WT, G>(st, g, a.h, kf, vf, g.sub == 0, qs);
  }
}

// Folds the wavefront's token sub-groups, leaves one record per (wavefront, head) in LDS.
template <typename WT, int G>
__device__ __forceinline__ void attn_to_lds(AttnState<WT, G>& st, const AttnGeo& g, int h, float* sm, int wave) {
  constexpr int V = Storage<WT>::kVec;
  const int rec = h + 2;
  for (int off = g.L; off < 64; off <<= 1) {
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
      const float mo = __shfl_xor(st.m[gi], off, 64), lo = __shfl_xor(st.l[gi], off, 64);
      const float mn = fmaxf(st.m[gi], mo);
      const float sa = __expf(st.m[gi] - mn), sb = __expf(mo - mn);
      st.l[gi] = st.l[gi] * sa + lo * sb;
#pragma unroll
      for (int e = 0; e < V; ++e) st.o[gi][e] = st.o[gi][e] * sa + __shfl_xor(st.o[gi][e], off, 64) * sb;
      st.m[gi] = mn;
    }
  }
  __syncthreads();                                             // queries in LDS are no longer needed
  if (g.sub == 0) {                                            // [wave][g][h + 2]
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
      float* r = sm + (wave * G + gi) * rec;
#pragma unroll
      for (int e = 0; e < V; ++e) r[g.hoff + e] = st.o[gi][e];
      if (g.hoff == 0) { r[h] = st.m[gi]; r[h + 1] = st.l[gi]; }
    }
  }
  __syncthreads();
}

// Wavefront records -> split partial (or the final output when there is one split);
// the last workgroup of a head group to arrive folds the splits in split order.
template <int G, typename AR, typename SL>
__device__ __forceinline__ void attn_finish(const AttnGeo& g, const AR& a, const SL& S, const float* sm, int* s_flag, unsigned epoch) {
  const unsigned wtag = epoch + 1;
  const int h = a.h, rec = h + 2;
  if (!g.active) return;
  const bool single = S.n_splits == 1;
  for (int idx = threadIdx.x; idx < G * h; idx += kStepThreads) {
    const int gi = idx / h, e = idx - gi * h;
    float m = -1e30f;
    for (int w = 0; w < kStepWaves; ++w) m = fmaxf(m, sm[(w * G + gi) * rec + h]);
    float l = 0.f, o = 0.f;
    for (int w = 0; w < kStepWaves; ++w) {
      const float* r = sm + (w * G + gi) * rec;
      const float sc = __expf(r[h] - m);
      l += r[h + 1] * sc; o += r[e] * sc;
    }
    const int head = g.hg * G + gi;
    if (single) {
      st_tag(S.o + (long)head * h + e, o / l, wtag);
    } else {
      tagged_t* pr = S.part + ((long)head * kMaxSplits + g.split) * rec;
      st_tag(pr + e, o, wtag);
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
  for (int idx = threadIdx.x; idx < G * h; idx += kStepThreads) {
    const int gi = idx / h, e = idx - gi * h;
    const int head = g.hg * G + gi;
    const tagged_t* pr = S.part + (long)head * kMaxSplits * rec;
    // splits are folded in split order, eight at a time so that their loads are in flight together
    float m = -1e30f, l = 0.f, o = 0.f;
    for (int sp0 = 0; sp0 < S.n_splits; sp0 += 8) {
      tagged_t rm[8], rl[8], ro[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const bool ok = sp0 + k < S.n_splits;
        const tagged_t* r = pr + (sp0 + k) * rec;
        rm[k] = ok ? ld_raw(r + h) : 0ull; rl[k] = ok ? ld_raw(r + h + 1) : 0ull; ro[k] = ok ? ld_raw(r + e) : 0ull;
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (sp0 + k < S.n_splits) {
          const tagged_t* r = pr + (sp0 + k) * rec;
          const float mk = settle(r + h, rm[k], wtag, a.spin_limit, a.err);
          const float lk = settle(r + h + 1, rl[k], wtag, a.spin_limit, a.err);
          const float ok_ = settle(r + e, ro[k], wtag, a.spin_limit, a.err);
          const float mn = fmaxf(m, mk);
          const float sa = __expf(m - mn), sb = __expf(mk - mn);
          l = l * sa + lk * sb;
          o = o * sa + ok_ * sb;
          m = mn;
        }
      }
    }
    st_tag(S.o + (long)head * h + e, o / l, wtag);
  }
  if (threadIdx.x == 0) __hip_atomic_store(S.tickets + g.hg, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------------------

// Geometry of the four GEMV phases lives in LDS as plain integers (it depends on the workgroup
// only); a phase reloads what it needs, so only two geometries are ever live in registers.
constexpr int kGeoInts = 10;
__device__ __forceinline__ int* lds_geo() { extern __shared__ float smem[]; return (int*)(smem + 16) + 4; }   // 32 ints after the flags

template <typename WT>
__device__ __forceinline__ void store_geo(int j, int N, int Kd, int rope_h, int wg, int nwg) {
  const Geo g = make_geo<WT>(nullptr, N, Kd, rope_h, wg, nwg, 0);
  int* o = lds_geo() + j * kGeoInts;
  o[0] = g.N; o[1] = g.units; o[2] = g.cpp; o[3] = g.rope_h; o[4] = g.p_lo; o[5] = g.n_pl; o[6] = g.dq; o[7] = g.dr; o[8] = g.bshift; o[9] = g.nwg;
}
__device__ __forceinline__ Geo load_geo(int j, const void* W, int wave) {
  const int* o = lds_geo() + j * kGeoInts;
  Geo g;
  g.W = W;
  g.N = __builtin_amdgcn_readfirstlane(o[0]); g.units = __builtin_amdgcn_readfirstlane(o[1]);
  g.cpp = __builtin_amdgcn_readfirstlane(o[2]); g.rope_h = __builtin_amdgcn_readfirstlane(o[3]);
  g.p_lo = __builtin_amdgcn_readfirstlane(o[4]); g.n_pl = __builtin_amdgcn_readfirstlane(o[5]);
  g.dq = __builtin_amdgcn_readfirstlane(o[6]); g.dr = __builtin_amdgcn_readfirstlane(o[7]);
  g.bshift = __builtin_amdgcn_readfirstlane(o[8]); g.nwg = __builtin_amdgcn_readfirstlane(o[9]);
  const int flat = g.n_pl * g.cpp;
  g.n_k = flat > wave ? (flat - wave + kStepWaves - 1) / kStepWaves : 0;
  geo_rows(g);
  return g;
}
// GEMV phases in order: 0 = QKV, 1 = output projection, 2 = MLP up, 3 = MLP down
__device__ __forceinline__ int gemv_index(int ph) { return ph == PH_QKV ? 0 : ph - 1; }
// Every layer occupies an identically laid out block of the arena, so layer i's pointers are
// the first layer's advanced by i strides: no pointer has to be fetched from memory.
template <typename T> __device__ __forceinline__ T* advance(T* p, long bytes) { return p ? (T*)((char*)p + bytes) : p; }
__device__ __forceinline__ const void* advance(const void* p, long bytes) { return p ? (const void*)((const char*)p + bytes) : p; }
template <typename AR>
__device__ __forceinline__ StepLayer layer_at(const AR& a, int layer) {
  const long w = a.w_stride * layer, kv = a.kv_stride * layer;
  StepLayer L;
  L.wqkv = advance(a.l0.wqkv, w); L.wo = advance(a.l0.wo, w); L.wup = advance(a.l0.wup, w); L.wdown = advance(a.l0.wdown, w);
  L.bqkv = advance(a.l0.bqkv, w); L.bo = advance(a.l0.bo, w); L.bup = advance(a.l0.bup, w); L.bdown = advance(a.l0.bdown, w);
  L.ln1_g = advance(a.l0.ln1_g, w); L.ln1_b = advance(a.l0.ln1_b, w); L.ln2_g = advance(a.l0.ln2_g, w); L.ln2_b = advance(a.l0.ln2_b, w);
  L.kv = advance(a.l0.kv, kv);
  return L;
}
__device__ __forceinline__ const void* layer_matrix(const StepLayer& L, int j) {
  return j == 0 ? L.wqkv : j == 1 ? L.wo : j == 2 ? L.wup : L.wdown;
}

template <typename WT, int G>
__global__ __launch_bounds__(kStepThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_step(StepArgs a) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // a set of nwg workgroups takes its messages in turn inside every phase; two sets share the compute units
  const int nwg = a.nwg, wg = blockIdx.x % nwg;
  const int set = (int)blockIdx.x / nwg;
  const int slot_lo = a.set_lo[set], slot_hi = a.set_lo[set + 1];
  // the other set's first message: how far its workgroup of the same index has come is what this one paces itself by
  const StepSlot& O = a.s[a.set_lo[a.n_sets == 2 ? (set ^ 1) : 0]];
  float* part = lds_part();
  float* xs = lds_vec(a.part_floats);
  float* red = lds_red();
  int* s_flag = lds_flag();

  if (threadIdx.x == 0) {
    store_geo<WT>(0, (a.H + 2 * a.K) * a.h, a.d, a.h, wg, nwg);       // pairs (i, i + h/2): the RoPE partners
    store_geo<WT>(1, a.d, a.H * a.h, 0, wg, nwg);
    store_geo<WT>(2, a.mlp_kind == MDI_MLP_SWIGLU ? 2 * a.F : a.F, a.d, 0, wg, nwg);
    store_geo<WT>(3, a.d, a.F, 0, wg, nwg);
    if (wg == 0)
      for (int m = 0; m < a.n_slots; ++m)
        if (a.s[m].table_entry) *a.s[m].table_entry = a.s[m].new_page;
  }
  __syncthreads();

  float acc0 = 0.f, acc1 = 0.f;
  AttnState<WT, G> st;
  AttnGeo ga{};
  Tile A, B;
  Cursor ci, cc;                             // the GEMV phases' issue and multiply cursors
  int pgA[kTile], pgB[kTile];               // page numbers of the attention tiles that go into A and B next
  // requested while finishing the previous (message, phase): the next one's flags and the head of its input vector
  bool early_flags = false, early_vec = false;
  unsigned efl[4] = {0u, 0u, 0u, 0u};
  tagged_t eraw[8] = {0ull, 0ull, 0ull, 0ull, 0ull, 0ull, 0ull, 0ull};
  float egain[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};

#pragma nounroll
  for (int layer = 0; layer < a.n_layer; ++layer) {
    const StepLayer Lv = layer_at(a, layer);
    const StepLayer* L = &Lv;
#pragma nounroll
    for (int ph = 0; ph < 5; ++ph) {
#pragma nounroll
      for (int slot = slot_lo; slot < slot_hi; ++slot) {
        // Messages alternate inside a phase: while this message's flags and input vector make their round trips,
        // the memory system is still busy with the other message's stream, and by the time a message reaches its
        // next phase every workgroup has long finished its previous one.
        const StepSlot& S = a.s[slot];
        const unsigned epoch = S.epoch0 + (unsigned)(layer * 5 + ph);
        // ---- this phase's first two tiles: their addresses depend on nothing another workgroup writes,
        //      so they are in flight while the barrier completes and the input vector is staged
        const int j = gemv_index(ph);
        const Geo g = load_geo(j, layer_matrix(Lv, j), wave);
        if (ph == PH_ATTN) {
          ga = make_attn_geo<WT, G>(a, S, wg, wave, lane);
          attn_pages(pgA, ga, a, S, 0, wave); attn_pages(pgB, ga, a, S, 1, wave);
          attn_issue<WT>(A, pgA, ga, a, S, L->kv, 0, wave); attn_issue<WT>(B, pgB, ga, a, S, L->kv, 1, wave);
        } else { ci = cc = cursor_start(g, wave); gemv_issue(A, g, ci, lane); gemv_issue(B, g, ci, lane); }

        auto early_requests = [&]() __attribute__((always_inline)) {
          // ---- requests for the next (message, phase), answered while this phase is being finished: with two
          //      messages alternating, what the next one needs was published a whole phase ago
          early_flags = false; early_vec = false;
          // whatever was requested a phase ago has been used: giving every register a value here, on every path,
          // tells the compiler that none of them is live across the streaming loops above
#pragma unroll
          for (int k = 0; k < 4; ++k) efl[k] = 0u;
#pragma unroll
          for (int jj = 0; jj < 8; ++jj) { eraw[jj] = 0ull; egain[jj] = 1.f; }
          if (slot_hi - slot_lo > 1) {
            int nslot = slot + 1, nph = ph, nlayer = layer;
            if (nslot == slot_hi) { nslot = slot_lo; if (++nph == 5) { nph = 0; ++nlayer; } }
            if (nlayer < a.n_layer) {
              const StepSlot& N = a.s[nslot];
              const unsigned nepoch = N.epoch0 + (unsigned)(nlayer * 5 + nph);
              if (nwg <= 256 && threadIdx.x < 64) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                  const int i = (int)threadIdx.x + 64 * k;
                  efl[k] = i < nwg ? __hip_atomic_load(N.flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : nepoch;
                }
                early_flags = true;
              }
              if (nph != PH_ATTN && !(nph == PH_QKV && nlayer == 0)) {
                const tagged_t* nsrc = nph == PH_OPROJ ? N.o : nph == PH_DOWN ? N.u : N.xres;
                const int nn = nph == PH_OPROJ ? a.H * a.h : nph == PH_DOWN ? a.F : a.d;
                const bool nrms = (nph == PH_QKV || nph == PH_UP) && a.norm_kind == MDI_NORM_RMSNORM;
                const float* ngain = advance(nph == PH_QKV ? a.l0.ln1_g : a.l0.ln2_g, a.w_stride * nlayer);
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                  const int i = (int)threadIdx.x + jj * kStepThreads;
                  eraw[jj] = i < nn ? ld_raw(nsrc + i) : 0ull;
                }
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                  const int i = (int)threadIdx.x + jj * kStepThreads;
                  egain[jj] = (nrms && i < nn) ? ngain[i] : 1.f;
                }
                early_vec = true;
              }
            }
          }
        };

        // Two sets share a compute unit's memory pipeline, and the hardware serves the older wavefronts (the set
        // that was dispatched first) or the higher priority first; left alone, one set finishes a fifth earlier
        // and the other runs the rest of the launch on half the wavefronts.  So the set that is behind takes the
        // higher priority, phase by phase.
        unsigned other_done = 0u;
        const bool pace = a.n_sets == 2 && slot == slot_lo;
        if (pace) other_done = __hip_atomic_load(O.flags + wg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - O.epoch0;

        // ---- wait until every workgroup has finished the previous phase ----------------------------
        stamp(a, S, layer, ph, 0);
        if (threadIdx.x < 64) {
          bool ok = true;
          int it = 0;
          bool seen = early_flags;                   // the flags requested early may already show everyone
#pragma unroll
          for (int k = 0; k < 4; ++k) seen = seen && ((int)(efl[k] - epoch) >= 0);
          while (!__all(seen)) {
            bool all = true;
            for (int i = threadIdx.x; i < nwg; i += 64) {
              const unsigned v = __hip_atomic_load(S.flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
        if (!s_flag[0]) return;
        stamp(a, S, layer, ph, 1);
        if (pace) {
          // work left, in (message, phase) units; the set with more of it goes first
          const int seen = __builtin_amdgcn_readfirstlane((int)other_done), total = a.n_layer * 5;
          const int left = (total - (layer * 5 + ph)) * (slot_hi - slot_lo);
          const int other_left = (total - seen) * (a.set_lo[2 - set] - a.set_lo[1 - set]);
          if (left > other_left || (left == other_left && set == 1)) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
        }

        if (ph == PH_ATTN) {
          // ---- attention over the sample's pages -----------------------------------------------------
          attn_begin<WT, G>(st, ga, a, S, xs, epoch);
          stamp(a, S, layer, ph, 2);
          const int nte = ((ga.n_k + kTile - 1) / kTile + 1) & ~1;
          attn_stream<WT, G>(st, A, B, pgA, pgB, ga, a, S, L->kv, nte, wave, xs);
          stamp(a, S, layer, ph, 3);
          early_requests();
          attn_to_lds<WT, G>(st, ga, a.h, xs, wave);
          attn_finish<G>(ga, a, S, xs, s_flag, epoch);
        } else {
          // ---- a GEMV phase ----------------------------------------------------------------------------
          for (int i = threadIdx.x; i < g.n_pl * 2 * kStepWaves; i += kStepThreads) part[i] = 0.f;
          const bool normed = ph == PH_QKV || ph == PH_UP;
          const bool fused_rms = normed && a.norm_kind == MDI_NORM_RMSNORM;
          const float* gain = ph == PH_QKV ? L->ln1_g : L->ln2_g;
          float row_scale = 1.f;                       // 1/rms when the norm is folded into the epilogue
          if (ph == PH_QKV && layer == 0) {
            stage_input<WT>(a, S, xs, load_geo(1, nullptr, wave), epoch);
            if (fused_rms) {
              // same arithmetic, element order and thread mapping as stage_coherent, so that a layer gives the same
              // bits whether it is the first of its partition or not (where the model is cut changes nothing)
              __syncthreads();                          // stage_input has read its rows of xs
              float ss = 0.f;
              for (int i0 = threadIdx.x; i0 < a.d; i0 += 8 * kStepThreads) {
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                  const int i = i0 + jj * kStepThreads;
                  if (i < a.d) { const float x = xs[i]; ss += x * x; xs[i] = x * gain[i]; }
                }
              }
              row_scale = 1.f / sqrtf(block_sum(ss, red) / (float)a.d + a.eps);
            }
          } else {
            const tagged_t* src = ph == PH_OPROJ ? S.o : ph == PH_DOWN ? S.u : S.xres;
            const float ss = stage_coherent(src, g.units * Storage<WT>::kVec, xs, fused_rms ? gain : nullptr, epoch, a.spin_limit, a.err,
                                            early_vec, eraw, egain);
            if (fused_rms) row_scale = 1.f / sqrtf(block_sum(ss, red) / (float)a.d + a.eps);
          }
          // zeros behind the vector up to a whole 64-lane chunk (the host sizes the LDS for it): see gemv_compute
          for (int i = g.units * Storage<WT>::kVec + (int)threadIdx.x; i < g.cpp * 64 * Storage<WT>::kVec; i += kStepThreads) xs[i] = 0.f;
          __syncthreads();
          if (normed && !fused_rms) {
            normalise(xs, a.d, a.norm_kind, a.eps, gain, ph == PH_QKV ? L->ln1_b : L->ln2_b, red);
            __syncthreads();
          }
          // residual phases: fetch this thread's rows of x now, the stream below hides the latency
          tagged_t x0 = 0ull, x1 = 0ull;
          if ((ph == PH_OPROJ || ph == PH_DOWN) && (int)threadIdx.x < g.n_pl) {
            const int r0 = 2 * geo_pair(g, (int)threadIdx.x);
            x0 = ld_raw(S.xres + r0);
            if (r0 + 1 < g.N) x1 = ld_raw(S.xres + r0 + 1);
          }
          stamp(a, S, layer, ph, 2);

          const int nte = ((g.n_k + kTile - 1) / kTile + 1) & ~1;
#pragma nounroll
          for (int t = 0; t < nte; t += 2) {
            gemv_compute<WT, true>(A, g, t, cc, wave, lane, xs, part, acc0, acc1);
            gemv_issue(A, g, ci, lane);
            gemv_compute<WT, true>(B, g, t + 1, cc, wave, lane, xs, part, acc0, acc1);
            gemv_issue(B, g, ci, lane);
          }
          stamp(a, S, layer, ph, 3);
          early_requests();
          gemv_finish<WT>(ph, g, L, layer, a, S, part, row_scale, x0, x1, epoch);
        }

        // ---- publish: this workgroup is done with the phase ---------------------------------------------
        stamp(a, S, layer, ph, 5);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // this thread's stores have completed
        __syncthreads();
        stamp(a, S, layer, ph, 6);
        if (threadIdx.x == 0) __hip_atomic_store(S.flags + wg, epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

template <typename WT>
static void launch_step_t(hipStream_t s, int G, int nwg, size_t lds, const StepArgs& a) {
  const dim3 grid(nwg * a.n_sets), block(kStepThreads);
  // G = query heads per attention work item: the host asks for 1 or 2 (larger groups were measured slower)
  if (G == 2) hipLaunchKernelGGL((k_step<WT, 2>), grid, block, lds, s, a);
  else hipLaunchKernelGGL((k_step<WT, 1>), grid, block, lds, s, a);
}

#if MDI_STEP_WAVES == 8
// ---------------------------------------------------------------------------
// Output layers (Alg. 1: "process output layers ... get token"): final norm, vocabulary projection and greedy
// argmax as one launch that streams the vocabulary matrix the way a GEMV phase of k_step does (same work split,
// same two register tiles in flight per wavefront across row boundaries), without any exchange: every workgroup
// normalises the activation itself.  Logits are optional; the argmax (lowest index on exact ties) is folded per
// workgroup and then by the last workgroup to arrive, in index order.
__device__ __forceinline__ bool better_logit(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

template <typename WT>
__global__ __launch_bounds__(kStepThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_logits(LogitsArgs a) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wg = blockIdx.x, nwg = gridDim.x;
  float* part = lds_part();
  float* xs = lds_vec(a.part_floats);
  float* red = lds_red();
  const Geo g = make_geo<WT>(a.W, a.N, a.Kd, 0, wg, nwg, wave);
  Tile A, B;
  Cursor ci = cursor_start(g, wave), cc = ci;
  gemv_issue(A, g, ci, lane);
  gemv_issue(B, g, ci, lane);
  for (int i = threadIdx.x; i < a.Kd; i += kStepThreads) xs[i] = load_kind(a.x, a.x_kind, i);
  for (int i = threadIdx.x; i < g.n_pl * 2 * kStepWaves; i += kStepThreads) part[i] = 0.f;
  __syncthreads();
  normalise(xs, a.Kd, a.norm_kind, a.eps, a.g, a.b, red);
  __syncthreads();
  float acc0 = 0.f, acc1 = 0.f;
  const int nte = ((g.n_k + kTile - 1) / kTile + 1) & ~1;
#pragma nounroll
  for (int t = 0; t < nte; t += 2) {
    gemv_compute<WT, false>(A, g, t, cc, wave, lane, xs, part, acc0, acc1);
    gemv_issue(A, g, ci, lane);
    gemv_compute<WT, false>(B, g, t + 1, cc, wave, lane, xs, part, acc0, acc1);
    gemv_issue(B, g, ci, lane);
  }
  __syncthreads();                                           // all wavefronts' partials are in LDS
  float bv = -INFINITY; int bi = 0x7FFFFFFF;
  for (int pl = threadIdx.x; pl < g.n_pl; pl += kStepThreads) {
    float v0 = 0.f, v1 = 0.f;
#pragma unroll
    for (int w = 0; w < kStepWaves; ++w) { v0 += part[(pl * 2) * kStepWaves + w]; v1 += part[(pl * 2 + 1) * kStepWaves + w]; }
    const int r0 = 2 * geo_pair(g, pl), r1 = r0 + 1;
    if (a.out) a.out[r0] = v0;
    if (better_logit(v0, r0, bv, bi)) { bv = v0; bi = r0; }
    if (r1 < a.N) {
      if (a.out) a.out[r1] = v1;
      if (better_logit(v1, r1, bv, bi)) { bv = v1; bi = r1; }
    }
  }
  // workgroup best, then the last workgroup to arrive folds the per-workgroup candidates
  __shared__ float sv[kStepWaves];
  __shared__ int si[kStepWaves];
  __shared__ int s_last;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64); const int oi = __shfl_xor(bi, off, 64);
    if (better_logit(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
  __syncthreads();
  // The candidate crosses workgroups as two 8-byte words that carry the call's counter (value | tag, index | tag),
  // stored and loaded at agent scope; the last workgroup to arrive reloads a word until its tag is this call's.  No
  // fence: on this chip an agent-scope fence writes back a die's L2 (measured: about 5 us per wavefront that runs one).
  if (threadIdx.x == 0) {
    for (int k = 1; k < kStepWaves; ++k) if (better_logit(sv[k], si[k], bv, bi)) { bv = sv[k]; bi = si[k]; }
    __hip_atomic_store(a.cand + 2 * wg, ((tagged_t)a.tag << 32) | __float_as_uint(bv), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(a.cand + 2 * wg + 1, ((tagged_t)a.tag << 32) | (uint32_t)bi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned ticket = __hip_atomic_fetch_add(a.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = ticket == (unsigned)nwg - 1;
  }
  __syncthreads();
  if (s_last) {
    bv = -INFINITY; bi = 0x7FFFFFFF;
    for (int k = threadIdx.x; k < nwg; k += kStepThreads) {
      tagged_t uv = ld_raw(a.cand + 2 * k), ui = ld_raw(a.cand + 2 * k + 1);
      int it = 0;
      while ((uint32_t)(uv >> 32) != a.tag || (uint32_t)(ui >> 32) != a.tag) {
        if (++it > a.spin_limit) { __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
        __builtin_amdgcn_s_sleep(1);
        uv = ld_raw(a.cand + 2 * k); ui = ld_raw(a.cand + 2 * k + 1);
      }
      const float v = __uint_as_float((uint32_t)uv);
      const int i = (int)(uint32_t)ui;
      if (better_logit(v, i, bv, bi)) { bv = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(bv, off, 64); const int oi = __shfl_xor(bi, off, 64);
      if (better_logit(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    __syncthreads();
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int k = 1; k < kStepWaves; ++k) if (better_logit(sv[k], si[k], bv, bi)) { bv = sv[k]; bi = si[k]; }
      *a.token_out = bi;
      __hip_atomic_store(a.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}
#endif

}  // namespace step_w<waves>

#if MDI_STEP_WAVES == 8
void launch_logits(hipStream_t s, int dtype, int nwg, size_t lds, const LogitsArgs& a) {
  using namespace step_w8;
  const dim3 grid(nwg), block(kStepThreads);
  if (dtype == MDI_BF16) hipLaunchKernelGGL(k_logits<bf16_t>, grid, block, lds, s, a);
  else hipLaunchKernelGGL(k_logits<float>, grid, block, lds, s, a);
}
#endif

void MDI_STEP_CAT(launch_step_w, MDI_STEP_WAVES)(hipStream_t s, int dtype, int G, int nwg, size_t lds, const StepArgs& a) {
  using namespace MDI_STEP_CAT(step_w, MDI_STEP_WAVES);
  if (dtype == MDI_BF16) launch_step_t<bf16_t>(s, G, nwg, lds, a); else launch_step_t<float>(s, G, nwg, lds, a);
}

}  // namespace mdi
