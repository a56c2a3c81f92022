// One decode step of a whole partition as ONE persistent kernel launch.
//
// A later visit of a sample (Sec. III-D) pushes a single position through every
// local layer; each layer is five dependent matrix-vector / attention phases whose
// inputs are full vectors produced by the previous phase.  Launching them as
// separate kernels leaves the memory system idle at every boundary (drain, launch,
// ramp-up), which at M = 1 costs more than the work itself on small layers and a
// third of the time on 7B-sized ones.  Here one workgroup per compute unit stays
// resident for the whole step:
//
//   * phases are separated by a grid-wide barrier built from per-workgroup epoch
//     flags.  Everything that crosses workgroups (x, q, o, u, attention partials,
//     the newest K/V row, the flags) is written and read with agent-scope relaxed
//     atomics, i.e. cache-coherent (sc1) loads/stores, so the barrier needs no L2
//     write-back/invalidate; ordering inside a workgroup comes from
//     workgroup-scope fences (plain waits on outstanding memory operations).
//   * weight and KV-cache addresses do not depend on activations, so every
//     wavefront keeps two register tiles (16 x 16-byte loads per lane each) in
//     flight and, while it finishes a phase, already issues the first two tiles of
//     the NEXT phase.  The barrier latency and the vector staging after it are
//     covered by those loads.
//   * inside a workgroup the rows of a phase are laid out as one flat sequence of
//     (row pair, 1-KiB chunk) items that is cut into eight equal contiguous ranges,
//     one per wavefront, so wavefronts stay balanced whatever the shape; a pair
//     that straddles two ranges is completed through an LDS slot per wavefront and
//     summed in wavefront order (deterministic, no float atomics).
//
// Every spin is bounded: a workgroup that waits longer than `spin_limit` polls
// raises the partition's error flag and leaves, and so does every other one.
#include "device_utils.h"

namespace mdi {

constexpr int kTile = 4;                 // items per register tile (two 16-byte loads each)

struct Tile { uint4 r[2 * kTile]; };

__device__ __forceinline__ float ld_sc(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t ld_sc(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_sc(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_sc(bf16_t* p, float v) { __hip_atomic_store(p, f32_to_bf16(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

template <typename T> struct Unpack;
template <> struct Unpack<float> {
  __device__ __forceinline__ static __forceinline__ void go(const uint4& t, float (&v)[4]) {
    v[0] = __uint_as_float(t.x); v[1] = __uint_as_float(t.y); v[2] = __uint_as_float(t.z); v[3] = __uint_as_float(t.w);
  }
};
template <> struct Unpack<bf16_t> {
  __device__ __forceinline__ static __forceinline__ void go(const uint4& t, float (&v)[8]) {
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
    v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xFFFF0000u);
    v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xFFFF0000u);
  }
};

enum StepPhase { PH_QKV = 0, PH_ATTN = 1, PH_OPROJ = 2, PH_UP = 3, PH_DOWN = 4 };

// ---------------------------------------------------------------------------
// GEMV phase geometry for one wavefront.
template <typename WT>
struct GemvPh {
  static constexpr int V = Storage<WT>::kVec;
  const WT* W;
  int N, Kd, cpp;        // rows, columns, 64-lane chunks per row
  int rope_h;            // > 0: pair (i, i + h/2) inside heads of size h; 0: rows (2p, 2p + 1)
  int p_lo, n_pl;        // this workgroup's pairs
  int f_lo, f_hi;        // this wavefront's range in the flat (pair, chunk) space

  __device__ __noinline__ void setup(int N_, int Kd_, int rope_h_, int wg, int nwg, int wave) {
    N = N_; Kd = Kd_; rope_h = rope_h_; W = nullptr;
    cpp = (Kd + 64 * V - 1) / (64 * V);
    const int pairs = (N + 1) >> 1;
    p_lo = (int)((long)pairs * wg / nwg);
    n_pl = (int)((long)pairs * (wg + 1) / nwg) - p_lo;
    const int flat = n_pl * cpp;
    f_lo = flat * wave / kStepWaves;
    f_hi = flat * (wave + 1) / kStepWaves;
  }
  __device__ __forceinline__ int n_tiles() const { return (f_hi - f_lo + kTile - 1) / kTile; }
  __device__ __forceinline__ int row(int p, int j) const {
    if (rope_h) {
      const int half = rope_h >> 1, head = p / half, i = p - head * half;
      return head * rope_h + i + j * half;
    }
    return 2 * p + j;
  }
  __device__ __forceinline__ void issue(Tile& t, int ti, int lane) const {
    int f = f_lo + ti * kTile;
    int pl = f / cpp, c = f - pl * cpp;
#pragma unroll
    for (int s = 0; s < kTile; ++s) {
      const int piece = c * 64 + lane;
      const bool ok = (f + s < f_hi) && (piece * V < Kd);
      const int r0 = min(row(p_lo + pl, 0), N - 1), r1 = min(row(p_lo + pl, 1), N - 1);
      const uint4 z = {0u, 0u, 0u, 0u};
      t.r[2 * s] = ok ? *reinterpret_cast<const uint4*>(W + (long)r0 * Kd + piece * V) : z;
      t.r[2 * s + 1] = ok ? *reinterpret_cast<const uint4*>(W + (long)r1 * Kd + piece * V) : z;
      if (++c == cpp) { c = 0; ++pl; }
    }
  }
  // part: LDS [n_pl][2][8 wavefronts]
  __device__ __forceinline__ void compute(const Tile& t, int ti, int lane, int wave, const float* xs, float* part,
                                          float& acc0, float& acc1) const {
    int f = f_lo + ti * kTile;
    int pl = f / cpp, c = f - pl * cpp;
#pragma unroll
    for (int s = 0; s < kTile; ++s) {
      if (f + s < f_hi) {                          // uniform across the wavefront
        const int piece = c * 64 + lane;
        if (piece * V < Kd) {
          float w0[V], w1[V], xv[V];
          Unpack<WT>::go(t.r[2 * s], w0);
          Unpack<WT>::go(t.r[2 * s + 1], w1);
#pragma unroll
          for (int e = 0; e < V; e += 4) {
            const float4 q4 = *reinterpret_cast<const float4*>(xs + piece * V + e);
            xv[e] = q4.x; xv[e + 1] = q4.y; xv[e + 2] = q4.z; xv[e + 3] = q4.w;
          }
#pragma unroll
          for (int e = 0; e < V; ++e) { acc0 = fmaf(w0[e], xv[e], acc0); acc1 = fmaf(w1[e], xv[e], acc1); }
        }
        if (c == cpp - 1 || f + s == f_hi - 1) {   // the pair, or this wavefront's share of it, is complete
          const float r0 = wave_sum(acc0), r1 = wave_sum(acc1);
          if (lane == 0) { part[(pl * 2) * kStepWaves + wave] = r0; part[(pl * 2 + 1) * kStepWaves + wave] = r1; }
          acc0 = 0.f; acc1 = 0.f;
        }
      }
      if (++c == cpp) { c = 0; ++pl; }
    }
  }
};

// ---------------------------------------------------------------------------
template <typename WT, int G>
struct Step {
  static constexpr int V = Storage<WT>::kVec;
  const StepArgs& a;
  const int lane, wave, wg, nwg;
  // LDS
  float* red;      // 16 floats
  int* s_flag;     // 2 ints
  float* part;     // GEMV pair partials [pairs][2][8]
  float* xs;       // staged vector / attention scratch
  unsigned epoch;
  GemvPh<WT> qkv, op, up, dn;
  const StepLayer* L;      // current layer
  int layer;
  float acc0, acc1;
  // attention geometry
  int at_hg, at_split, at_s0, at_s1, at_s1p, at_kvh, at_L, at_tpw, at_sub, at_hoff;
  bool at_active;
  float at_m[G], at_l[G], at_o[G][V];

  __device__ __forceinline__ Step(const StepArgs& a_, float* smem)
      : a(a_), lane(threadIdx.x & 63), wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)), wg(blockIdx.x), nwg(gridDim.x) {
    red = smem; s_flag = (int*)(smem + 16); part = smem + 32; xs = part + a.part_floats;
    epoch = a.epoch0;
    acc0 = acc1 = 0.f;
  }

  // ---- grid barrier -------------------------------------------------------
  __device__ __noinline__ void arrive() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // this thread's stores have completed
    __syncthreads();
    ++epoch;
    if (threadIdx.x == 0) __hip_atomic_store(a.flags + wg, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __device__ __noinline__ bool wait() {
    if (wave == 0) {
      bool ok = true;
      int it = 0;
      for (;;) {
        bool all = true;
        for (int i = lane; i < nwg; i += 64) {
          const unsigned v = __hip_atomic_load(a.flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          all = all && ((int)(v - epoch) >= 0);
        }
        if (__all(all)) break;
        if (++it > a.spin_limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      if (lane == 0) {
        s_flag[0] = ok;
        if (!ok) __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return s_flag[0] != 0;
  }

  // ---- vector staging -------------------------------------------------------
  // raw vector -> xs; optionally normalise in place.  src_kind: 0 = fp32 buffer written in this launch
  // (coherent loads), 1 = the step's input (token embedding or previous stage's activation).
  __device__ __noinline__ void stage(const float* src, int n, bool from_input, bool norm, const float* g, const float* b) {
    if (from_input) {
      if (a.in_kind == IN_TOKEN) {
        const long tok = *(const int32_t*)a.in;
        for (int i = threadIdx.x; i < n; i += kStepThreads) {
          float v = Storage<WT>::get((const WT*)a.wte + tok * n + i);
          if (a.wpe) v += Storage<WT>::get((const WT*)a.wpe + (long)a.pos * n + i);
          xs[i] = v;
        }
      } else {
        for (int i = threadIdx.x; i < n; i += kStepThreads) xs[i] = load_kind(a.in, a.in_kind, i);
      }
      // the rows this workgroup owns in the residual phases get their starting value
      __syncthreads();
      const int r_lo = 2 * op.p_lo, r_hi = min(op.N, 2 * (op.p_lo + op.n_pl));
      for (int r = r_lo + threadIdx.x; r < r_hi; r += kStepThreads) st_sc(a.xres + r, xs[r]);
    } else {
      for (int i = threadIdx.x; i < n; i += kStepThreads) xs[i] = ld_sc(src + i);
    }
    if (norm) {
      if (a.norm_kind == MDI_NORM_LAYERNORM) {
        float s = 0.f;
        for (int i = threadIdx.x; i < n; i += kStepThreads) s += xs[i];
        const float mean = block_sum(s, red) / (float)n;
        float s2 = 0.f;
        for (int i = threadIdx.x; i < n; i += kStepThreads) { const float c = xs[i] - mean; s2 += c * c; }
        const float rstd = 1.f / sqrtf(block_sum(s2, red) / (float)n + a.eps);
        for (int i = threadIdx.x; i < n; i += kStepThreads) xs[i] = (xs[i] - mean) * rstd * g[i] + (b ? b[i] : 0.f);
      } else {
        float s2 = 0.f;
        for (int i = threadIdx.x; i < n; i += kStepThreads) s2 += xs[i] * xs[i];
        const float rstd = 1.f / sqrtf(block_sum(s2, red) / (float)n + a.eps);
        for (int i = threadIdx.x; i < n; i += kStepThreads) xs[i] = xs[i] * rstd * g[i];
      }
    }
    __syncthreads();
  }

  // ---- GEMV phases ----------------------------------------------------------
  template <int PH> __device__ __forceinline__ GemvPh<WT>& gph() {
    if (PH == PH_QKV) return qkv;
    if (PH == PH_OPROJ) return op;
    if (PH == PH_UP) return up;
    return dn;
  }

  template <int PH> __device__ __noinline__ bool pre_gemv() {
    if (!wait()) return false;
    zero_part(gph<PH>().n_pl);                       // ordered before use by the barrier that ends stage()
    if (PH == PH_QKV) stage(a.xres, a.d, layer == 0, true, L->ln1_g, L->ln1_b);
    else if (PH == PH_OPROJ) stage(a.o, a.H * a.h, false, false, nullptr, nullptr);
    else if (PH == PH_UP) stage(a.xres, a.d, false, true, L->ln2_g, L->ln2_b);
    else stage(a.u, a.F, false, false, nullptr, nullptr);
    return true;
  }

  template <int PH> __device__ __noinline__ void post_gemv() {
    GemvPh<WT>& g = gph<PH>();
    __syncthreads();                                   // all wavefronts' partials are in LDS
    for (int pl = threadIdx.x; pl < g.n_pl; pl += kStepThreads) {
      float v0 = 0.f, v1 = 0.f;
#pragma unroll
      for (int w = 0; w < kStepWaves; ++w) { v0 += part[(pl * 2) * kStepWaves + w]; v1 += part[(pl * 2 + 1) * kStepWaves + w]; }
      const int p = g.p_lo + pl;
      const int r0 = g.row(p, 0), r1 = g.row(p, 1);
      if (PH == PH_QKV) {
        if (L->bqkv) { v0 += L->bqkv[r0]; v1 += L->bqkv[r1]; }
        const int head = r0 / a.h, i = r0 - head * a.h;
        if (a.rope && head < a.H + a.K) {
          const float2 cs = a.rope[i];
          const float t0 = v0 * cs.x - v1 * cs.y, t1 = v0 * cs.y + v1 * cs.x;
          v0 = t0; v1 = t1;
        }
        if (head < a.H) {
          st_sc(a.q + r0, v0); st_sc(a.q + r1, v1);
        } else {
          const bool is_v = head >= a.H + a.K;
          const int kvh = head - a.H - (is_v ? a.K : 0);
          WT* dst = (WT*)L->kv + a.kv_tok_off + (long)(kvh * 2 + (is_v ? 1 : 0)) * a.pt_h + i;
          st_sc(dst, v0); st_sc(dst + (a.h >> 1), v1);
        }
      } else if (PH == PH_UP) {
        if (a.mlp_kind == MDI_MLP_SWIGLU) {
          st_sc(a.u + p, silu_f(v0) * v1);               // rows (2f, 2f+1) = (gate_f, up_f)
        } else {
          if (L->bup) { v0 += L->bup[r0]; if (r1 < g.N) v1 += L->bup[r1]; }
          const bool tanh_form = a.mlp_kind == MDI_MLP_GELU_TANH;
          st_sc(a.u + r0, tanh_form ? gelu_tanh_f(v0) : gelu_erf_f(v0));
          if (r1 < g.N) st_sc(a.u + r1, tanh_form ? gelu_tanh_f(v1) : gelu_erf_f(v1));
        }
      } else {                                            // residual phases
        const float* bias = PH == PH_OPROJ ? L->bo : L->bdown;
        const bool last = PH == PH_DOWN && layer == a.n_layer - 1;
        {
          float v = v0 + ld_sc(a.xres + r0) + (bias ? bias[r0] : 0.f);
          st_sc(a.xres + r0, v);
          if (last) store_kind(a.act_out, a.act_kind, r0, v);
        }
        if (r1 < g.N) {
          float v = v1 + ld_sc(a.xres + r1) + (bias ? bias[r1] : 0.f);
          st_sc(a.xres + r1, v);
          if (last) store_kind(a.act_out, a.act_kind, r1, v);
        }
      }
    }
    arrive();
  }

  // ---- attention phase --------------------------------------------------------
  __device__ __noinline__ void attn_setup() {
    at_L = a.h / V; at_tpw = 64 / at_L; at_sub = lane / at_L; at_hoff = (lane % at_L) * V;
    const int n_units = a.n_hg * a.n_splits;
    at_active = wg < n_units;
    at_hg = at_active ? wg % a.n_hg : 0;
    at_split = at_active ? wg / a.n_hg : 0;
    at_kvh = (at_hg * G) / (a.H / a.K);
    at_s0 = at_split * a.chunk;
    at_s1 = min(a.ctx, at_s0 + a.chunk);
    at_s1p = min(at_s1, a.ctx - 1);                     // the newest row is written in this launch
  }
  __device__ __forceinline__ int attn_tiles() const {
    if (!at_active) return 0;
    const int steps = (at_s1p - at_s0 + at_tpw - 1) / at_tpw;           // wavefront steps in the slice
    const int mine = (steps - wave + kStepWaves - 1) / kStepWaves;      // steps st with st % 8 == wave
    return mine > 0 ? (mine + kTile - 1) / kTile : 0;
  }
  __device__ __forceinline__ void attn_issue(Tile& t, int ti) const {
    const WT* pool = (const WT*)L->kv;
#pragma unroll
    for (int s = 0; s < kTile; ++s) {
      const int st = (ti * kTile + s) * kStepWaves + wave;
      const int tok = at_s0 + st * at_tpw + at_sub;
      const bool ok = at_active && tok < at_s1p;
      const uint4 z = {0u, 0u, 0u, 0u};
      uint4 kq = z, vq = z;
      if (ok) {
        const int page = a.table[tok / a.pt];
        const WT* kp = pool + ((long)page * a.K + at_kvh) * 2 * a.pt_h + (long)(tok % a.pt) * a.h + at_hoff;
        kq = *reinterpret_cast<const uint4*>(kp);
        vq = *reinterpret_cast<const uint4*>(kp + a.pt_h);
      }
      t.r[2 * s] = kq; t.r[2 * s + 1] = vq;
    }
  }
  __device__ __forceinline__ void attn_update(const uint4& kq, const uint4& vq, bool valid, const float* qs) {
    float kf[V], vf[V];
    Unpack<WT>::go(kq, kf);
    Unpack<WT>::go(vq, vf);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < V; e += 4) {
        const float4 q4 = *reinterpret_cast<const float4*>(qs + g * a.h + at_hoff + e);
        s = fmaf(q4.x, kf[e], s); s = fmaf(q4.y, kf[e + 1], s); s = fmaf(q4.z, kf[e + 2], s); s = fmaf(q4.w, kf[e + 3], s);
      }
      for (int off = 1; off < at_L; off <<= 1) s += __shfl_xor(s, off, 64);
      if (valid) {
        const float mn = fmaxf(at_m[g], s);
        const float alpha = __expf(at_m[g] - mn), p = __expf(s - mn);
        at_m[g] = mn;
        at_l[g] = at_l[g] * alpha + p;
#pragma unroll
        for (int e = 0; e < V; ++e) at_o[g][e] = at_o[g][e] * alpha + p * vf[e];
      }
    }
  }
  __device__ __forceinline__ void attn_compute(const Tile& t, int ti) {
    const float* qs = xs;
#pragma unroll
    for (int s = 0; s < kTile; ++s) {
      const int st = (ti * kTile + s) * kStepWaves + wave;
      if (at_active && at_s0 + st * at_tpw < at_s1p) {    // uniform: some lane of this step has a token
        const int tok = at_s0 + st * at_tpw + at_sub;
        attn_update(t.r[2 * s], t.r[2 * s + 1], tok < at_s1p, qs);
      }
    }
  }
  __device__ __noinline__ bool pre_attn() {
    if (!wait()) return false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      at_m[g] = -1e30f; at_l[g] = 0.f;
#pragma unroll
      for (int e = 0; e < V; ++e) at_o[g][e] = 0.f;
    }
    if (at_active) {
      // the group's query heads, pre-scaled, into LDS
      for (int i = threadIdx.x; i < G * a.h; i += kStepThreads) xs[i] = ld_sc(a.q + (long)at_hg * G * a.h + i) * a.scale;
    }
    __syncthreads();
    // the newest position (written by the QKV phase of this launch): coherent 4-byte loads
    if (at_active && at_s1 == a.ctx && wave == 0) {
      const WT* kp = (const WT*)L->kv + a.kv_tok_off + (long)(at_kvh * 2) * a.pt_h + at_hoff;
      uint4 kq = {0u, 0u, 0u, 0u}, vq = {0u, 0u, 0u, 0u};
      if (at_sub == 0) {
        const uint32_t* k32 = (const uint32_t*)kp;
        const uint32_t* v32 = (const uint32_t*)(kp + a.pt_h);
        kq = make_uint4(ld_sc(k32), ld_sc(k32 + 1), ld_sc(k32 + 2), ld_sc(k32 + 3));
        vq = make_uint4(ld_sc(v32), ld_sc(v32 + 1), ld_sc(v32 + 2), ld_sc(v32 + 3));
      }
      attn_update(kq, vq, at_sub == 0, xs);
    }
    return true;
  }
  __device__ __noinline__ void post_attn() {
    const int h = a.h, rec = h + 2;
    // merge the token sub-groups of the wavefront
    for (int off = at_L; off < 64; off <<= 1) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float mo = __shfl_xor(at_m[g], off, 64), lo = __shfl_xor(at_l[g], off, 64);
        const float mn = fmaxf(at_m[g], mo);
        const float sa = __expf(at_m[g] - mn), sb = __expf(mo - mn);
        at_l[g] = at_l[g] * sa + lo * sb;
#pragma unroll
        for (int e = 0; e < V; ++e) at_o[g][e] = at_o[g][e] * sa + __shfl_xor(at_o[g][e], off, 64) * sb;
        at_m[g] = mn;
      }
    }
    __syncthreads();                                     // queries in xs are no longer needed
    float* sm = xs;                                      // [wave][g][h + 2]
    if (at_sub == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float* r = sm + (wave * G + g) * rec;
#pragma unroll
        for (int e = 0; e < V; ++e) r[at_hoff + e] = at_o[g][e];
        if (at_hoff == 0) { r[h] = at_m[g]; r[h + 1] = at_l[g]; }
      }
    }
    __syncthreads();
    if (at_active) {
      const bool single = a.n_splits == 1;
      for (int idx = threadIdx.x; idx < G * h; idx += kStepThreads) {
        const int g = idx / h, e = idx - g * h;
        float m = -1e30f;
        for (int w = 0; w < kStepWaves; ++w) m = fmaxf(m, sm[(w * G + g) * rec + h]);
        float l = 0.f, o = 0.f;
        for (int w = 0; w < kStepWaves; ++w) {
          const float* r = sm + (w * G + g) * rec;
          const float sc = __expf(r[h] - m);
          l += r[h + 1] * sc; o += r[e] * sc;
        }
        const int head = at_hg * G + g;
        if (single) {
          st_sc(a.o + (long)head * h + e, o / l);
        } else {
          float* pr = a.part + ((long)head * kMaxSplits + at_split) * rec;
          st_sc(pr + e, o);
          if (e == 0) { st_sc(pr + h, m); st_sc(pr + h + 1, l); }
        }
      }
      if (!single) {
        // the last workgroup of the head group to get here folds the splits in split order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (threadIdx.x == 0) {
          const unsigned ticket = __hip_atomic_fetch_add(a.tickets + at_hg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          s_flag[1] = ticket == (unsigned)a.n_splits - 1;
        }
        __syncthreads();
        if (s_flag[1]) {
          for (int idx = threadIdx.x; idx < G * h; idx += kStepThreads) {
            const int g = idx / h, e = idx - g * h;
            const int head = at_hg * G + g;
            const float* pr = a.part + (long)head * kMaxSplits * rec;
            float m = -1e30f;
            for (int sp = 0; sp < a.n_splits; ++sp) m = fmaxf(m, ld_sc(pr + sp * rec + h));
            float l = 0.f, o = 0.f;
            for (int sp = 0; sp < a.n_splits; ++sp) {
              const float* r = pr + sp * rec;
              const float sc = __expf(ld_sc(r + h) - m);
              l += ld_sc(r + h + 1) * sc; o += ld_sc(r + e) * sc;
            }
            st_sc(a.o + (long)head * h + e, o / l);
          }
          if (threadIdx.x == 0) __hip_atomic_store(a.tickets + at_hg, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
    arrive();
  }

  // ---- uniform phase interface ------------------------------------------------
  template <int PH> __device__ __forceinline__ int n_tiles() { return PH == PH_ATTN ? attn_tiles() : gph<PH>().n_tiles(); }
  template <int PH> __device__ __forceinline__ void issue(Tile& t, int ti) {
    if (PH == PH_ATTN) attn_issue(t, ti); else gph<PH>().issue(t, ti, lane);
  }
  template <int PH> __device__ __forceinline__ void compute(const Tile& t, int ti) {
    if (PH == PH_ATTN) attn_compute(t, ti); else gph<PH>().compute(t, ti, lane, wave, xs, part, acc0, acc1);
  }

  // Runs phase PH whose first two tiles are already in A and B, and leaves the
  // first two tiles of phase NX in A and B (unless this is the last phase of the launch).
  template <int PH, int NX> __device__ __forceinline__ bool run(Tile& A, Tile& B, bool has_next) {
    if (PH == PH_ATTN) { if (!pre_attn()) return false; } else { if (!pre_gemv<PH>()) return false; }
    const int nt = n_tiles<PH>();
    const int nte = (nt + 1) & ~1;
    if (nte == 0 && has_next) { issue<NX>(A, 0); issue<NX>(B, 1); }
    for (int t = 0; t < nte; t += 2) {
      compute<PH>(A, t);
      if (t + 2 < nte) issue<PH>(A, t + 2); else if (has_next) issue<NX>(A, 0);
      compute<PH>(B, t + 1);
      if (t + 3 < nte) issue<PH>(B, t + 3); else if (has_next) issue<NX>(B, 1);
    }
    if (PH == PH_ATTN) post_attn(); else post_gemv<PH>();
    return true;
  }

  __device__ __forceinline__ void bind_weights() {
    qkv.W = (const WT*)L->wqkv; op.W = (const WT*)L->wo; up.W = (const WT*)L->wup; dn.W = (const WT*)L->wdown;
  }
  __device__ __forceinline__ void zero_part(int n_pl) {
    for (int i = threadIdx.x; i < n_pl * 2 * kStepWaves; i += kStepThreads) part[i] = 0.f;
  }
};

template <typename WT, int G>
__global__ __launch_bounds__(kStepThreads) void k_step(StepArgs a) {
  extern __shared__ float smem[];
  Step<WT, G> S(a, smem);
  const int nwg = gridDim.x, wg = blockIdx.x;
  S.qkv.setup((a.H + 2 * a.K) * a.h, a.d, a.h, wg, nwg, S.wave);   // pairs (i, i + h/2): the RoPE partners
  S.op.setup(a.d, a.H * a.h, 0, wg, nwg, S.wave);
  S.up.setup(a.mlp_kind == MDI_MLP_SWIGLU ? 2 * a.F : a.F, a.d, 0, wg, nwg, S.wave);
  S.dn.setup(a.d, a.F, 0, wg, nwg, S.wave);
  S.attn_setup();
  if (wg == 0 && threadIdx.x == 0 && a.table_entry) *a.table_entry = a.new_page;

  Tile A, B;
  S.layer = 0;
  S.L = a.layers;
  S.bind_weights();
  S.template issue<PH_QKV>(A, 0);
  S.template issue<PH_QKV>(B, 1);
  // the first wait() of the launch must pass at once: every flag already holds epoch0
  for (int l = 0; l < a.n_layer; ++l) {
    S.layer = l;
    S.L = a.layers + l;
    S.bind_weights();
    const bool more = l + 1 < a.n_layer;
    if (!S.template run<PH_QKV, PH_ATTN>(A, B, true)) return;
    if (!S.template run<PH_ATTN, PH_OPROJ>(A, B, true)) return;
    if (!S.template run<PH_OPROJ, PH_UP>(A, B, true)) return;
    if (!S.template run<PH_UP, PH_DOWN>(A, B, true)) return;
    if (more) S.qkv.W = (const WT*)a.layers[l + 1].wqkv;   // the down phase prefetches the next layer's first tiles
    if (!S.template run<PH_DOWN, PH_QKV>(A, B, more)) return;
  }
}

template <typename WT>
static void launch_step_t(hipStream_t s, int G, int nwg, size_t lds, const StepArgs& a) {
  const dim3 grid(nwg), block(kStepThreads);
  switch (G) {
    case 8: hipLaunchKernelGGL((k_step<WT, 8>), grid, block, lds, s, a); break;
    case 4: hipLaunchKernelGGL((k_step<WT, 4>), grid, block, lds, s, a); break;
    case 2: hipLaunchKernelGGL((k_step<WT, 2>), grid, block, lds, s, a); break;
    default: hipLaunchKernelGGL((k_step<WT, 1>), grid, block, lds, s, a); break;
  }
}

void launch_step(hipStream_t s, int dtype, int G, int nwg, size_t lds, const StepArgs& a) {
  if (dtype == MDI_BF16) launch_step_t<bf16_t>(s, G, nwg, lds, a); else launch_step_t<float>(s, G, nwg, lds, a);
}

}  // namespace mdi
