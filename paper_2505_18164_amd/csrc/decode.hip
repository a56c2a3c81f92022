// Decode-step kernels: one position of one sample through a decoder layer
// (Sec. III-D: after the first visit only the newest token's activation is
// propagated, and the sample's cached keys/values are extended, not rebuilt).
//
// Everything here is bound by HBM bandwidth: each matrix is read exactly once
// per step (M = 1), so the kernels are row-streaming GEMVs with 16-byte
// coalesced loads, the vector operand staged once per workgroup in LDS, and the
// small elementwise work (norm, bias, RoPE, activation, residual) fused into the
// prologue/epilogue so no intermediate makes an extra trip through memory.
#include "device_utils.h"

namespace mdi {

// ---------------------------------------------------------------------------
// step input: token embedding (+ learned position) or the previous stage's
// activation, widened into the fp32 residual stream.
__global__ __launch_bounds__(kBlock) void k_input(InputArgs a) {
  if (threadIdx.x == 0 && blockIdx.x == 0 && a.table_entry) *a.table_entry = a.new_page;
  const int stride = gridDim.x * blockDim.x;
  if (a.in_kind == IN_TOKEN) {
    const long tok = checked_token(a.in, 0, a.vocab, a.err);
    const int wk = a.dtype == MDI_BF16 ? IN_BF16 : IN_F32;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.d; i += stride) {
      float v = load_kind(a.wte, wk, tok * a.d + i);
      if (a.wpe) v += load_kind(a.wpe, wk, (long)a.pos * a.d + i);
      a.xres[i] = v;
    }
  } else {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < a.d; i += stride) a.xres[i] = load_kind(a.in, a.in_kind, i);
  }
}

void launch_input(hipStream_t s, const InputArgs& a) {
  const int blocks = (a.d + kBlock * 4 - 1) / (kBlock * 4);
  hipLaunchKernelGGL(k_input, dim3(blocks), dim3(kBlock), 0, s, a);
}

// ---------------------------------------------------------------------------
// GEMV family.
//
// A wavefront owns four rows at a time; each lane streams 16-byte pieces of
// those rows (lane l takes elements [l*V, l*V+V) of every 64*V-wide column
// window), multiplies with the LDS copy of the vector and the four sums are
// folded across the wavefront with xor-shuffles.  Row groups are dealt to
// wavefronts round-robin so that, at any moment, the grid reads one contiguous
// window of the matrix.
template <int PRO>
__device__ __forceinline__ void stage_vector(const GemvArgs& a, float* xs, float* red) {
  const int Kd = a.Kd;
  for (int i = threadIdx.x; i < Kd; i += kBlock) xs[i] = load_kind(a.x, a.x_kind, i);
  if (PRO == PRO_NORM) {
    // every thread re-reads only the elements it wrote, so no barrier is needed before the sums
    if (a.norm_kind == MDI_NORM_LAYERNORM) {
      float s = 0.f;
      for (int i = threadIdx.x; i < Kd; i += kBlock) s += xs[i];
      const float mean = block_sum(s, red) / (float)Kd;
      float s2 = 0.f;
      for (int i = threadIdx.x; i < Kd; i += kBlock) { const float c = xs[i] - mean; s2 += c * c; }
      const float var = block_sum(s2, red) / (float)Kd;
      const float rstd = 1.f / sqrtf(var + a.eps);
      for (int i = threadIdx.x; i < Kd; i += kBlock) xs[i] = (xs[i] - mean) * rstd * a.g[i] + (a.b ? a.b[i] : 0.f);
    } else {
      float s2 = 0.f;
      for (int i = threadIdx.x; i < Kd; i += kBlock) s2 += xs[i] * xs[i];
      const float ms = block_sum(s2, red) / (float)Kd;
      const float rstd = 1.f / sqrtf(ms + a.eps);
      for (int i = threadIdx.x; i < Kd; i += kBlock) xs[i] = xs[i] * rstd * a.g[i];
    }
  }
  __syncthreads();
}

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

template <typename WT, int PRO, int EPI>
__global__ __launch_bounds__(kBlock) void k_gemv(GemvArgs a) {
  extern __shared__ float smem[];
  float* red = smem;        // 8 floats of reduction scratch
  float* xs = smem + 8;     // Kd floats
  constexpr int V = Storage<WT>::kVec;
  stage_vector<PRO>(a, xs, red);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const WT* W = (const WT*)a.W;
  const int N = a.N, Kd = a.Kd;
  const int n_groups = (N + 3) >> 2;
  const int half = a.h >> 1;
  float best_v = -INFINITY; int best_i = 0x7FFFFFFF;

  for (int grp = blockIdx.x * 4 + wave; grp < n_groups; grp += gridDim.x * 4) {
    int rows[4];
    if (EPI == EPI_QKV) {
      // two RoPE pairs (i, i + h/2) of one head per group
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int p = grp * 2 + j, head = p / half, i = p - head * half;
        rows[2 * j] = head * a.h + i;
        rows[2 * j + 1] = rows[2 * j] + half;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) rows[j] = grp * 4 + j;
    }
    const WT* wp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) wp[j] = W + (long)min(rows[j], N - 1) * Kd;

    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
    for (int c = lane * V; c < Kd; c += 64 * V) {
      float w[4][V];
#pragma unroll
      for (int j = 0; j < 4; ++j) Storage<WT>::load(wp[j] + c, w[j]);
      float xv[V];
#pragma unroll
      for (int e = 0; e < V; e += 4) {
        const float4 t = *reinterpret_cast<const float4*>(xs + c + e);
        xv[e] = t.x; xv[e + 1] = t.y; xv[e + 2] = t.z; xv[e + 3] = t.w;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < V; ++e) acc[j] = fmaf(w[j][e], xv[e], acc[j]);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = wave_sum(acc[j]);

    if (EPI == EPI_QKV) {
      if (lane < 2) {
        const int r0 = lane ? rows[2] : rows[0], r1 = lane ? rows[3] : rows[1];
        float v0 = lane ? acc[2] : acc[0], v1 = lane ? acc[3] : acc[1];
        if (a.bias) { v0 += a.bias[r0]; v1 += a.bias[r1]; }
        const int head = r0 / a.h, i = r0 - head * a.h;
        if (a.rope && head < a.H + a.K) {
          const float2 cs = a.rope[i];
          const float t0 = v0 * cs.x - v1 * cs.y, t1 = v0 * cs.y + v1 * cs.x;
          v0 = t0; v1 = t1;
        }
        if (head < a.H) {
          a.out[r0] = v0; a.out[r1] = v1;
        } else {
          const bool is_v = head >= a.H + a.K;
          const int kvh = head - a.H - (is_v ? a.K : 0);
          WT* dst = (WT*)a.kv_tok + (long)(kvh * 2 + (is_v ? 1 : 0)) * a.pt_h + i;
          Storage<WT>::put(dst, v0);
          Storage<WT>::put(dst + half, v1);
        }
      }
    } else if (EPI == EPI_SWIGLU) {
      // rows (2f, 2f+1) hold gate_f and up_f
      if (lane < 2) {
        const int f = grp * 2 + lane;
        const float gate = lane ? acc[2] : acc[0], up = lane ? acc[3] : acc[1];
        if (2 * f + 1 < N) a.out[f] = silu_f(gate) * up;
      }
    } else {
      if (lane < 4) {
        const int r = grp * 4 + lane;
        float v = lane == 0 ? acc[0] : lane == 1 ? acc[1] : lane == 2 ? acc[2] : acc[3];
        if (r < N) {
          if (a.bias) v += a.bias[r];
          if (EPI == EPI_RESID) {
            v += a.resid[r];
            a.out[r] = v;
            if (a.act_out) store_kind(a.act_out, a.act_kind, r, v);
          } else if (EPI == EPI_GELU_TANH) {
            a.out[r] = gelu_tanh_f(v);
          } else if (EPI == EPI_GELU_ERF) {
            a.out[r] = gelu_erf_f(v);
          } else {  // EPI_LOGITS
            if (a.out) a.out[r] = v;
            if (better(v, r, best_v, best_i)) { best_v = v; best_i = r; }
          }
        }
      }
    }
  }

  if (EPI == EPI_LOGITS) {
    // greedy argmax, lowest index on exact ties: workgroup best, then the last
    // workgroup to arrive folds the per-workgroup candidates in index order.
    __shared__ float sv[16];
    __shared__ int si[16];
    __shared__ int s_last;
    if (lane < 4) { sv[wave * 4 + lane] = best_v; si[wave * 4 + lane] = best_i; }
    __syncthreads();
    if (threadIdx.x == 0) {
      float bv = sv[0]; int bi = si[0];
      for (int k = 1; k < 16; ++k) if (better(sv[k], si[k], bv, bi)) { bv = sv[k]; bi = si[k]; }
      a.amax_val[blockIdx.x] = bv; a.amax_idx[blockIdx.x] = bi;
      __threadfence();
      const unsigned ticket = atomicAdd(a.counter, 1u);
      s_last = ticket == gridDim.x - 1;
    }
    __syncthreads();
    if (s_last) {
      __threadfence();
      float bv = -INFINITY; int bi = 0x7FFFFFFF;
      for (int k = threadIdx.x; k < (int)gridDim.x; k += kBlock) {
        const float v = __hip_atomic_load(a.amax_val + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int i = __hip_atomic_load(a.amax_idx + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (better(v, i, bv, bi)) { bv = v; bi = i; }
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off, 64); const int oi = __shfl_xor(bi, off, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
      }
      __syncthreads();
      if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
      __syncthreads();
      if (threadIdx.x == 0) {
        for (int k = 1; k < 4; ++k) if (better(sv[k], si[k], bv, bi)) { bv = sv[k]; bi = si[k]; }
        *a.token_out = bi;
        *a.counter = 0u;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Draw from the top-k tempered pmf (Alg. 1 samples the output distribution).  One workgroup: every thread keeps the
// best of the logits it owns (index = thread + 1024 j); k rounds of a workgroup-wide argmax (lowest index on ties)
// pick the candidates in rank order, the owner of a winner strikes it out and rescans only its own elements.
// Thread 0 then inverts the cumulative distribution at the uniform number of Philox-4x32-10 (Salmon et al., SC'11)
// for counter (sample, step, 0, 0): weights exp((l_j - l_max) / T) in rank order, binary32, summed sequentially.
__device__ __forceinline__ uint32_t philox4x32_10_first(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
  for (int r = 0; r < 10; ++r) {
    if (r) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
    const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
    c0 = n0; c1 = l1; c2 = n2; c3 = l0;
  }
  return c0;
}

__device__ __forceinline__ void sample_topk_body(const SampleArgs& a) {
  __shared__ float cv[kMaxTopK];
  __shared__ int ci[kMaxTopK];
  __shared__ float rv[16];
  __shared__ int ri[16];
  __shared__ int s_win;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float bv; int bi;
  auto scan = [&]() {
    bv = -INFINITY; bi = 0x7FFFFFFF;
    for (int i = tid; i < a.V; i += 1024) {
      const float v = a.logits[i];
      if (better(v, i, bv, bi)) { bv = v; bi = i; }
    }
  };
  scan();
  for (int r = 0; r < a.k; ++r) {
    float wv = bv; int wi = bi;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(wv, off, 64); const int oi = __shfl_xor(wi, off, 64);
      if (better(ov, oi, wv, wi)) { wv = ov; wi = oi; }
    }
    if (lane == 0) { rv[wave] = wv; ri[wave] = wi; }
    __syncthreads();
    if (tid == 0) {
      for (int w = 1; w < 16; ++w) if (better(rv[w], ri[w], wv, wi)) { wv = rv[w]; wi = ri[w]; }
      cv[r] = wv; ci[r] = wi; s_win = wi;
    }
    __syncthreads();
    if (bi == s_win && bi != 0x7FFFFFFF) { a.logits[bi] = -INFINITY; scan(); }   // only the owner's elements change
  }
  if (tid == 0) {
    const float lmax = cv[0];
    float total = 0.f;
    for (int j = 0; j < a.k; ++j) { cv[j] = expf((cv[j] - lmax) * a.inv_t); total += cv[j]; }
    const float u = (float)(philox4x32_10_first(a.ctr0, a.ctr1, 0u, 0u, a.key0, a.key1) >> 8) * (1.0f / 16777216.0f);
    const float target = u * total;
    float acc = 0.f;
    int tok = ci[a.k - 1];
    for (int j = 0; j < a.k; ++j) {
      acc += cv[j];
      if (target < acc) { tok = ci[j]; break; }
    }
    *a.token_out = tok;
  }
}
__global__ __launch_bounds__(1024) void k_sample_topk(SampleArgs a) { sample_topk_body(a); }
// one workgroup per sample of a batch: sample j works on row j of the logits with its own counter
__global__ __launch_bounds__(1024) void k_sample_topk_batch(SampleBatchArgs b) {
  const int j = blockIdx.x;
  const SampleArgs a{b.logits + (long)j * b.stride, b.V, b.k, b.inv_t, b.ctr0[j], b.ctr1[j], b.key0, b.key1, b.token_out + j};
  sample_topk_body(a);
}
void launch_sample_topk(hipStream_t s, const SampleArgs& a) { hipLaunchKernelGGL(k_sample_topk, dim3(1), dim3(1024), 0, s, a); }
void launch_sample_topk_batch(hipStream_t s, int m, const SampleBatchArgs& a) { hipLaunchKernelGGL(k_sample_topk_batch, dim3(m), dim3(1024), 0, s, a); }

// c1[r] = sum_k W[r][k] g[k], c2[r] = sum_k W[r][k] b[k] for a bf16 matrix W [N, Kd]: what LayerNorm's mean and bias
// contribute to a product whose input travels as x * gain (the batched decode pass).  One wavefront per row.
__global__ __launch_bounds__(256) void k_row_dots(const bf16_t* W, int N, int Kd, const float* g, const float* b, float* c1, float* c2) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= N) return;
  float s1 = 0.f, s2 = 0.f;
  for (int k = lane; k < Kd; k += 64) {
    const float w = load_kind(W, IN_BF16, (long)row * Kd + k);
    s1 += w * g[k];
    s2 += w * (b ? b[k] : 0.f);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) { s1 += __shfl_xor(s1, off, 64); s2 += __shfl_xor(s2, off, 64); }
  if (lane == 0) { c1[row] = s1; c2[row] = s2; }
}
void launch_row_dots(hipStream_t s, const void* W, int N, int Kd, const float* g, const float* b, float* c1, float* c2) {
  hipLaunchKernelGGL(k_row_dots, dim3((N + 3) / 4), dim3(256), 0, s, (const bf16_t*)W, N, Kd, g, b, c1, c2);
}

int gemv_grid(int N) {
  const int n_groups = (N + 3) / 4;
  const int blocks = (n_groups + 3) / 4;
  return blocks < 1024 ? blocks : 1024;
}

template <typename WT>
static void launch_gemv_t(hipStream_t s, int pro, int epi, const GemvArgs& a) {
  const dim3 grid(gemv_grid(a.N)), block(kBlock);
  const size_t lds = (size_t)(a.Kd + 8) * sizeof(float);
#define MDI_GEMV(P, E) hipLaunchKernelGGL((k_gemv<WT, P, E>), grid, block, lds, s, a)
  if (pro == PRO_NORM) {
    switch (epi) {
      case EPI_QKV: MDI_GEMV(PRO_NORM, EPI_QKV); break;
      case EPI_SWIGLU: MDI_GEMV(PRO_NORM, EPI_SWIGLU); break;
      case EPI_GELU_TANH: MDI_GEMV(PRO_NORM, EPI_GELU_TANH); break;
      case EPI_GELU_ERF: MDI_GEMV(PRO_NORM, EPI_GELU_ERF); break;
      case EPI_LOGITS: MDI_GEMV(PRO_NORM, EPI_LOGITS); break;
      default: break;
    }
  } else {
    switch (epi) {
      case EPI_RESID: MDI_GEMV(PRO_COPY, EPI_RESID); break;
      default: break;
    }
  }
#undef MDI_GEMV
}

void launch_gemv(hipStream_t s, int dtype, int pro, int epi, const GemvArgs& a) {
  if (dtype == MDI_BF16) launch_gemv_t<bf16_t>(s, pro, epi, a); else launch_gemv_t<float>(s, pro, epi, a);
}

// ---------------------------------------------------------------------------
// Single-query attention over the sample's paged KV cache.
//
// Grid = (head groups, context splits, query rows).  A workgroup scans its slice
// of the context for one kv head and the G query heads that share it (GQA), so
// keys/values are read once per group.  A token's head vector is spread over
// L = h*sizeof(T)/16 lanes (one 16-byte load each); a wavefront therefore takes
// 64/L tokens per step.  Scores are completed with xor-shuffles inside the L-lane
// group, each group keeps an online-softmax state (max, sum, weighted V
// fragment), groups are merged by butterflies, wavefronts through LDS, and
// context splits through a partials buffer that the last-arriving workgroup
// folds in split order (no float atomics: results are run-to-run identical).
constexpr float kNegBig = -1e30f;

template <int G, int V>
struct SoftAcc {
  float m[G], l[G], o[G][V];
};

template <typename KT, int G>
__global__ __launch_bounds__(kBlock) void k_attn(AttnArgs a) {
  constexpr int V = Storage<KT>::kVec;
  const int h = a.h;
  const int L = h / V;                  // lanes per token (power of two)
  const int tpw = 64 / L;               // tokens per wavefront step
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hg = blockIdx.x;            // head group: query heads hg*G .. hg*G+G-1
  const int kvh = (hg * G) / (a.H / a.K);
  const int split = blockIdx.y;
  const int qrow = blockIdx.z;
  const int ctx = a.ctx0 + qrow;
  const int s0 = split * a.chunk;
  const int s1 = min(ctx, s0 + a.chunk);
  const int hoff = (lane % L) * V;
  const int sub = lane / L;

  float qf[G][V];
  const float* q = a.q + qrow * a.q_stride + (long)hg * G * h + hoff;
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < V; ++e) qf[g][e] = q[g * h + e] * a.scale;

  SoftAcc<G, V> st;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    st.m[g] = kNegBig; st.l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < V; ++e) st.o[g][e] = 0.f;
  }

  const KT* pool = (const KT*)a.pool;
  const long pt_h = (long)a.pt * h;
  for (int t0 = s0 + wave * tpw; t0 < s1; t0 += 4 * tpw) {
    const int tok = t0 + sub;
    const bool valid = tok < s1;
    const int tk = valid ? tok : s1 - 1;
    // coherent load: the entry may have been written by the previous launch from another compute die
    const int page = __hip_atomic_load(a.table + tk / a.pt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const KT* kp = pool + ((long)page * a.K + kvh) * 2 * pt_h + (long)(tk % a.pt) * h + hoff;
    float kf[V], vf[V];
    Storage<KT>::load(kp, kf);
    Storage<KT>::load(kp + pt_h, vf);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < V; ++e) s = fmaf(qf[g][e], kf[e], s);
      for (int off = 1; off < L; off <<= 1) s += __shfl_xor(s, off, 64);
      if (valid) {
        const float mn = fmaxf(st.m[g], s);
        const float alpha = __expf(st.m[g] - mn), p = __expf(s - mn);
        st.m[g] = mn;
        st.l[g] = st.l[g] * alpha + p;
#pragma unroll
        for (int e = 0; e < V; ++e) st.o[g][e] = st.o[g][e] * alpha + p * vf[e];
      }
    }
  }

  // merge the token sub-groups of the wavefront
  for (int off = L; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mo = __shfl_xor(st.m[g], off, 64), lo = __shfl_xor(st.l[g], off, 64);
      const float mn = fmaxf(st.m[g], mo);
      const float sa = __expf(st.m[g] - mn), sb = __expf(mo - mn);
      st.l[g] = st.l[g] * sa + lo * sb;
#pragma unroll
      for (int e = 0; e < V; ++e) st.o[g][e] = st.o[g][e] * sa + __shfl_xor(st.o[g][e], off, 64) * sb;
      st.m[g] = mn;
    }
  }

  // merge the four wavefronts through LDS: layout [wave][g][h + 2]
  extern __shared__ float sm[];
  const int rec = h + 2;
  if (sub == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float* r = sm + (wave * G + g) * rec;
#pragma unroll
      for (int e = 0; e < V; ++e) r[hoff + e] = st.o[g][e];
      if (hoff == 0) { r[h] = st.m[g]; r[h + 1] = st.l[g]; }
    }
  }
  __syncthreads();

  const bool single = a.n_splits == 1;
  for (int idx = threadIdx.x; idx < G * h; idx += kBlock) {
    const int g = idx / h, e = idx - g * h;
    float m = kNegBig;
    for (int w = 0; w < 4; ++w) m = fmaxf(m, sm[(w * G + g) * rec + h]);
    float l = 0.f, o = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float* r = sm + (w * G + g) * rec;
      const float sc = __expf(r[h] - m);
      l += r[h + 1] * sc; o += r[e] * sc;
    }
    const int head = hg * G + g;
    if (single) {
      store_kind(a.out, a.out_kind, qrow * a.out_stride + (long)head * h + e, o / l);
    } else {
      float* pr = a.part + ((long)head * kMaxSplits + split) * rec;
      pr[e] = o;
      if (e == 0) { pr[h] = m; pr[h + 1] = l; }
    }
  }
  if (single) return;

  __shared__ int s_last;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned ticket = atomicAdd(a.counters + hg, 1u);
    s_last = ticket == (unsigned)a.n_splits - 1;
  }
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  for (int idx = threadIdx.x; idx < G * h; idx += kBlock) {
    const int g = idx / h, e = idx - g * h;
    const int head = hg * G + g;
    const float* pr = a.part + (long)head * kMaxSplits * rec;
    float m = kNegBig;
    for (int sp = 0; sp < a.n_splits; ++sp)
      m = fmaxf(m, __hip_atomic_load(pr + sp * rec + h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    float l = 0.f, o = 0.f;
    for (int sp = 0; sp < a.n_splits; ++sp) {
      const float* r = pr + sp * rec;
      const float sc = __expf(__hip_atomic_load(r + h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - m);
      l += __hip_atomic_load(r + h + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * sc;
      o += __hip_atomic_load(r + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * sc;
    }
    store_kind(a.out, a.out_kind, qrow * a.out_stride + (long)head * h + e, o / l);
  }
  if (threadIdx.x == 0) a.counters[hg] = 0u;
}

template <typename KT>
static void launch_attn_t(hipStream_t s, const AttnArgs& a) {
  const int group = a.H / a.K;
  const int G = (group == 8 || group == 4 || group == 2) ? group : 1;
  const dim3 grid(a.H / G, a.n_splits, a.n_q), block(kBlock);
  const size_t lds = (size_t)4 * G * (a.h + 2) * sizeof(float);
  switch (G) {
    case 8: hipLaunchKernelGGL((k_attn<KT, 8>), grid, block, lds, s, a); break;
    case 4: hipLaunchKernelGGL((k_attn<KT, 4>), grid, block, lds, s, a); break;
    case 2: hipLaunchKernelGGL((k_attn<KT, 2>), grid, block, lds, s, a); break;
    default: hipLaunchKernelGGL((k_attn<KT, 1>), grid, block, lds, s, a); break;
  }
}

void launch_attn(hipStream_t s, int dtype, const AttnArgs& a) {
  if (dtype == MDI_BF16) launch_attn_t<bf16_t>(s, a); else launch_attn_t<float>(s, a);
}

}  // namespace mdi
