// First-visit kernels: all T prompt positions of a sample go through the local
// layers at once and fill the sample's KV cache (Alg. 1 round 0, Alg. 2 "first
// iteration for current sample").  With T rows the linear layers are dense
// contractions, so in bf16 mode they run on the matrix cores
// (v_mfma_f32_32x32x16_bf16, LDS-tiled); fp32 mode keeps exact fp32 products on
// the vector ALUs.
#include <algorithm>

#include <mutex>

#include "device_utils.h"

namespace mdi {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_rows_input(RowsInArgs a) {
  const int t = blockIdx.x;
  float* xr = a.xres + (long)t * a.d;
  if (a.in_kind == IN_TOKEN) {
    const long tok = checked_token(a.in, t, a.vocab, a.err);
    const int wk = a.dtype == MDI_BF16 ? IN_BF16 : IN_F32;
    for (int i = threadIdx.x; i < a.d; i += kBlock) {
      float v = load_kind(a.wte, wk, tok * a.d + i);
      if (a.wpe) v += load_kind(a.wpe, wk, (long)(a.pos0 + t) * a.d + i);
      xr[i] = v;
    }
  } else {
    for (int i = threadIdx.x; i < a.d; i += kBlock) xr[i] = load_kind(a.in, a.in_kind, (long)t * a.d + i);
  }
}
void launch_rows_input(hipStream_t s, const RowsInArgs& a) {
  hipLaunchKernelGGL(k_rows_input, dim3(a.T), dim3(kBlock), 0, s, a);
}

// ---------------------------------------------------------------------------
// One workgroup per row; d is a multiple of 8, so rows are read as float4 and written four values at a time.
__global__ __launch_bounds__(kBlock) void k_norm_rows(NormRowsArgs a) {
  __shared__ float red[8];
  const int t = blockIdx.x, d4 = a.d >> 2;
  const float4* x = reinterpret_cast<const float4*>(a.x + (long)t * a.d);
  const float4* g4 = reinterpret_cast<const float4*>(a.g);
  const float4* b4 = reinterpret_cast<const float4*>(a.b);
  float mean = 0.f, rstd;
  if (a.norm_kind == MDI_NORM_LAYERNORM) {
    float s = 0.f;
    for (int i = threadIdx.x; i < d4; i += kBlock) { const float4 v = x[i]; s += (v.x + v.y) + (v.z + v.w); }
    mean = block_sum(s, red) / (float)a.d;
    float s2 = 0.f;
    for (int i = threadIdx.x; i < d4; i += kBlock) {
      const float4 v = x[i];
      const float c0 = v.x - mean, c1 = v.y - mean, c2 = v.z - mean, c3 = v.w - mean;
      s2 += (c0 * c0 + c1 * c1) + (c2 * c2 + c3 * c3);
    }
    rstd = 1.f / sqrtf(block_sum(s2, red) / (float)a.d + a.eps);
  } else {
    float s2 = 0.f;
    for (int i = threadIdx.x; i < d4; i += kBlock) { const float4 v = x[i]; s2 += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w); }
    rstd = 1.f / sqrtf(block_sum(s2, red) / (float)a.d + a.eps);
  }
  for (int i = threadIdx.x; i < d4; i += kBlock) {
    const float4 v = x[i], g = g4[i];
    float4 o = {(v.x - mean) * rstd * g.x, (v.y - mean) * rstd * g.y, (v.z - mean) * rstd * g.z, (v.w - mean) * rstd * g.w};
    if (a.b) { const float4 b = b4[i]; o.x += b.x; o.y += b.y; o.z += b.z; o.w += b.w; }
    const long at = (long)t * a.d + 4 * i;
    if (a.out_kind == IN_BF16) {
      uint2 p;
      p.x = (uint32_t)f32_to_bf16(o.x) | ((uint32_t)f32_to_bf16(o.y) << 16);
      p.y = (uint32_t)f32_to_bf16(o.z) | ((uint32_t)f32_to_bf16(o.w) << 16);
      *reinterpret_cast<uint2*>((bf16_t*)a.out + at) = p;
    } else {
      *reinterpret_cast<float4*>((float*)a.out + at) = o;
    }
  }
}
void launch_norm_rows(hipStream_t s, const NormRowsArgs& a) {
  hipLaunchKernelGGL(k_norm_rows, dim3(a.T), dim3(kBlock), 0, s, a);
}

// ---------------------------------------------------------------------------
// Epilogue shared by both GEMM kernels.  (t, n) is the output coordinate, v the
// accumulated dot product, partner the value of column n^1 (SwiGLU pairs).
template <int EPI>
__device__ __forceinline__ void gemm_store(const GemmArgs& a, int out_kind, int t, int n, float v, float partner) {
  if (t >= a.T || n >= a.N) return;
  if (EPI == GEPI_SWIGLU) {
    if (n & 1) return;
    store_kind(a.out_act, out_kind, (long)t * (a.N >> 1) + (n >> 1), silu_f(v) * partner);
    return;
  }
  if (a.bias) v += a.bias[n];
  const long o = (long)t * a.N + n;
  if (EPI == GEPI_F32_BIAS) {
    a.out_f32[o] = v;
  } else if (EPI == GEPI_RESID) {
    v += a.out_f32[o];
    a.out_f32[o] = v;
    if (a.out_act) store_kind(a.out_act, out_kind, o, v);
  } else if (EPI == GEPI_GELU_TANH) {
    store_kind(a.out_act, out_kind, o, gelu_tanh_f(v));
  } else {
    store_kind(a.out_act, out_kind, o, gelu_erf_f(v));
  }
}

// ---------------------------------------------------------------------------
// bf16 GEMM on MFMA: C[T, N] = A[T, Kd] * W[N, Kd]^T, fp32 accumulate.
// Workgroup tile BM (tokens) x BN (weight rows), K step 64; four wavefronts in a
// 2 x 2 arrangement, each owning (BM/2) x (BN/2) as MFMA tiles of 32 x 32.
// Both operands are K-contiguous, so a lane's MFMA fragment (8 consecutive k of
// one row) is one 16-byte LDS read; LDS rows are padded by 16 bytes, which makes
// the 16 lanes served together hit 16 different bank groups.  LDS is double
// buffered and fed from two register stages, so a K step costs one workgroup barrier and a
// global load has two K steps to arrive.
constexpr int BK = 64, LDS_STRIDE = BK + 8;

// NW wavefronts in a WM x (NW / WM) arrangement.  Shapes in use: 4 wavefronts (2 x 2) on tiles of 128 x 128 or
// 128 x 64, two workgroups per compute unit; 8 wavefronts on 256 x 192 (4 x 2) or 128 x 128 (2 x 4), one workgroup
// per compute unit.  What a compute unit can pull out of L2 per unit of time is the bound on this machine (about 65 GB/s each,
// measured): a 128 x 128 tile needs 256 bytes of operands per 128 x 128 x 1 products, a 256 x 192 tile 0.58 of that.
template <int EPI, int BM, int BN, int NW, int WM>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(1, 2))) void k_gemm_bf16(GemmArgs a) {
  constexpr int kThreads = NW * 64, WN = NW / WM;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;  // MFMA tiles per wavefront
  constexpr int PA = BM * 8 / kThreads, PB = BN * 8 / kThreads;   // 16-byte pieces per thread per K step
  constexpr int PROWS = kThreads / 8;                  // tile rows covered by one piece per thread
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && (BM * 8) % kThreads == 0 && (BN * 8) % kThreads == 0, "tile shape");
  extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem[];
  bf16_t* As = (bf16_t*)gemm_smem;                     // [2][BM][LDS_STRIDE]
  bf16_t* Bs = As + 2 * BM * LDS_STRIDE;               // [2][BN][LDS_STRIDE]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / WN) * (BM / WM), wn = (wave % WN) * (BN / WN);
  // Workgroup -> tile.  Workgroups are handed to the eight compute dies in turn (die = id % 8) and each die has an
  // L2 of its own, so die c takes the tile columns c, c + 8, ... and walks down a column (all row tiles of the same
  // weight rows) before moving on: the weight tile is fetched from memory once, by one die, while the workgroups
  // that share it are running; the activation tiles are the ones every column of a die re-uses.
  const int m_tiles = (a.T + BM - 1) / BM, n_tiles = (a.N + BN - 1) / BN;
  const int die = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int tile_m = seq % m_tiles, tile_n = die + 8 * (seq / m_tiles);
  if (tile_n >= n_tiles) return;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const bf16_t* A = (const bf16_t*)a.A;
  const bf16_t* W = (const bf16_t*)a.W;
  const int Kd = a.Kd;

  // piece p of a tile covers row p / 8, k-offset (p % 8) * 8; rows past the matrix re-read its last row
  const int prow = tid >> 3, pk = (tid & 7) * 8;
  const bf16_t* ga[PA];
  const bf16_t* gb[PB];
#pragma unroll
  for (int i = 0; i < PA; ++i) ga[i] = A + (long)min(m0 + prow + i * PROWS, a.T - 1) * Kd + pk;
#pragma unroll
  for (int i = 0; i < PB; ++i) gb[i] = W + (long)min(n0 + prow + i * PROWS, a.N - 1) * Kd + pk;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const u32x4 z4 = {0u, 0u, 0u, 0u};
  // Two register stages: while step k is multiplied out of LDS, the operands of step k + 1 wait in one stage to be
  // written to the other LDS buffer and those of step k + 2 are still on their way into the second stage, so a
  // global load has two K steps of arithmetic to arrive (one is not enough, a third stage costs more registers
  // than it gains).
  u32x4 ra0[PA], rb0[PB], ra1[PA], rb1[PB];
  const int nk = (Kd + BK - 1) / BK;
  auto fetch_full = [&](u32x4 (&ra)[PA], u32x4 (&rb)[PB], int step) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < PA; ++i) ra[i] = *reinterpret_cast<const u32x4*>(ga[i] + step * BK);
#pragma unroll
    for (int i = 0; i < PB; ++i) rb[i] = *reinterpret_cast<const u32x4*>(gb[i] + step * BK);
  };
  auto fetch_guarded = [&](u32x4 (&ra)[PA], u32x4 (&rb)[PB], int step) __attribute__((always_inline)) {
    const bool ok = step * BK + pk < Kd;              // steps past the matrix, and its last columns when Kd % 64 != 0, are zero
#pragma unroll
    for (int i = 0; i < PA; ++i) ra[i] = ok ? *reinterpret_cast<const u32x4*>(ga[i] + step * BK) : z4;
#pragma unroll
    for (int i = 0; i < PB; ++i) rb[i] = ok ? *reinterpret_cast<const u32x4*>(gb[i] + step * BK) : z4;
  };
  auto stash = [&](const u32x4 (&ra)[PA], const u32x4 (&rb)[PB], int buf) __attribute__((always_inline)) {
    bf16_t* An = As + buf * BM * LDS_STRIDE;
    bf16_t* Bn = Bs + buf * BN * LDS_STRIDE;
#pragma unroll
    for (int i = 0; i < PA; ++i) *reinterpret_cast<u32x4*>(An + (prow + i * PROWS) * LDS_STRIDE + pk) = ra[i];
#pragma unroll
    for (int i = 0; i < PB; ++i) *reinterpret_cast<u32x4*>(Bn + (prow + i * PROWS) * LDS_STRIDE + pk) = rb[i];
  };
  auto multiply = [&](int buf) __attribute__((always_inline)) {
    const bf16_t* Ac = As + buf * BM * LDS_STRIDE;
    const bf16_t* Bc = Bs + buf * BN * LDS_STRIDE;
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      const int kk = ks + (lane >> 5) * 8;
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(Ac + (wm + i * 32 + (lane & 31)) * LDS_STRIDE + kk);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(Bc + (wn + j * 32 + (lane & 31)) * LDS_STRIDE + kk);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };

  // One K step: multiply the step in LDS buffer `buf`; write the step waiting in a register stage into the other
  // buffer and refill that stage with step `fstep`; one barrier.  (Letting the two halves of an 8-wavefront
  // workgroup take the two parts in opposite order, one multiplying while the other moves data, was measured: no
  // faster.)
  auto kstep = [&](int buf, u32x4 (&ra)[PA], u32x4 (&rb)[PB], bool move, int fstep, bool full) __attribute__((always_inline)) {
    multiply(buf);
    if (move) {
      stash(ra, rb, buf ^ 1);
      if (full) fetch_full(ra, rb, fstep); else fetch_guarded(ra, rb, fstep);
    }
    __syncthreads();
  };

  // invariant at an even step k: LDS buffer 0 holds step k, stage 0 step k + 1, stage 1 step k + 2
  int k = 0;
  if (5 * BK <= Kd) {
    // The usual case has its own, branch-free lead-in, so that the loop below is entered with its loads outstanding
    // in the order the loop itself issues them (the compiler then waits for one stage while the other is in flight).
    fetch_full(ra0, rb0, 0);
    stash(ra0, rb0, 0);
    fetch_full(ra0, rb0, 1);
    __builtin_amdgcn_sched_barrier(0);              // the two stages' loads must not be interleaved
    fetch_full(ra1, rb1, 2);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    for (; (k + 5) * BK <= Kd; k += 2) {            // every fetch below is of a whole step inside the matrix
      kstep(0, ra0, rb0, true, k + 3, true);
      kstep(1, ra1, rb1, true, k + 4, true);
    }
  } else {
    fetch_guarded(ra0, rb0, 0);
    stash(ra0, rb0, 0);
    fetch_guarded(ra0, rb0, 1);
    fetch_guarded(ra1, rb1, 2);
    __syncthreads();
  }
  for (; k < nk; k += 2) {
    kstep(0, ra0, rb0, k + 1 < nk, k + 3, false);
    if (k + 1 < nk) kstep(1, ra1, rb1, k + 2 < nk, k + 4, false);
  }

  // accumulator layout of the 32x32 MFMA: register r of lane l holds
  // C[row = 8*(r/4) + 4*(l/32) + r%4][col = l%32].  Per MFMA tile a lane owns one column n and 16 rows:
  // everything it needs from memory (bias, residual) is fetched before the first store, so the loads
  // are in flight together instead of one round trip per element.
  float* __restrict__ out_f32 = a.out_f32;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn + j * 32 + (lane & 31);
      const int tb = m0 + wm + i * 32 + 4 * (lane >> 5);
      const bool n_ok = n < a.N;
      const float bias = (EPI != GEPI_SWIGLU && a.bias && n_ok) ? a.bias[n] : 0.f;
      float res[16];
      if (EPI == GEPI_RESID) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int t = tb + 8 * (r >> 2) + (r & 3);
          res[r] = (n_ok && t < a.T) ? out_f32[(long)t * a.N + n] : 0.f;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int t = tb + 8 * (r >> 2) + (r & 3);
        float v = acc[i][j][r];
        if (EPI == GEPI_SWIGLU) {
          const float partner = __shfl_xor(v, 1, 64);          // column n^1: rows (2f, 2f+1) = (gate_f, up_f)
          if (n_ok && t < a.T && !(n & 1)) store_kind(a.out_act, IN_BF16, (long)t * (a.N >> 1) + (n >> 1), silu_f(v) * partner);
        } else if (n_ok && t < a.T) {
          const long o = (long)t * a.N + n;
          v += bias;
          if (EPI == GEPI_F32_BIAS) {
            out_f32[o] = v;
          } else if (EPI == GEPI_RESID) {
            v += res[r];
            out_f32[o] = v;
            if (a.out_act) store_kind(a.out_act, IN_BF16, o, v);
          } else if (EPI == GEPI_GELU_TANH) {
            store_kind(a.out_act, IN_BF16, o, gelu_tanh_f(v));
          } else {
            store_kind(a.out_act, IN_BF16, o, gelu_erf_f(v));
          }
        }
      }
    }
}

// ---------------------------------------------------------------------------
// fp32 GEMM on the vector ALUs (exact fp32 products; used by the fp32 mode whose
// parity bar is 1e-4).  64 x 64 tile, K step 16, each thread a 4 x 4 block.
template <int EPI>
__global__ __launch_bounds__(kBlock) void k_gemm_f32(GemmArgs a) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;   // n block, t block
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const float* A = (const float*)a.A;
  const float* W = (const float*)a.W;
  const int Kd = a.Kd;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < Kd; k0 += 16) {
    {
      // 64 rows x 16 k per operand = 1024 values, 4 per thread (one float4 along k)
      const int r = tid >> 2, kk = (tid & 3) * 4;
      const int ar = min(m0 + r, a.T - 1), br = min(n0 + r, a.N - 1);
      float4 va = {0, 0, 0, 0}, vb = {0, 0, 0, 0};
      if (k0 + kk < Kd) {   // Kd is a multiple of 8, so a float4 never straddles the end
        va = *reinterpret_cast<const float4*>(A + (long)ar * Kd + k0 + kk);
        vb = *reinterpret_cast<const float4*>(W + (long)br * Kd + k0 + kk);
      }
      __syncthreads();
      As[kk][r] = va.x; As[kk + 1][r] = va.y; As[kk + 2][r] = va.z; As[kk + 3][r] = va.w;
      Bs[kk][r] = vb.x; Bs[kk + 1][r] = vb.y; Bs[kk + 2][r] = vb.z; Bs[kk + 3][r] = vb.w;
      __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[k][ty * 4 + i]; bv[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      gemm_store<EPI>(a, IN_F32, m0 + ty * 4 + i, n0 + tx * 4 + j, acc[i][j], acc[i][j ^ 1]);
}

template <int BM, int BN, int NW, int WM>
static void launch_gemm_bf16(hipStream_t s, int epi, const GemmArgs& a) {
  const int m_tiles = (a.T + BM - 1) / BM, n_tiles = (a.N + BN - 1) / BN;
  const dim3 grid(8 * m_tiles * ((n_tiles + 7) / 8)), block(NW * 64);   // see the tile mapping in the kernel
  const size_t lds = (size_t)2 * (BM + BN) * LDS_STRIDE * sizeof(bf16_t);
  if (lds > 64 * 1024) {                             // 256 x 192 tiles need more LDS than a kernel gets by default
    static std::once_flag raised;
    std::call_once(raised, [&]() {
      (void)hipFuncSetAttribute((const void*)k_gemm_bf16<GEPI_F32_BIAS, BM, BN, NW, WM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      (void)hipFuncSetAttribute((const void*)k_gemm_bf16<GEPI_RESID, BM, BN, NW, WM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      (void)hipFuncSetAttribute((const void*)k_gemm_bf16<GEPI_SWIGLU, BM, BN, NW, WM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      (void)hipFuncSetAttribute((const void*)k_gemm_bf16<GEPI_GELU_TANH, BM, BN, NW, WM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      (void)hipFuncSetAttribute((const void*)k_gemm_bf16<GEPI_GELU_ERF, BM, BN, NW, WM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
  }
  switch (epi) {
    case GEPI_F32_BIAS: hipLaunchKernelGGL((k_gemm_bf16<GEPI_F32_BIAS, BM, BN, NW, WM>), grid, block, lds, s, a); break;
    case GEPI_RESID: hipLaunchKernelGGL((k_gemm_bf16<GEPI_RESID, BM, BN, NW, WM>), grid, block, lds, s, a); break;
    case GEPI_SWIGLU: hipLaunchKernelGGL((k_gemm_bf16<GEPI_SWIGLU, BM, BN, NW, WM>), grid, block, lds, s, a); break;
    case GEPI_GELU_TANH: hipLaunchKernelGGL((k_gemm_bf16<GEPI_GELU_TANH, BM, BN, NW, WM>), grid, block, lds, s, a); break;
    default: hipLaunchKernelGGL((k_gemm_bf16<GEPI_GELU_ERF, BM, BN, NW, WM>), grid, block, lds, s, a); break;
  }
}

void launch_gemm(hipStream_t s, int dtype, int epi, const GemmArgs& a) {
  if (dtype == MDI_BF16) {
    // 256 x 192 tiles (one 8-wavefront workgroup per compute unit) when the grid they give keeps at least 70 % of
    // the compute units busy over its rounds
    static const long n_cu = []() {
      int dev = 0, n = 0;
      if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
      return (long)n;
    }();
    const long big = (long)((a.N + 191) / 192) * ((a.T + 255) / 256);
    const long rounds = (big + n_cu - 1) / n_cu;
    if (a.T >= 256 && big * 10 >= rounds * n_cu * 7) { launch_gemm_bf16<256, 192, 8, 4>(s, epi, a); return; }
    // 256 x 128 tiles when they give one round that keeps at least 70 % of the compute units busy (2048 rows x 4096
    // outputs: exactly one tile each): a quarter less operand traffic per product than 128 x 128 tiles
    const long mid = (long)((a.N + 127) / 128) * ((a.T + 255) / 256);
    if (a.T >= 256 && mid <= n_cu && mid * 10 >= n_cu * 7) { launch_gemm_bf16<256, 128, 8, 4>(s, epi, a); return; }
    // a grid of 128 x 128 tiles that cannot give every compute unit two 4-wavefront workgroups: one 8-wavefront
    // workgroup each (a third less operand traffic than two 128 x 64 tiles), or narrower tiles when even that
    // leaves compute units idle
    const long tiles = (long)((a.N + 127) / 128) * ((a.T + 127) / 128);
    // (few rows and a narrow product: even 128 x 64 tiles leave compute units without a workgroup; 64 x 64 tiles give
    // twice as many)
    const long narrow = (long)((a.N + 63) / 64) * ((a.T + 127) / 128);
    if (tiles <= n_cu && 2 * tiles > n_cu) launch_gemm_bf16<128, 128, 8, 2>(s, epi, a);
    else if (2 * tiles <= n_cu && narrow < n_cu) launch_gemm_bf16<64, 64, 4, 2>(s, epi, a);
    else if (2 * tiles <= n_cu) launch_gemm_bf16<128, 64, 4, 2>(s, epi, a);
    else launch_gemm_bf16<128, 128, 4, 2>(s, epi, a);
    return;
  }
  const dim3 grid((a.N + 63) / 64, (a.T + 63) / 64), block(kBlock);
  switch (epi) {
    case GEPI_F32_BIAS: hipLaunchKernelGGL((k_gemm_f32<GEPI_F32_BIAS>), grid, block, 0, s, a); break;
    case GEPI_RESID: hipLaunchKernelGGL((k_gemm_f32<GEPI_RESID>), grid, block, 0, s, a); break;
    case GEPI_SWIGLU: hipLaunchKernelGGL((k_gemm_f32<GEPI_SWIGLU>), grid, block, 0, s, a); break;
    case GEPI_GELU_TANH: hipLaunchKernelGGL((k_gemm_f32<GEPI_GELU_TANH>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((k_gemm_f32<GEPI_GELU_ERF>), grid, block, 0, s, a); break;
  }
}

// ---------------------------------------------------------------------------
// Rotate q and k by their positions, keep q in fp32 for the attention kernel
// and scatter k, v into the sample's pages.  One workgroup per prompt position.
__global__ __launch_bounds__(kBlock) void k_rope_scatter(RopeScatterArgs a) {
  const int t = blockIdx.x, h = a.h, half = h >> 1;
  const int n_heads = a.H + 2 * a.K;
  if (t >= a.T) {                                   // padding rows of the attention operand: keys nobody may see, but finite
    for (int i = threadIdx.x; i < a.K * h; i += kBlock) a.k_bf[((long)(i / h) * a.ldk + a.pos0 + t) * h + i % h] = 0;
    return;
  }
  const float* row = a.qkv + (long)t * n_heads * h;
  const int pos = a.pos0 + t;
  const int page = a.table[pos / a.pt], slot = pos % a.pt;
  const long pt_h = (long)a.pt * h;
  const bool bf = a.dtype == MDI_BF16;
  // four consecutive pairs (i, i + h/2) per thread: h/2 is a multiple of 4, so everything moves in 8- or 16-byte pieces
  auto put4 = [&](void* base, bool as_bf16, long o, const float4& v) __attribute__((always_inline)) {
    if (as_bf16) {
      uint2 w;
      w.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
      w.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
      *reinterpret_cast<uint2*>((bf16_t*)base + o) = w;
    } else {
      *reinterpret_cast<float4*>((float*)base + o) = v;
    }
  };
  const int q4 = half >> 2;
  for (int p = threadIdx.x; p < n_heads * q4; p += kBlock) {
    const int head = p / q4, i = (p - head * q4) * 4;
    float4 v0 = *reinterpret_cast<const float4*>(row + head * h + i);
    float4 v1 = *reinterpret_cast<const float4*>(row + head * h + i + half);
    if (a.rope && head < a.H + a.K) {
      const float4 c01 = *reinterpret_cast<const float4*>(a.rope + (long)pos * half + i);       // (cos, sin) of pairs i, i+1
      const float4 c23 = *reinterpret_cast<const float4*>(a.rope + (long)pos * half + i + 2);   // ... i+2, i+3
      const float4 r0 = {v0.x * c01.x - v1.x * c01.y, v0.y * c01.z - v1.y * c01.w, v0.z * c23.x - v1.z * c23.y, v0.w * c23.z - v1.w * c23.w};
      const float4 r1 = {v0.x * c01.y + v1.x * c01.x, v0.y * c01.w + v1.y * c01.z, v0.z * c23.y + v1.z * c23.x, v0.w * c23.w + v1.w * c23.z};
      v0 = r0; v1 = r1;
    }
    if (head < a.H) {
      const long o = (long)t * a.H * h + head * h + i;
      if (a.q_out) { put4(a.q_out, false, o, v0); put4(a.q_out, false, o + half, v1); }
      if (a.q_bf) {
        const float sc = a.scale;
        put4(a.q_bf, true, o, float4{v0.x * sc, v0.y * sc, v0.z * sc, v0.w * sc});
        put4(a.q_bf, true, o + half, float4{v1.x * sc, v1.y * sc, v1.z * sc, v1.w * sc});
      }
    } else {
      const bool is_v = head >= a.H + a.K;
      const int kvh = head - a.H - (is_v ? a.K : 0);
      const long o = (((long)page * a.K + kvh) * 2 + (is_v ? 1 : 0)) * pt_h + (long)slot * h + i;
      put4(a.pool, bf, o, v0);
      put4(a.pool, bf, o + half, v1);
      if (a.k_bf && !is_v) {
        const long k = ((long)kvh * a.ldk + pos) * h + i;
        put4(a.k_bf, true, k, v0);
        put4(a.k_bf, true, k + half, v1);
      }
    }
  }
}
void launch_rope_scatter(hipStream_t s, const RopeScatterArgs& a) {
  hipLaunchKernelGGL(k_rope_scatter, dim3(a.k_bf ? a.n_rows : a.T), dim3(kBlock), 0, s, a);
}

// ---------------------------------------------------------------------------
// set-up kernels
__global__ void k_rope_table(float2* table, int max_ctx, int half, int h, double base) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)max_ctx * half) return;
  const int p = idx / half, i = idx % half;
  const double ang = (double)p * pow(base, -2.0 * (double)i / (double)h);
  table[idx] = make_float2((float)cos(ang), (float)sin(ang));
}
void launch_rope_table(hipStream_t s, float2* table, int max_ctx, int h, double base) {
  const long n = (long)max_ctx * (h / 2);
  hipLaunchKernelGGL(k_rope_table, dim3((n + 255) / 256), dim3(256), 0, s, table, max_ctx, h / 2, h, base);
}

template <typename T>
__global__ void k_copy_rows(const T* src, T* dst, long rows, long cols, long row_mul, long row_off) {
  const long n = rows * cols;
  for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (long)gridDim.x * blockDim.x) {
    const long r = idx / cols, c = idx - r * cols;
    dst[(r * row_mul + row_off) * cols + c] = src[idx];
  }
}
void launch_copy_rows(hipStream_t s, int elem_bytes, const void* src, void* dst, long rows, long cols, long row_mul, long row_off) {
  const long n = rows * cols;
  if (n == 0) return;
  const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  if (elem_bytes == 2)
    hipLaunchKernelGGL(k_copy_rows<uint16_t>, dim3(blocks), dim3(256), 0, s, (const uint16_t*)src, (uint16_t*)dst, rows, cols, row_mul, row_off);
  else
    hipLaunchKernelGGL(k_copy_rows<uint32_t>, dim3(blocks), dim3(256), 0, s, (const uint32_t*)src, (uint32_t*)dst, rows, cols, row_mul, row_off);
}

__global__ void k_fill_u32(uint32_t* dst, long n, uint32_t v) {
  for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (long)gridDim.x * blockDim.x) dst[idx] = v;
}
void launch_fill_u32(hipStream_t s, uint32_t* dst, long n, uint32_t v) {
  if (n == 0) return;
  const int blocks = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
  hipLaunchKernelGGL(k_fill_u32, dim3(blocks), dim3(256), 0, s, dst, n, v);
}
void launch_fill_f32(hipStream_t s, float* dst, long n, float v) {
  uint32_t u;
  __builtin_memcpy(&u, &v, 4);
  launch_fill_u32(s, (uint32_t*)dst, n, u);
}

}  // namespace mdi
