// Causal attention of a first visit (all T prompt positions of a sample at once; Alg. 1 round 0,
// Alg. 2 "first iteration") on the matrix cores: bf16 operands, fp32 scores, softmax and output
// accumulation.
//
// Everything is computed transposed, S^T = K Q^T and O^T = V^T P^T, because of where the matrix
// core leaves its results: with v_mfma_f32_32x32x16_bf16, register r of lane l is element
// (row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32).  In the transposed products a column is a
// query, so each lane owns one query: its running maximum, its sum and the rescaling of its output
// are plain per-lane scalars (lanes l and l + 32 share a query and exchange two numbers per block of
// keys), and P^T leaves the first product in exactly the register layout the second one wants as
// its B operand, without any data movement.  The price is that the values are needed with the key
// index contiguous (A operand of V^T P^T), so a small kernel writes V transposed beforehand.
#include <mutex>

#include "device_utils.h"

namespace mdi {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BQ = 128;       // queries per workgroup (32 per wavefront)
constexpr int BK = 64;        // keys per step

// values of the T new positions: fp32 rows of the fused QKV product -> bf16 [kv head][h][ldk], row t at column
// pos0 + t; columns up to pos0 + n_cols - 1 are cleared (keys nobody may see, but finite)
__global__ __launch_bounds__(256) void k_v_transpose(const float* qkv, int T, int n_cols, int pos0, int ldk, int n_rows, int v_off, int h, bf16_t* vt) {
  __shared__ bf16_t tile[64][64 + 2];
  const int t0 = blockIdx.x * 64, c0 = blockIdx.y * 64;          // 64 positions x 64 channels of the K*h value channels
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int tt = i >> 6, c = i & 63;
    const int t = t0 + tt;
    tile[tt][c] = t < T ? f32_to_bf16(qkv[(long)t * n_rows + v_off + c0 + c]) : (bf16_t)0;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int c = i >> 6, tt = i & 63;
    if (t0 + tt < n_cols) vt[(long)(c0 + c) * ldk + pos0 + t0 + tt] = tile[tt][c];          // channel c0 + c = kv head * h + element
  }
}

// A later piece of a first visit attends to the positions already in the cache as well (Alg. 2: the cache is
// extended, never rebuilt): their keys and values are brought from the sample's pages into the operand arrays, keys
// as they are, values transposed.  One workgroup per (64 positions, 64 channels of one kv head).
__global__ __launch_bounds__(256) void k_cache_gather(const bf16_t* pool, const int32_t* table, int n_pos, int K, int h, int pt, int ldk,
                                                      bf16_t* k_bf, bf16_t* vt) {
  __shared__ bf16_t tile[64][64 + 2];
  const int t0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int kvh = c0 / h, e0 = c0 - kvh * h;
  const long pt_h = (long)pt * h;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int tt = i >> 6, c = i & 63;
    const int t = t0 + tt;
    if (t < n_pos) {
      const long base = ((long)table[t / pt] * K + kvh) * 2 * pt_h + (long)(t % pt) * h + e0 + c;
      k_bf[((long)kvh * ldk + t) * h + e0 + c] = pool[base];
      tile[tt][c] = pool[base + pt_h];
    } else {
      tile[tt][c] = (bf16_t)0;
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int c = i >> 6, tt = i & 63;
    if (t0 + tt < n_pos) vt[(long)(c0 + c) * ldk + t0 + tt] = tile[tt][c];
  }
}

// Two groups of four wavefronts work on the same 128 queries: group g takes the key blocks 2 i + g, so the longest
// workgroup (the last queries, which see every key) has half as many steps in a row, and a SIMD holds two wavefronts
// whose matrix and softmax arithmetic overlap.  The groups' running (maximum, sum, output) are folded through LDS at
// the end, group 0 first: the result does not depend on timing.
template <int HD>
__global__ __launch_bounds__(512) void k_flash_prefill(FlashArgs a) {
  constexpr int KS = HD + 8;            // LDS row stride of a key (elements): 16 bytes of padding spread the rows over the banks
  constexpr int VS = BK + 4;            // LDS row stride of a value channel: an odd number of 8-byte units
  constexpr int HT = HD / 32;           // 32-channel tiles of the output
  constexpr int KP = BK * HD / 8 / 256; // 16-byte pieces of a key block per thread of a group
  extern __shared__ __attribute__((aligned(16))) unsigned char flash_smem[];
  bf16_t* Ks_all = (bf16_t*)flash_smem;                 // [2][BK * KS]
  bf16_t* Vs_all = Ks_all + 2 * BK * KS;                // [2][HD * VS]

  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;   // position inside the group
  const int grp = threadIdx.x >> 8;
  bf16_t* Ks = Ks_all + grp * BK * KS;
  bf16_t* Vs = Vs_all + grp * HD * VS;
  const int qb = gridDim.x - 1 - blockIdx.x;                     // the longest rows first
  const int head = blockIdx.y, kvh = head / (a.H / a.K);
  const int q0 = qb * BQ, qw0 = q0 + 32 * wave;
  const int col = lane & 31, half = lane >> 5;
  const int query = qw0 + col;
  const long HH = (long)a.H * HD;

  // this lane's query as B operand of K Q^T: elements [16 ks + 8 half, + 8) for every step ks
  bf16x8 qf[HD / 16];
  {
    const bf16_t* qp = a.q + (long)min(query, a.T - 1) * HH + (long)head * HD + 8 * half;
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }

  f32x16 o[HT];
#pragma unroll
  for (int i = 0; i < HT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float m = -1e30f, l = 0.f;

  const bf16_t* kbase = a.k + (long)kvh * a.ldk * HD;
  const bf16_t* vbase = a.vt + (long)kvh * HD * a.ldk;
  const int p0 = a.p0;                                           // position of query 0: keys 0 .. p0 + query are visible
  const int n_kb = min((p0 + q0 + BQ + BK - 1) / BK, a.Tk / BK); // key blocks any query of this workgroup may see
  const int n_it = (n_kb + 1) / 2;                               // steps: block 2 it + grp each

  // staging registers: the next block's keys and values travel global -> registers during the arithmetic
  // (a group whose last step has no block re-reads block 0 and skips the arithmetic)
  u32x4 kreg[KP], vreg[KP];
  auto fetch = [&](int kb) {
    if (kb >= n_kb) kb = 0;
#pragma unroll
    for (int i = 0; i < KP; ++i) {
      const int p = tid + i * 256;                               // piece p: key p / (HD/8), elements 8 (p % (HD/8))
      kreg[i] = *reinterpret_cast<const u32x4*>(kbase + ((long)kb * BK + p / (HD / 8)) * HD + 8 * (p % (HD / 8)));
      const int c = p / (BK / 8), j = p % (BK / 8);              // channel c, keys [8 j, 8 j + 8) of the block
      vreg[i] = *reinterpret_cast<const u32x4*>(vbase + (long)c * a.ldk + (long)kb * BK + 8 * j);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int i = 0; i < KP; ++i) {
      const int p = tid + i * 256;
      *reinterpret_cast<u32x4*>(Ks + (p / (HD / 8)) * KS + 8 * (p % (HD / 8))) = kreg[i];
      const int c = p / (BK / 8), j = p % (BK / 8);
      u32x2* d = reinterpret_cast<u32x2*>(Vs + c * VS + 8 * j);  // 8-byte aligned: VS * 2 is a multiple of 8
      d[0] = u32x2{vreg[i].x, vreg[i].y};
      d[1] = u32x2{vreg[i].z, vreg[i].w};
    }
  };

  fetch(grp);
  for (int it = 0; it < n_it; ++it) {
    const int kb = 2 * it + grp;
    __syncthreads();                                             // everybody is done with the previous blocks
    stash();
    __syncthreads();
    if (it + 1 < n_it) fetch(kb + 2);
    const int k0 = kb * BK;
    if (kb >= n_kb || k0 > p0 + qw0 + 31) continue;              // no block, or this wavefront's queries see none of these keys

    // ---- S^T = K Q^T: two tiles of 32 keys x 32 queries
    f32x16 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
      const bf16_t* kr = Ks + (32 * t + col) * KS + 8 * half;
#pragma unroll
      for (int ks = 0; ks < HD / 16; ++ks)
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(kr + 16 * ks), qf[ks], s[t], 0, 0, 0);
    }
    // ---- causal mask and the lane's share of the row statistics (row of S = column here = this lane's query)
    float mloc = -1e30f;
    const bool diag = k0 + BK - 1 > p0 + qw0;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = k0 + 32 * t + 8 * (r >> 2) + 4 * half + (r & 3);
        if (diag && key > p0 + query) s[t][r] = -1e30f;
        mloc = fmaxf(mloc, s[t][r]);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float mn = fmaxf(m, mloc);
    const float alpha = __expf(m - mn);
    m = mn;
    float lsum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) { const float p = __expf(s[t][r] - mn); s[t][r] = p; lsum += p; }
    l = l * alpha + lsum;                                        // the two lanes of a query keep separate sums until the end
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[i][r] *= alpha;

    // ---- O^T += V^T P^T.  Step (t, pp) contracts keys [32 t + 16 pp, + 16); inside a step this half of the
    // wavefront supplies keys {0..3, 8..11} + 4 half, which is what registers 8 pp .. 8 pp + 7 of tile t hold
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int pp = 0; pp < 2; ++pp) {
        bf16x8 pf;
#pragma unroll
        for (int j = 0; j < 8; ++j) pf[j] = (__bf16)s[t][8 * pp + j];
        const bf16_t* vr = Vs + col * VS + 32 * t + 16 * pp + 4 * half;
#pragma unroll
        for (int i = 0; i < HT; ++i) {
          const u32x2 lo = *reinterpret_cast<const u32x2*>(vr + 32 * i * VS);
          const u32x2 hi = *reinterpret_cast<const u32x2*>(vr + 32 * i * VS + 8);
          const u32x4 vf = {lo.x, lo.y, hi.x, hi.y};
          o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf), pf, o[i], 0, 0, 0);
        }
      }
  }

  // ---- fold the two groups: group 1 hands its state over through LDS (the K/V area, no longer needed);
  //      element j of thread t at [j][t], so that a wavefront's accesses are consecutive
  float* fold = (float*)flash_smem;
  __syncthreads();
  if (grp == 1) {
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) fold[(i * 16 + r) * 256 + tid] = o[i][r];
    fold[(HT * 16) * 256 + tid] = m;
    fold[(HT * 16 + 1) * 256 + tid] = l;
  }
  __syncthreads();
  if (grp == 1) return;
  {
    const float m1 = fold[(HT * 16) * 256 + tid], l1 = fold[(HT * 16 + 1) * 256 + tid];
    const float mn = fmaxf(m, m1);
    const float a0 = __expf(m - mn), a1 = __expf(m1 - mn);       // a group that saw no key has m = -1e30, l = 0, o = 0
    l = l * a0 + l1 * a1;
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[i][r] = o[i][r] * a0 + fold[(i * 16 + r) * 256 + tid] * a1;
  }

  l += __shfl_xor(l, 32, 64);
  if (query < a.T) {
    const float inv = 1.f / l;
    bf16_t* op = a.out + (long)query * HH + (long)head * HD;
#pragma unroll
    for (int i = 0; i < HT; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {                              // four consecutive channels: 32 i + 8 g + 4 half + 0..3
        const uint32_t w0 = (uint32_t)f32_to_bf16(o[i][4 * g] * inv) | ((uint32_t)f32_to_bf16(o[i][4 * g + 1] * inv) << 16);
        const uint32_t w1 = (uint32_t)f32_to_bf16(o[i][4 * g + 2] * inv) | ((uint32_t)f32_to_bf16(o[i][4 * g + 3] * inv) << 16);
        *reinterpret_cast<u32x2*>(op + 32 * i + 8 * g + 4 * half) = u32x2{w0, w1};
      }
  }
}

template <int HD>
constexpr size_t flash_lds_bytes() {
  // two key blocks and two value blocks; the fold at the end needs HD / 2 + 2 floats per thread of one group
  const size_t kv = (size_t)2 * (BK * (HD + 8) + HD * (BK + 4)) * sizeof(bf16_t);
  const size_t fold = (size_t)(HD / 2 + 2) * 256 * sizeof(float);
  return kv > fold ? kv : fold;
}

}  // namespace

bool flash_supported(int dtype, int h) { return dtype == MDI_BF16 && (h == 64 || h == 128); }

void launch_v_transpose(hipStream_t s, const float* qkv, int T, int n_cols, int pos0, int ldk, int H, int K, int h, bf16_t* vt) {
  const dim3 grid((n_cols + 63) / 64, K * h / 64);
  hipLaunchKernelGGL(k_v_transpose, grid, dim3(256), 0, s, qkv, T, n_cols, pos0, ldk, (H + 2 * K) * h, (H + K) * h, h, vt);
}

void launch_cache_gather(hipStream_t s, const void* pool, const int32_t* table, int n_pos, int K, int h, int pt, int ldk,
                         bf16_t* k_bf, bf16_t* vt) {
  if (n_pos <= 0) return;
  const dim3 grid((n_pos + 63) / 64, K * h / 64);
  hipLaunchKernelGGL(k_cache_gather, grid, dim3(256), 0, s, (const bf16_t*)pool, table, n_pos, K, h, pt, ldk, k_bf, vt);
}

void launch_flash_prefill(hipStream_t s, const FlashArgs& a) {
  const dim3 grid(a.Tp / BQ, a.H);
  if (a.h == 128) {
    constexpr size_t lds = flash_lds_bytes<128>();               // above the 64 KiB a kernel gets by default
    static std::once_flag raised;
    std::call_once(raised, []() {
      (void)hipFuncSetAttribute((const void*)k_flash_prefill<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    hipLaunchKernelGGL(k_flash_prefill<128>, grid, dim3(512), lds, s, a);
  } else {
    hipLaunchKernelGGL(k_flash_prefill<64>, grid, dim3(512), flash_lds_bytes<64>(), s, a);
  }
}

}  // namespace mdi
