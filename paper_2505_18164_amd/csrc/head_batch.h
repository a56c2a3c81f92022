// Output layers for several samples with ONE pass over the vocabulary matrix (bf16 storage).
//
// Alg. 1 runs the output layers once per returning sample ("process output layers ... get token").  When several
// samples' last hidden states wait at the starter together (Sec. III-C: several samples are in flight), their
// projections share the matrix: a tile of 16 vocabulary rows is fetched once and multiplied with up to 16
// normalised activations on the matrix cores (v_mfma_f32_16x16x32_bf16: first operand = 16 rows x 32 columns of
// the matrix straight from row-major memory, second = 32 columns x 16 samples, read from LDS).
//
//   * Every workgroup normalises all activations itself (final RMSNorm or LayerNorm, rounded to bf16 once) and
//     keeps them in LDS as [group of 8 columns][sample] 16-byte units (the sample index xor-ed with the group's, so
//     that the staging's writes of one sample's groups spread over the banks): a wavefront's read of one column
//     step is one contiguous KiB.
//   * A wavefront owns whole rows: blocks of 16 rows are dealt round-robin over (workgroup, wavefront), so the
//     grid reads one contiguous window of the matrix at any moment, nothing is summed across wavefronts and the
//     stream never stops at a workgroup barrier.  Two register tiles (8 column steps each) are in flight (four were measured slower).
//   * Logits (optional) are written from the accumulators; every lane keeps the best (value, row) of its sample,
//     folded per wavefront, per workgroup, and by the last workgroup to arrive (lowest index on exact ties).
//
// Included by step_w8.hip after step_batch.h.
namespace mdi {
namespace step_w8 {

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

constexpr int kHbGroups = 9;          // 16-byte groups of an activation per lane: widths up to 64 * 9 * 8 = 4608
// Where a wavefront is in its stream: block, how many of the block's column tiles are done, and the tile it started
// the block with.  Rows are a power of two apart in memory; block b starts at tile b mod (tiles per row) and wraps,
// so that at any moment the grid's reads are spread over a whole row's width instead of all wavefronts asking for
// the same columns (a precaution against crowding a few memory channels; on this chip it measured neither faster
// nor slower than starting every block at column 0).
struct HbCursor { int blk, tin, rot; };
__device__ __forceinline__ int hb_tile(const HbCursor& c, int nt) { const int t = c.tin + c.rot; return t >= nt ? t - nt : t; }
__device__ __forceinline__ void hb_next(HbCursor& c, int nt, int stride_blk) {
  if (++c.tin == nt) { c.tin = 0; c.blk += stride_blk; c.rot = c.blk % nt; }
}

__device__ __forceinline__ void hb_issue(Tile& t, const LogitsBatchArgs& a, HbCursor& c, int nt, int nsteps, int stride_blk, int lane) {
  // Loaded in the matrix instruction's own operand order: lane (i = lane mod 16, kg = lane div 16) takes 16 bytes of
  // row i at column group kg.  (Loading with four neighbouring lanes per row - 16 instead of 64 cache lines touched
  // per instruction - and permuting to operand order with ds_bpermute measured -2.5 % on the largest head and +5 %
  // on a narrow one: not kept.)
  const int i = lane & 15, kg = lane >> 4;
  const int row = min(c.blk * 16 + i, a.N - 1);
  const uint32_t off = (uint32_t)row * (uint32_t)(2 * a.Kd) + (uint32_t)(kg << 4);
  const int tile = hb_tile(c, nt);
  const MDI_GLOBAL char* base = (const MDI_GLOBAL char*)a.W + ((long)tile << 9);
  const int last = nsteps - 1 - tile * 8;                  // >= 0: the tile's last valid step
#pragma unroll
  for (int s = 0; s < 8; ++s)
    t.r[s] = *reinterpret_cast<const MDI_GLOBAL u32x4*>(base + ((long)min(s, last) << 6) + off);
  hb_next(c, nt, stride_blk);
}

__global__ __launch_bounds__(kStepThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_logits_batch(LogitsBatchArgs a) {
  extern __shared__ float smem[];
  u32x4* Bs = reinterpret_cast<u32x4*>(smem);               // [Kd / 8][16 samples]
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wg = blockIdx.x, nwg = gridDim.x;
  const int nsteps = a.Kd >> 5, nt = (nsteps + 7) >> 3;
  const int nblk = (a.N + 15) >> 4;
  const int stride_blk = nwg * kStepWaves;
  const int blk0 = wg * kStepWaves + wave;
  const int nb_mine = nblk > blk0 ? (nblk - blk0 + stride_blk - 1) / stride_blk : 0;
  Tile T0, T1;
  HbCursor ci{blk0, 0, blk0 % nt}, cc = ci;

  // ---- final norm of every sample (wavefront w takes samples 2w, 2w + 1), result to LDS as bf16.  Everything a
  // lane needs - its 16-byte groups of both activations and of the gain - is requested at once and kept in
  // registers, so the staging costs one round trip to memory, not one per group.
  const int ngroups = a.Kd >> 3;
  {
    const int n0 = 2 * wave;
    const u32x4* x0 = reinterpret_cast<const u32x4*>(a.x[min(n0, a.m - 1)]);
    const u32x4* x1 = reinterpret_cast<const u32x4*>(a.x[min(n0 + 1, a.m - 1)]);
    const f32x4* gp = reinterpret_cast<const f32x4*>(a.g);
    u32x4 xa[kHbGroups], xb[kHbGroups];
    f32x4 glo[kHbGroups], ghi[kHbGroups];
#pragma unroll
    for (int j = 0; j < kHbGroups; ++j) {
      const int gi = min(lane + 64 * j, ngroups - 1);
      xa[j] = x0[gi]; xb[j] = x1[gi];
      glo[j] = gp[2 * gi]; ghi[j] = gp[2 * gi + 1];
    }
    const f32x4* bp = reinterpret_cast<const f32x4*>(a.b);   // LayerNorm's bias, or nullptr
    float sa = 0.f, sb = 0.f, ma = 0.f, mb = 0.f;
#pragma unroll
    for (int j = 0; j < kHbGroups; ++j) {
      const float live = lane + 64 * j < ngroups ? 1.f : 0.f;
      float ta = 0.f, tb = 0.f, ua = 0.f, ub = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float al = bf16_bits_to_f32(xa[j][e] & 0xFFFFu), ah = bf16_bits_to_f32(xa[j][e] >> 16);
        const float bl = bf16_bits_to_f32(xb[j][e] & 0xFFFFu), bh = bf16_bits_to_f32(xb[j][e] >> 16);
        ta += al * al + ah * ah; tb += bl * bl + bh * bh;
        ua += al + ah; ub += bl + bh;
      }
      sa += live * ta; sb += live * tb; ma += live * ua; mb += live * ub;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      sa += __shfl_xor(sa, off, 64); sb += __shfl_xor(sb, off, 64);
      ma += __shfl_xor(ma, off, 64); mb += __shfl_xor(mb, off, 64);
    }
    // RMSNorm: x / rms * g.  LayerNorm: (x - mean) / std * g + b (biased variance).  Samples beyond the call's count
    // are zero columns.
    const bool ln = a.norm_kind == MDI_NORM_LAYERNORM;
    const float inv_n = 1.0f / (float)a.Kd;
    const float mua = ln ? ma * inv_n : 0.f, mub = ln ? mb * inv_n : 0.f;
    const float ra = n0 < a.m ? 1.0f / sqrtf(fmaxf(sa * inv_n - mua * mua, 0.f) + a.eps) : 0.f;
    const float rb = n0 + 1 < a.m ? 1.0f / sqrtf(fmaxf(sb * inv_n - mub * mub, 0.f) + a.eps) : 0.f;
    const float ka = n0 < a.m ? 1.f : 0.f, kb = n0 + 1 < a.m ? 1.f : 0.f;     // bias only into live columns
#pragma unroll
    for (int j = 0; j < kHbGroups; ++j) {
      const int gi = lane + 64 * j;
      if (gi < ngroups) {
        f32x4 blo = {0.f, 0.f, 0.f, 0.f}, bhi = {0.f, 0.f, 0.f, 0.f};
        if (bp) { blo = bp[2 * gi]; bhi = bp[2 * gi + 1]; }
        u32x4 oa, ob;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float g0 = e < 2 ? glo[j][2 * e] : ghi[j][2 * e - 4], g1 = e < 2 ? glo[j][2 * e + 1] : ghi[j][2 * e - 3];
          const float b0 = e < 2 ? blo[2 * e] : bhi[2 * e - 4], b1 = e < 2 ? blo[2 * e + 1] : bhi[2 * e - 3];
          oa[e] = pack_bf16x2((bf16_bits_to_f32(xa[j][e] & 0xFFFFu) - mua) * ra * g0 + ka * b0, (bf16_bits_to_f32(xa[j][e] >> 16) - mua) * ra * g1 + ka * b1);
          ob[e] = pack_bf16x2((bf16_bits_to_f32(xb[j][e] & 0xFFFFu) - mub) * rb * g0 + kb * b0, (bf16_bits_to_f32(xb[j][e] >> 16) - mub) * rb * g1 + kb * b1);
        }
        Bs[gi * 16 + (n0 ^ (gi & 15))] = oa; Bs[gi * 16 + ((n0 + 1) ^ (gi & 15))] = ob;
      }
    }
  }
  hb_issue(T0, a, ci, nt, nsteps, stride_blk, lane);         // (requested here, not earlier: the staging needs the registers)
  hb_issue(T1, a, ci, nt, nsteps, stride_blk, lane);
  __syncthreads();

  // ---- the stream: 16 rows x all columns per block, accumulators = 4 rows x 1 sample per lane
  const int n = lane & 15, kg = lane >> 4;
  float bv = -INFINITY; int bi = 0x7FFFFFFF;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  auto compute = [&](const Tile& t) {
    if (cc.blk < nblk) {                                     // uniform
      const int tile = hb_tile(cc, nt);
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const int ks = tile * 8 + s;
        if (ks < nsteps) {                                   // uniform
          const u32x4 b = Bs[(ks * 4 + kg) * 16 + (n ^ ((ks * 4 + kg) & 15))];
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t.r[s]), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
        }
      }
      if (cc.tin == nt - 1) {
        const int r0 = cc.blk * 16 + 4 * kg;
        if (n < a.m) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (r0 + r < a.N) {
              if (a.out) a.out[(long)n * a.out_stride + r0 + r] = acc[r];
              if (better_logit(acc[r], r0 + r, bv, bi)) { bv = acc[r]; bi = r0 + r; }
            }
          }
        }
        acc = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
    hb_next(cc, nt, stride_blk);
  };
  const int total = (nb_mine * nt + 1) & ~1;
#pragma nounroll
  for (int t = 0; t < total; t += 2) {
    compute(T0);
    hb_issue(T0, a, ci, nt, nsteps, stride_blk, lane);
    compute(T1);
    hb_issue(T1, a, ci, nt, nsteps, stride_blk, lane);
  }

  // ---- argmax per sample: lanes with the same sample, then wavefronts, then workgroups
  __shared__ float sv[kStepWaves][kMaxBatch];
  __shared__ int si[kStepWaves][kMaxBatch];
  __shared__ int s_last;
#pragma unroll
  for (int off = 32; off >= 16; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64); const int oi = __shfl_xor(bi, off, 64);
    if (better_logit(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if (lane < 16) { sv[wave][lane] = bv; si[wave][lane] = bi; }
  __syncthreads();
  // Candidates cross workgroups as 8-byte words that carry the call's counter (value | tag, index | tag), stored and
  // loaded at agent scope: the last workgroup to arrive reloads a word until its tag is this call's, so no fence
  // (on this chip: a write-back of a die's L2, several microseconds per wavefront that executes one) is needed.
  if (threadIdx.x < kMaxBatch) {
    bv = sv[0][threadIdx.x]; bi = si[0][threadIdx.x];
    for (int k = 1; k < kStepWaves; ++k) if (better_logit(sv[k][threadIdx.x], si[k][threadIdx.x], bv, bi)) { bv = sv[k][threadIdx.x]; bi = si[k][threadIdx.x]; }
    tagged_t* c = a.cand + ((long)threadIdx.x * nwg + wg) * 2;
    st_pair(c, __float_as_uint(bv), a.tag);
    st_pair(c + 1, (uint32_t)bi, a.tag);
  }
  if (threadIdx.x == 0) {                                    // after this wavefront's stores in program order
    const unsigned ticket = __hip_atomic_fetch_add(a.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = ticket == (unsigned)nwg - 1;
  }
  __syncthreads();
  if (s_last) {
    for (int q = 0; q < 2; ++q) {
      const int sm = 2 * wave + q;
      if (sm >= a.m) continue;                               // uniform
      bv = -INFINITY; bi = 0x7FFFFFFF;
      for (int k = lane; k < nwg; k += 64) {
        const tagged_t* c = a.cand + ((long)sm * nwg + k) * 2;
        const float v = __uint_as_float(settle_bits(c, ld_raw(c), a.tag, a.spin_limit, a.err));
        const int i = (int)settle_bits(c + 1, ld_raw(c + 1), a.tag, a.spin_limit, a.err);
        if (better_logit(v, i, bv, bi)) { bv = v; bi = i; }
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off, 64); const int oi = __shfl_xor(bi, off, 64);
        if (better_logit(ov, oi, bv, bi)) { bv = ov; bi = oi; }
      }
      if (lane == 0) a.token_out[sm] = bi;
    }
    if (threadIdx.x == 0) __hip_atomic_store(a.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

}  // namespace step_w8

bool logits_batch_allow_lds(size_t lds) {
  return hipFuncSetAttribute((const void*)step_w8::k_logits_batch, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
}
void launch_logits_batch(hipStream_t s, int nwg, size_t lds, const LogitsBatchArgs& a) {
  hipLaunchKernelGGL(step_w8::k_logits_batch, dim3(nwg), dim3(step_w8::kStepThreads), lds, s, a);
}

}  // namespace mdi
