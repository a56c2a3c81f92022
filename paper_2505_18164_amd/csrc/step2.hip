// One decode step of a whole partition as ONE persistent launch with specialised wavefronts.
//
// A later visit of a sample (Sec. III-D) pushes one position through every local layer; each layer
// is five dependent phases (QKV + RoPE + KV append, attention over the sample's cache, output
// projection, MLP up, MLP down) whose inputs are full vectors produced by the previous phase on
// other compute units.  The bytes a step must move (every matrix once, the sample's keys and values
// once) have addresses that do not depend on any activation, so the memory stream never has to
// stop at a phase boundary -- provided the wavefronts that stream never wait for the exchange of
// the small vectors.  Vector-memory results return to a wavefront in issue order, so a wavefront
// that polls another workgroup's flag sits behind everything it prefetched.  Hence two roles:
//
//   * S streaming wavefronts own a ring of NT register tiles (eight 16-byte loads per lane each)
//     that runs NT tiles ahead of the arithmetic, straight across phase and layer boundaries.
//     They touch global memory through those loads only; everything else they need (the phase's
//     input vector, the sample's page ids) is in LDS.
//   * E exchange wavefronts do what crosses workgroups: they wait for the producers of the next
//     phase's input, copy it into LDS (normalising it when the phase starts with a norm), and
//     after the streaming wavefronts have left their partial sums in LDS, add them up, apply the
//     phase's epilogue and publish the results.
//
// Exchange protocol (no cache write-back or invalidate anywhere): every published value is an
// 8-byte (float bits, phase counter) word written and read with agent-scope (cache-coherent)
// accesses.  A reader that finds another counter loads again, so data validates itself; the
// per-workgroup flags are only a cheap thing to poll.  A buffer is overwritten at the earliest two
// phases after it was read, and a workgroup can only get that far after consuming the outputs of
// every reader, so no flag is needed to protect readers either.
//
// Roles meet at workgroup barriers; per phase both execute the same three: B (raw input vector in
// LDS), C (input vector final), A (partial sums of the phase in LDS).  Every wait on another
// workgroup is bounded: when it expires the workgroup raises the partition's error word, and all
// its wavefronts leave after the next barrier.
#include <type_traits>
#include <utility>

#include "device_utils.h"

namespace mdi {
namespace {

#define MDI_GLOBAL __attribute__((address_space(1)))

// LDS is addressed through pointers that carry their address space, so every access is a ds_
// instruction (a generic pointer could turn into a flat access, which also counts as vector memory)
typedef __attribute__((address_space(3))) float lds_float;
typedef __attribute__((address_space(3))) int lds_int;
typedef __attribute__((address_space(3))) uint16_t lds_u16;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) f32x4 lds_float4;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kLoads = 8;                       // 16-byte loads per lane in a tile (1 KiB per wavefront each)
constexpr int kItems = 4;                       // attention: items per tile, one K and one V load each
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// The ring lives in accumulation registers named in the asm text itself (tile slot i = a[32 i, 32 i + 32)),
// and is requested, waited for and read by hand-written instructions only.  The compiler's own accounting
// of outstanding loads gives up on this control flow (a tile is consumed several phases of branches after
// it was requested) and would wait for everything at every tile; and a register allocator that may split
// or copy a live range cannot be allowed near registers with a load in flight (the data would land in a
// register that holds something else by then).  Every asm statement below names all ring registers as
// clobbered, so the compiler keeps nothing of its own there.
#define MDI_RING_REGS "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63", "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95", "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127"
constexpr int kRingMax = 4;                       // tile slots the clobber list covers (with 8 wavefronts of 256 registers, 128 are accumulation registers)

// request: 16 bytes per lane into a[R, R + 4); address = uniform base + per-lane byte offset (below 4 GiB)
template <int R>
__device__ __forceinline__ void ring_load(const void* base, uint32_t off) {
  asm volatile("global_load_dwordx4 a[%2:%3], %0, %1" : : "v"(off), "s"(base), "n"(R), "n"(R + 3) : MDI_RING_REGS);
}
// Waits until at most (NT - 1 - j) tiles requested after the oldest one are outstanding, j being how many
// refills were held back since (0 in the steady state); the branches on the uniform j are inside the asm.
template <int NT>
__device__ __forceinline__ void ring_wait(int j) {
  static_assert(kLoads == 8 && NT >= 2 && NT <= kRingMax, "wait ladder below");
  constexpr int n1 = kLoads * (NT - 1), n2 = kLoads * (NT > 2 ? NT - 2 : 0), n3 = kLoads * (NT > 3 ? NT - 3 : 0),
                n4 = kLoads * (NT > 4 ? NT - 4 : 0), n5 = kLoads * (NT > 5 ? NT - 5 : 0);
  asm volatile(
      "s_waitcnt vmcnt(%1)\n\t"
      "s_cmp_lt_i32 %0, 1\n\t"
      "s_cbranch_scc1 .Lring_done%=\n\t"
      "s_waitcnt vmcnt(%2)\n\t"
      "s_cmp_lt_i32 %0, 2\n\t"
      "s_cbranch_scc1 .Lring_done%=\n\t"
      "s_waitcnt vmcnt(%3)\n\t"
      "s_cmp_lt_i32 %0, 3\n\t"
      "s_cbranch_scc1 .Lring_done%=\n\t"
      "s_waitcnt vmcnt(%4)\n\t"
      "s_cmp_lt_i32 %0, 4\n\t"
      "s_cbranch_scc1 .Lring_done%=\n\t"
      "s_waitcnt vmcnt(%5)\n\t"
      "s_cmp_lt_i32 %0, 5\n\t"
      "s_cbranch_scc1 .Lring_done%=\n\t"
      "s_waitcnt vmcnt(0)\n"
      ".Lring_done%=:"
      : : "s"(j), "n"(n1), "n"(n2), "n"(n3), "n"(n4), "n"(n5) : "scc", MDI_RING_REGS);
}
// acc += W tile (a[R, R + 4): 16 rows x 4 V columns) x the vector's piece xv, on the matrix core.  The leading
// wait state covers a vector-ALU write of an operand just before (the compiler does not look inside).
template <typename WT, int R> struct RingMfma;
template <int R> struct RingMfma<bf16_t, R> {
  __device__ static __forceinline__ void go(f32x4& acc, const f32x4& xv) {
    asm volatile("s_nop 1\n\tv_mfma_f32_16x16x32_bf16 %0, a[%2:%3], %1, %0" : "+v"(acc) : "v"(xv), "n"(R), "n"(R + 3) : MDI_RING_REGS);
  }
};
template <int R> struct RingMfma<float, R> {
  __device__ static __forceinline__ void go(f32x4& acc, const f32x4& xv) {
    asm volatile("s_nop 1\n\t"
                 "v_mfma_f32_16x16x4_f32 %0, a[%5], %1, %0\n\t"
                 "v_mfma_f32_16x16x4_f32 %0, a[%6], %2, %0\n\t"
                 "v_mfma_f32_16x16x4_f32 %0, a[%7], %3, %0\n\t"
                 "v_mfma_f32_16x16x4_f32 %0, a[%8], %4, %0"
                 : "+v"(acc) : "v"(xv.x), "v"(xv.y), "v"(xv.z), "v"(xv.w), "n"(R), "n"(R + 1), "n"(R + 2), "n"(R + 3) : MDI_RING_REGS);
  }
};
// the accumulator is about to be read by something else than the matrix core: let its last instruction retire
__device__ __forceinline__ void mfma_drain(f32x4& acc) {
  asm volatile("s_nop 15\n\ts_nop 7" : "+v"(acc) : : MDI_RING_REGS);
}
// a[R, R + 4) -> ordinary registers (for the vector ALUs)
template <int R>
__device__ __forceinline__ u32x4 ring_read() {
  u32x4 v;
  asm volatile("v_accvgpr_read_b32 %0, a[%4]\n\tv_accvgpr_read_b32 %1, a[%5]\n\tv_accvgpr_read_b32 %2, a[%6]\n\tv_accvgpr_read_b32 %3, a[%7]"
               : "=v"(v.x), "=v"(v.y), "=v"(v.z), "=v"(v.w) : "n"(R), "n"(R + 1), "n"(R + 2), "n"(R + 3) : MDI_RING_REGS);
  return v;
}

enum Phase { PH_QKV = 0, PH_ATTN = 1, PH_OPROJ = 2, PH_UP = 3, PH_DOWN = 4 };

// LDS header (ints)
enum { L_ABORT = 0, L_NEXT = 1, L_GO = 6, L_NT = 8, L_ATT = 16, L_GEO = 32, L_GEO_INTS = 12, L_TRACE = 96, L_TRACE_INTS = 3 * 5 * 16 };   // L_NEXT: 5 ints
// attention geometry slots
enum { A_ACTIVE = 0, A_HG, A_SPLIT, A_KVH, A_S0, A_S1, A_S1P, A_STEPS };

__device__ __forceinline__ int rfl(int v) { return __builtin_amdgcn_readfirstlane(v); }

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): loops whose index must be a constant expression
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits for every
// outstanding global load of the wavefront, which would drain the prefetch ring at each phase.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ void st_tag(tagged_t* p, float v, unsigned tag) {
  __hip_atomic_store(p, ((tagged_t)tag << 32) | (tagged_t)__float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ tagged_t ld_raw(const tagged_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }


struct Watch { int* err; lds_int* abort_flag; int spin_limit; };
__device__ __forceinline__ void give_up(const Watch& w) {
  __hip_atomic_store(w.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  *w.abort_flag = 1;
}
// Returns the value once its counter is `tag`; gives up after spin_limit reloads.
__device__ __forceinline__ float settle(const tagged_t* p, tagged_t u, unsigned tag, const Watch& w) {
  int it = 0;
  while ((uint32_t)(u >> 32) != tag) {
    if (++it > w.spin_limit) { give_up(w); break; }
    __builtin_amdgcn_s_sleep(1);
    u = ld_raw(p);
  }
  return __uint_as_float((uint32_t)u);
}
__device__ __forceinline__ float ld_tag(const tagged_t* p, unsigned tag, const Watch& w) { return settle(p, ld_raw(p), tag, w); }

// element i of the phase's input vector, kept in LDS in the matrices' type
template <typename WT> __device__ __forceinline__ void xs_put(lds_float* xs, int i, float v);
template <> __device__ __forceinline__ void xs_put<float>(lds_float* xs, int i, float v) { xs[i] = v; }
template <> __device__ __forceinline__ void xs_put<bf16_t>(lds_float* xs, int i, float v) { reinterpret_cast<lds_u16*>(xs)[i] = f32_to_bf16(v); }

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

// ---------------------------------------------------------------------------
// GEMV phases.  The matrices are stored as tiles of 16 rows x 1 KiB, in the order the matrix cores
// take their A operand: lane l of a wavefront holds row l % 16, elements [V * (l / 16), V * (l / 16) + V)
// of the tile's KT = 4 V columns (V = 8 bf16 or 4 fp32 per 16-byte load).  One load instruction
// therefore fetches one contiguous KiB and feeds the matrix core without unpacking; the B operand is
// the phase's input vector, the same in all 16 columns, so column 0 of the accumulator is the dot
// product of 16 rows, reduced over the lanes by the instruction itself.  Rows are stored in pair
// order (RoPE partners i / i + h/2 of a head next to each other, gate_f / up_f next to each other),
// so a 16-row block is 8 whole pairs.  Blocks are dealt round-robin to workgroups; a workgroup's
// (block, tile) items are dealt round-robin to its S streaming wavefronts, so at any moment it reads
// S consecutive KiB and the wavefronts are balanced; a wavefront's share of a block goes to an LDS
// slot of its own and the exchange wavefronts add the slots in wavefront order.
struct Geo {
  int N, n_kt, nb, rope_h, dq, dr;
  int n_k;               // this wavefront's items: item k is flat index wave + S * k, flat = block * n_kt + tile
};
// GEMV geometry slots in LDS
enum { G_N = 0, G_NKT, G_NB, G_ROPE_H, G_DQ, G_DR, G_TILES };

template <typename WT> __device__ __forceinline__ int k_tiles(int Kd) { return (Kd + 4 * Storage<WT>::kVec - 1) / (4 * Storage<WT>::kVec); }

template <typename WT, int S>
__device__ __forceinline__ void store_geo(lds_int* o, int N, int Kd, int rope_h, int wg, int nwg) {
  const int n_kt = k_tiles<WT>(Kd);
  const int nblk = (N + 15) >> 4;
  const int nb = nblk > wg ? (nblk - wg + nwg - 1) / nwg : 0;
  const int nk0 = (nb * n_kt + S - 1) / S;                                      // wavefront 0 has the most items
  o[G_N] = N; o[G_NKT] = n_kt; o[G_NB] = nb; o[G_ROPE_H] = rope_h;
  o[G_DQ] = S / n_kt; o[G_DR] = S % n_kt; o[G_TILES] = (nk0 + kLoads - 1) / kLoads;
}
template <int S>
__device__ __forceinline__ Geo load_geo(const lds_int* o, int wave) {
  Geo g;
  g.N = rfl(o[G_N]); g.n_kt = rfl(o[G_NKT]); g.nb = rfl(o[G_NB]); g.rope_h = rfl(o[G_ROPE_H]);
  g.dq = rfl(o[G_DQ]); g.dr = rfl(o[G_DR]);
  const int flat = g.nb * g.n_kt;
  g.n_k = flat > wave ? (flat - wave + S - 1) / S : 0;
  return g;
}
__device__ __forceinline__ void geo_next(const Geo& g, int& bl, int& kt) {
  kt += g.dr; bl += g.dq;
  if (kt >= g.n_kt) { kt -= g.n_kt; ++bl; }
}
// row of the source matrix stored at position j of pair p
__device__ __forceinline__ int geo_row(int rope_h, int p, int j) {
  if (rope_h) {                                     // head sizes are powers of two
    const int half = rope_h >> 1, sh = 31 - __builtin_clz(half);
    const int head = p >> sh, i = p & (half - 1);
    return head * rope_h + i + j * half;
  }
  return 2 * p + j;
}
__device__ __forceinline__ int gemv_index(int ph) { return ph == PH_QKV ? 0 : ph - 1; }   // QKV, oproj, up, down

template <typename T> __device__ __forceinline__ T* advance(T* p, long bytes) { return p ? (T*)((char*)p + bytes) : p; }
__device__ __forceinline__ const void* advance(const void* p, long bytes) { return p ? (const void*)((const char*)p + bytes) : p; }
// Every layer occupies an identically laid out block of the arena: layer i's pointers are the first
// layer's advanced by i strides, so no pointer is fetched from memory.
__device__ __forceinline__ StepLayer layer_at(const Step2Args& a, int layer) {
  const long w = a.w_stride * layer, kv = a.kv_stride * layer;
  StepLayer L;
  L.wqkv = advance(a.l0.wqkv, w); L.wo = advance(a.l0.wo, w); L.wup = advance(a.l0.wup, w); L.wdown = advance(a.l0.wdown, w);
  L.bqkv = advance(a.l0.bqkv, w); L.bo = advance(a.l0.bo, w); L.bup = advance(a.l0.bup, w); L.bdown = advance(a.l0.bdown, w);
  L.ln1_g = advance(a.l0.ln1_g, w); L.ln1_b = advance(a.l0.ln1_b, w); L.ln2_g = advance(a.l0.ln2_g, w); L.ln2_b = advance(a.l0.ln2_b, w);
  L.kv = advance(a.l0.kv, kv);
  return L;
}
__device__ __forceinline__ const void* phase_base(const Step2Args& a, int layer, int ph) {
  const long w = a.w_stride * layer;
  switch (ph) {
    case PH_QKV: return advance(a.l0.wqkv, w);
    case PH_ATTN: return advance((const void*)a.l0.kv, a.kv_stride * layer);
    case PH_OPROJ: return advance(a.l0.wo, w);
    case PH_UP: return advance(a.l0.wup, w);
    default: return advance(a.l0.wdown, w);
  }
}

// optional timeline: one thread per workgroup records 100 MHz timestamps per (layer, phase)
__device__ __forceinline__ void stamp(const Step2Args& a, bool who, int layer, int ph, int k) {
  if (a.trace && who) a.trace[(((long)blockIdx.x * a.n_layer + layer) * 5 + ph) * 8 + k] = wall_clock64();
}

template <typename WT, int G>
struct AttnState { float m[G], l[G], o[G][Storage<WT>::kVec]; };

// ---------------------------------------------------------------------------
template <typename WT, int G, int S, int E, int NT, int D>
__global__ __launch_bounds__((S + E) * 64) void k_step2(Step2Args a) {
  constexpr int V = Storage<WT>::kVec;
  constexpr int NTHREADS = (S + E) * 64;
  extern __shared__ float smem[];
  lds_float* sm = (lds_float*)smem;
  lds_int* si = (lds_int*)smem;
  const int lane = threadIdx.x & 63;
  const int wave = rfl(threadIdx.x >> 6);
  const int wg = blockIdx.x, nwg = gridDim.x;
  lds_int* tab = si + a.lds_tab;           // page ids of the sample
  lds_float* own = sm + a.lds_own;       // residual-stream rows this workgroup owns
  lds_float* part = sm + a.lds_part;     // [block][S][16] partial dot products
  lds_float* xs = sm + a.lds_xs;         // the phase's input vector in the matrices' type (attention: fp32 scaled queries, newest k, newest v)
  lds_float* xraw = sm + a.lds_xraw;     // residual stream before the norm
  lds_float* gain = sm + a.lds_gain;     // norm gain of the coming phase, then its bias (LayerNorm)
  lds_float* gbias = gain + a.d;
  lds_float* rec = sm + a.lds_rec;       // attention: [S + 1][G][h + 2] online-softmax records (the last: newest position)
  const int h = a.h, recsz = h + 2;

  // ---- set-up: geometry of every phase, the sample's page ids, cleared partial sums -------------
  if (threadIdx.x == 0) {
    const int nup = a.mlp_kind == MDI_MLP_SWIGLU ? 2 * a.F : a.F;
    store_geo<WT, S>(si + L_GEO + 0 * L_GEO_INTS, (a.H + 2 * a.K) * h, a.d, h, wg, nwg);   // pairs (i, i + h/2)
    store_geo<WT, S>(si + L_GEO + 1 * L_GEO_INTS, a.d, a.H * h, 0, wg, nwg);
    store_geo<WT, S>(si + L_GEO + 2 * L_GEO_INTS, nup, a.d, 0, wg, nwg);
    store_geo<WT, S>(si + L_GEO + 3 * L_GEO_INTS, a.d, a.F, 0, wg, nwg);
    // attention: workgroup = (head group, context split)
    const int active = wg < a.n_hg * a.n_splits;
    const int hg = active ? wg % a.n_hg : 0, split = active ? wg / a.n_hg : 0;
    const int s0 = split * a.chunk, s1 = min(a.ctx, s0 + a.chunk), s1p = min(s1, a.ctx - 1);   // the newest row is not in the cache yet
    const int tpw = 64 / (h / V);
    const int steps = active && s1p > s0 ? (s1p - s0 + tpw - 1) / tpw : 0;
    const int nk0 = (steps + S - 1) / S;
    lds_int* at = si + L_ATT;
    at[A_ACTIVE] = active; at[A_HG] = hg; at[A_SPLIT] = split; at[A_KVH] = (hg * G) / (a.H / a.K);
    at[A_S0] = s0; at[A_S1] = s1; at[A_S1P] = s1p; at[A_STEPS] = steps;
    si[L_NT + PH_QKV] = si[L_GEO + 0 * L_GEO_INTS + G_TILES];
    si[L_NT + PH_ATTN] = active ? max(1, (nk0 + kItems - 1) / kItems) : 0;
    si[L_NT + PH_OPROJ] = si[L_GEO + 1 * L_GEO_INTS + G_TILES];
    si[L_NT + PH_UP] = si[L_GEO + 2 * L_GEO_INTS + G_TILES];
    si[L_NT + PH_DOWN] = si[L_GEO + 3 * L_GEO_INTS + G_TILES];
    si[L_ABORT] = 0;
    si[L_GO] = (int)a.epoch0 - 1;
    // phase that follows each phase in this workgroup's stream (bit 4: in the next layer)
    if (si[L_NT] + si[L_NT + 1] + si[L_NT + 2] + si[L_NT + 3] + si[L_NT + 4] > 0)
      for (int ph = 0; ph < 5; ++ph) {
        int q = ph, wrap = 0;
        do { if (++q == 5) { q = 0; wrap = 16; } } while (si[L_NT + q] == 0);
        si[L_NEXT + ph] = q | wrap;
      }
    if (wg == 0 && a.table_entry) *a.table_entry = a.new_page;     // for later launches; this one never reads the new page
  }
  for (int i = threadIdx.x; i < a.n_tab; i += NTHREADS)
    tab[i] = __hip_atomic_load(a.table + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int i = threadIdx.x; i < a.part_floats; i += NTHREADS) part[i] = 0.f;
  __syncthreads();

  const lds_int* ntp = si + L_NT;
  const int tiles_layer = rfl(ntp[0] + ntp[1] + ntp[2] + ntp[3] + ntp[4]);
  const int att_hg = rfl(si[L_ATT + A_HG]), att_split = rfl(si[L_ATT + A_SPLIT]), att_kvh = rfl(si[L_ATT + A_KVH]);
  const int att_s0 = rfl(si[L_ATT + A_S0]), att_s1 = rfl(si[L_ATT + A_S1]), att_s1p = rfl(si[L_ATT + A_S1P]);
  const int att_steps = rfl(si[L_ATT + A_STEPS]);

  if (wave < S) {
    // =======================================================================================
    // streaming role
    // =======================================================================================
    if (tiles_layer == 0) return;
    const int Lh = h / V, tpw = 64 / Lh, sub = lane / Lh, hoff = (lane % Lh) * V;
    const int att_nk = att_steps > wave ? (att_steps - wave + S - 1) / S : 0;

    auto first_phase = [&](int& ph) __attribute__((always_inline)) { while (rfl(ntp[ph]) == 0) ++ph; };     // tiles_layer > 0: terminates
    // (layer, phase, tile) -> next tile of this workgroup's stream; true when a new phase starts
    auto next_tile = [&](int& layer, int& ph, int& t) __attribute__((always_inline)) -> bool {
      if (++t < rfl(ntp[ph])) return false;
      t = 0;
      const int nx = rfl(si[L_NEXT + ph]);
      ph = nx & 15; layer += nx >> 4;
      return true;
    };

    // consumer and producer cursors; the producer runs NT tiles ahead
    int c_layer = 0, c_ph = 0, c_t = 0, c_pl = 0, c_c = 0;
    int p_layer = 0, p_ph = 0, p_t = 0, p_pl = 0, p_c = 0;
    first_phase(c_ph); p_ph = c_ph;
    Geo gc, gp;
    const void* p_base = nullptr;
    auto enter_producer = [&]() __attribute__((always_inline)) {
      if (p_layer >= a.n_layer) return;
      p_base = phase_base(a, p_layer, p_ph);
      if (p_ph != PH_ATTN) { gp = load_geo<S>(si + L_GEO + gemv_index(p_ph) * L_GEO_INTS, wave); p_pl = wave / gp.n_kt; p_c = wave - p_pl * gp.n_kt; }
    };
    gp = load_geo<S>(si + L_GEO, wave); gc = gp;
    enter_producer();

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    AttnState<WT, G> st;

    // A tile's requests: one uniform base and a byte offset per load and lane.  Every tile is requested
    // with exactly kLoads loads, whatever the cursor: items past the end of the wavefront's share, and
    // tiles past the end of the step, read the first bytes of the arena instead.
    struct Req { const void* base; uint32_t off[kLoads]; };
    auto plan_tile = [&](Req& rq) __attribute__((always_inline)) {
      rq.base = a.l0.wqkv;
#pragma unroll
      for (int s = 0; s < kLoads; ++s) rq.off[s] = 0u;
      if (p_layer < a.n_layer) {
        rq.base = p_base;
        if (p_ph == PH_ATTN) {
          bool any = false;
#pragma unroll
          for (int s = 0; s < kItems; ++s) {
            const int k = p_t * kItems + s;
            const int tok = att_s0 + (k * S + wave) * tpw + sub;
            if (k < att_nk && tok < att_s1p) {
              const int pi = tok / a.pt;
              const int page = tab[pi];
              const uint32_t o = (uint32_t)((((long)page * a.K + att_kvh) * 2 * a.pt_h + (long)(tok - pi * a.pt) * h + hoff) * (long)sizeof(WT));
              rq.off[2 * s] = o;
              rq.off[2 * s + 1] = o + (uint32_t)(a.pt_h * (long)sizeof(WT));
              any = true;
            }
          }
          (void)any;
        } else {
#pragma unroll
          for (int s = 0; s < kLoads; ++s) {
            if (p_t * kLoads + s < gp.n_k) {                            // uniform
              rq.off[s] = (uint32_t)(((wg + p_pl * nwg) * gp.n_kt + p_c) * 1024 + lane * 16);   // block p_pl of this workgroup, tile p_c
              geo_next(gp, p_pl, p_c);
            }
          }
        }
        if (next_tile(p_layer, p_ph, p_t)) enter_producer();
      }
    };
    auto issue_tile = [&](auto slot) __attribute__((always_inline)) {
      constexpr int R0 = decltype(slot)::value * 4 * kLoads;
      Req rq;
      plan_tile(rq);
      static_for<kLoads>([&](auto ic) __attribute__((always_inline)) { constexpr int i = decltype(ic)::value; ring_load<R0 + 4 * i>(rq.base, rq.off[i]); });
    };

    // Arithmetic of one tile of a GEMV phase; with refill, each of the tile's registers is requested
    // again (next use of the slot) right after the matrix core has read it.  The input vector's pieces
    // come from LDS four items ahead, and nothing touches the accumulator between two matrix
    // instructions except where a block ends.
    auto consume_gemv = [&](auto slot, bool refill) __attribute__((always_inline)) {
      constexpr int R0 = decltype(slot)::value * 4 * kLoads;
      Req rq;
      if (refill) plan_tile(rq);
      // this tile's items: columns tile, validity, end of the wavefront's share of a block (all uniform)
      int kts[kLoads], bls[kLoads];
      unsigned validm = 0u, flushm = 0u;
#pragma unroll
      for (int s = 0; s < kLoads; ++s) {
        const int k = c_t * kLoads + s;
        kts[s] = c_c; bls[s] = c_pl;
        if (k < gc.n_k) {
          validm |= 1u << s;
          int nbl = c_pl, nkt = c_c;
          geo_next(gc, nbl, nkt);
          if (nbl != c_pl || k == gc.n_k - 1) flushm |= 1u << s;
          c_pl = nbl; c_c = nkt;
        }
      }
      const lds_float* xl = xs + (lane >> 4) * 4;     // lane l takes elements [V * (l / 16), + V) of a tile's columns: 16 bytes
      constexpr int XL = 4;                            // items the LDS reads run ahead of the matrix instructions
      f32x4 xv[XL];
#pragma unroll
      for (int s = 0; s < XL; ++s) xv[s] = *reinterpret_cast<const lds_float4*>(xl + kts[s] * 16);
      static_for<kLoads>([&](auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        if (validm & (1u << i)) RingMfma<WT, R0 + 4 * i>::go(acc, xv[i % XL]);
        if (i + XL < kLoads) xv[i % XL] = *reinterpret_cast<const lds_float4*>(xl + kts[(i + XL) % kLoads] * 16);
        if (refill) ring_load<R0 + 4 * i>(rq.base, rq.off[i]);
        if (flushm & (1u << i)) {                                   // this wavefront's share of the block is complete
          mfma_drain(acc);
          // accumulator register r of lane l is row 4 * (l / 16) + r, column l % 16; all columns are equal
          if ((lane & 15) == 0) *reinterpret_cast<lds_float4*>(part + (bls[i] * S + wave) * 16 + (lane >> 4) * 4) = acc;
          acc = f32x4{0.f, 0.f, 0.f, 0.f};
        }
      });
    };

    auto consume_attn = [&](auto slot) __attribute__((always_inline)) {
      constexpr int R0 = decltype(slot)::value * 4 * kLoads;
      static_for<kItems>([&](auto ic) __attribute__((always_inline)) {
        constexpr int s = decltype(ic)::value;
        const int k = c_t * kItems + s;
        if (k < att_nk) {                                           // uniform
          const int tok = att_s0 + (k * S + wave) * tpw + sub;
          const bool valid = tok < att_s1p;
          float kf[V], vf[V];
          Unpack<WT>::go(ring_read<R0 + 8 * s>(), kf);
          Unpack<WT>::go(ring_read<R0 + 8 * s + 4>(), vf);
#pragma unroll
          for (int gi = 0; gi < G; ++gi) {
            float sc = 0.f;
#pragma unroll
            for (int e = 0; e < V; e += 4) {
              const f32x4 q4 = *reinterpret_cast<const lds_float4*>(xs + gi * h + hoff + e);
              sc = fmaf(q4.x, kf[e], sc); sc = fmaf(q4.y, kf[e + 1], sc); sc = fmaf(q4.z, kf[e + 2], sc); sc = fmaf(q4.w, kf[e + 3], sc);
            }
            sc = group_sum(sc, Lh);
            if (valid) {
              const float mn = fmaxf(st.m[gi], sc);
              const float alpha = __expf(st.m[gi] - mn), p = __expf(sc - mn);
              st.m[gi] = mn;
              st.l[gi] = st.l[gi] * alpha + p;
#pragma unroll
              for (int e = 0; e < V; ++e) st.o[gi][e] = st.o[gi][e] * alpha + p * vf[e];
            }
          }
        }
      });
    };

    // folds the wavefront's token sub-groups and leaves one record per head in LDS
    auto attn_records = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        if (off < Lh) continue;
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
      if (sub == 0) {
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
          lds_float* r = rec + (wave * G + gi) * recsz;
#pragma unroll
          for (int e = 0; e < V; ++e) r[hoff + e] = st.o[gi][e];
          if (hoff == 0) { r[h] = st.m[gi]; r[h + 1] = st.l[gi]; }
        }
      }
    };

    // One tile of the stream: arithmetic on the oldest tile of the ring, then its slot is refilled.
    //
    // Refilling right away keeps the ring NT tiles ahead, but then the requests for the next phase have
    // all gone out (paced by the arithmetic) before this phase ends, and the memory system idles while
    // the workgroups exchange vectors.  So the refills of a phase's last D tiles are held back and go
    // out in one burst after its last tile: they are in flight exactly while the exchange happens.
    // While refills are held back fewer tiles are outstanding, which the wait for a tile accounts for.
    auto body = [&](auto slot) __attribute__((always_inline)) -> bool {
      constexpr int SL = decltype(slot)::value;
      if (c_layer >= a.n_layer) return false;
      if (c_t == 0) {                       // a phase begins: its input vector is in LDS after barriers B and C
        lds_barrier();
        lds_barrier();
        if (si[L_ABORT]) return false;
        if (c_ph == PH_ATTN) {
#pragma unroll
          for (int gi = 0; gi < G; ++gi) {
            st.m[gi] = -1e30f; st.l[gi] = 0.f;
#pragma unroll
            for (int e = 0; e < V; ++e) st.o[gi][e] = 0.f;
          }
        } else {
          gc = load_geo<S>(si + L_GEO + gemv_index(c_ph) * L_GEO_INTS, wave);
          c_pl = wave / gc.n_kt; c_c = wave - c_pl * gc.n_kt;
          acc = f32x4{0.f, 0.f, 0.f, 0.f};
        }
      }
      const int nt = rfl(ntp[c_ph]), held = min(D, nt);
      const bool tr = a.trace && wave == 0 && c_layer < 3;      // timeline of streaming wavefront 0, kept in LDS (no global stores here)
      lds_int* trp = si + L_TRACE + (c_layer * 5 + c_ph) * 16;
      if (tr && c_t < 4) trp[4 * c_t] = (int)wall_clock64();
      // the oldest tile has landed once only the younger ones are outstanding: NT - 1 tiles, less the refills held back so far
      ring_wait<NT>(max(0, c_t - (nt - held)));
      if (tr && c_t < 4) trp[4 * c_t + 1] = (int)wall_clock64();
      const bool refill = c_t < nt - held;
      if (c_ph == PH_ATTN) {
        consume_attn(slot);
        if (tr && c_t < 4) trp[4 * c_t + 2] = (int)wall_clock64();
        if (refill) issue_tile(slot);
      } else {
        consume_gemv(slot, refill);
        if (tr && c_t < 4) trp[4 * c_t + 2] = (int)wall_clock64();
      }
      if (tr && c_t < 4) trp[4 * c_t + 3] = (int)wall_clock64();
      if (c_t == nt - 1) {                  // the phase ends
        if (c_ph == PH_ATTN) attn_records();
        lds_barrier();                      // partial results are in LDS after barrier A
        // burst: the held-back slots, oldest first; slot (SL + i) % NT is the i-th to be consumed from here.
        // It comes after the barrier: the memory system takes requests only as fast as it serves them, so
        // this wavefront sits here for as long as the exchange wavefronts need for epilogue and exchange.
        if (NT >= 1 && 1 > NT - held) issue_tile(std::integral_constant<int, (SL + 1) % NT>{});
        if (NT >= 2 && 2 > NT - held) issue_tile(std::integral_constant<int, (SL + 2) % NT>{});
        if (NT >= 3 && 3 > NT - held) issue_tile(std::integral_constant<int, (SL + 3) % NT>{});
        if (NT >= 4 && 4 > NT - held) issue_tile(std::integral_constant<int, (SL + 4) % NT>{});
      }
      next_tile(c_layer, c_ph, c_t);
      return true;
    };

    static_assert(NT >= 2 && NT <= kRingMax && D >= 0 && D <= NT, "ring depth");
    issue_tile(std::integral_constant<int, 0>{}); issue_tile(std::integral_constant<int, 1>{});
    if (NT > 2) issue_tile(std::integral_constant<int, 2 % NT>{});
    if (NT > 3) issue_tile(std::integral_constant<int, 3 % NT>{});
    if (NT > 4) issue_tile(std::integral_constant<int, 4 % NT>{});
    if (NT > 5) issue_tile(std::integral_constant<int, 5 % NT>{});
    for (;;) {
      if (!body(std::integral_constant<int, 0>{})) return;
      if (!body(std::integral_constant<int, 1>{})) return;
      if (NT > 2) if (!body(std::integral_constant<int, 2 % NT>{})) return;
      if (NT > 3) if (!body(std::integral_constant<int, 3 % NT>{})) return;
      if (NT > 4) if (!body(std::integral_constant<int, 4 % NT>{})) return;
      if (NT > 5) if (!body(std::integral_constant<int, 5 % NT>{})) return;
    }
  } else {
    // =======================================================================================
    // exchange role
    // =======================================================================================
    const int et = threadIdx.x - S * 64, ew = wave - S;
    constexpr int ET = E * 64;
    const unsigned e_end = a.epoch0 + 5u * (unsigned)a.n_layer;
    if (tiles_layer == 0) {
      if (et == 0) __hip_atomic_store(a.flags + wg, e_end, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
    }
    const Watch watch{a.err, si + L_ABORT, a.spin_limit};
    const bool att_new = att_s1 == a.ctx;          // this split holds the newest position
    const bool tr = et == 0;

    // waits until every workgroup has finished all phases before `e` (a hint: data validates itself)
    // One wavefront polls (every poll of every workgroup lands on the same few cache lines, and requests
    // queued there delay the weight stream behind them); the others watch a word in LDS.
    auto wait_flags = [&](unsigned e) __attribute__((always_inline)) {
      int it = 0;
      if (ew == 0) {
        for (;;) {
          bool all = true;
          for (int i = lane; i < nwg; i += 64) {
            const unsigned v = __hip_atomic_load(a.flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            all = all && ((int)(v - e) >= 0);
          }
          if (__all(all)) break;
          if (++it > a.spin_limit) { give_up(watch); break; }
          __builtin_amdgcn_s_sleep(4);
        }
        __hip_atomic_store(si + L_GO, (int)e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      } else {
        while (__hip_atomic_load(si + L_GO, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != (int)e) {
          if (++it > 64 * a.spin_limit) { give_up(watch); break; }
          __builtin_amdgcn_s_sleep(1);
        }
      }
    };
    // n values published by the previous phase -> LDS (optionally scaled)
    // n values published by the previous phase -> LDS: as fp32 (scaled), or, with n_pad >= 0, in the
    // matrices' type and zero-filled up to n_pad elements (whole tiles of columns)
    auto stage = [&](const tagged_t* src, int n, lds_float* dst, unsigned tag, float scale, int n_pad) __attribute__((always_inline)) {
      constexpr int U = 16;                      // loads in flight per thread
      for (int i0 = et; i0 < n; i0 += U * ET) {
        tagged_t raw[U];
#pragma unroll
        for (int j = 0; j < U; ++j) { const int i = i0 + j * ET; raw[j] = i < n ? ld_raw(src + i) : 0ull; }
#pragma unroll
        for (int j = 0; j < U; ++j) {
          const int i = i0 + j * ET;
          if (i < n) {
            const float v = settle(src + i, raw[j], tag, watch);
            if (n_pad >= 0) xs_put<WT>(dst, i, v); else dst[i] = v * scale;
          }
        }
      }
      for (int i = n + et; i < n_pad; i += ET) xs_put<WT>(dst, i, 0.f);
    };
    // norm gain (and bias) of the coming phase -> LDS, requested before the wait for the producers
    auto prefetch_norm = [&](const float* g, const float* b) __attribute__((always_inline)) {
      constexpr int GB = 8;
      for (int i0 = et; i0 < a.d; i0 += GB * ET) {
        float gv[GB], bv[GB];
#pragma unroll
        for (int j = 0; j < GB; ++j) { const int i = i0 + j * ET; gv[j] = i < a.d ? g[i] : 0.f; bv[j] = (b && i < a.d) ? b[i] : 0.f; }
#pragma unroll
        for (int j = 0; j < GB; ++j) { const int i = i0 + j * ET; if (i < a.d) { gain[i] = gv[j]; if (b) gbias[i] = bv[j]; } }
      }
    };
    auto normalise = [&](const float* b) __attribute__((always_inline)) {
      const int n = a.d;
      float mean = 0.f, rstd;
      if (a.norm_kind == MDI_NORM_LAYERNORM) {
        float s = 0.f;
        for (int i = lane; i < n; i += 64) s += xraw[i];
        mean = wave_sum(s) / (float)n;
        float s2 = 0.f;
        for (int i = lane; i < n; i += 64) { const float c = xraw[i] - mean; s2 += c * c; }
        rstd = 1.f / sqrtf(wave_sum(s2) / (float)n + a.eps);
      } else {
        float s2 = 0.f;
        for (int i = lane; i < n; i += 64) s2 += xraw[i] * xraw[i];
        rstd = 1.f / sqrtf(wave_sum(s2) / (float)n + a.eps);
      }
      for (int i = et; i < n; i += ET) xs_put<WT>(xs, i, (xraw[i] - mean) * rstd * gain[i] + (b ? gbias[i] : 0.f));
      for (int i = n + et; i < k_tiles<WT>(n) * 4 * V; i += ET) xs_put<WT>(xs, i, 0.f);
    };

    const lds_int* gq = si + L_GEO;
    const int nb_d = rfl(gq[1 * L_GEO_INTS + G_NB]);   // blocks of the residual stream this workgroup owns

    if (et == 0 && ntp[0] == 0) {                       // nothing to do in the first phases: say so at once
      int q = 0;
      while (ntp[q] == 0) ++q;
      __hip_atomic_store(a.flags + wg, a.epoch0 + (unsigned)q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    for (int layer = 0; layer < a.n_layer; ++layer) {
      const StepLayer L = layer_at(a, layer);
      for (int ph = 0; ph < 5; ++ph) {
        if (rfl(ntp[ph]) == 0) continue;
        const unsigned e = a.epoch0 + 5u * (unsigned)layer + (unsigned)ph;   // inputs carry e, outputs e + 1
        const unsigned wtag = e + 1;
        const bool first = layer == 0 && ph == 0;
        stamp(a, tr, layer, ph, 0);
        if (ph == PH_QKV) prefetch_norm(L.ln1_g, L.ln1_b); else if (ph == PH_UP) prefetch_norm(L.ln2_g, L.ln2_b);
        if (!first) wait_flags(e);
        stamp(a, tr, layer, ph, 1);

        // ---- the phase's input vector --------------------------------------------------------
        if (ph == PH_QKV) {
          if (first) {
            // the step's own input: token embedding (+ learned position) or the previous stage's activation
            if (a.in_kind == IN_TOKEN) {
              const long tok = checked_token(a.in, 0, a.vocab, a.err);
              for (int i = et; i < a.d; i += ET) {
                float v = Storage<WT>::get((const WT*)a.wte + tok * a.d + i);
                if (a.wpe) v += Storage<WT>::get((const WT*)a.wpe + (long)a.pos * a.d + i);
                xraw[i] = v;
              }
            } else {
              for (int i = et; i < a.d; i += ET) xraw[i] = load_kind(a.in, a.in_kind, i);
            }
          } else {
            stage(a.xres, a.d, xraw, e, 1.f, -1);
          }
        } else if (ph == PH_ATTN) {
          stage(a.q + (long)att_hg * G * h, G * h, xs, e, a.scale, -1);
          if (att_new) {
            stage(a.knew + (long)att_kvh * h, h, xs + G * h, e, 1.f, -1);
            stage(a.knew + (long)(a.K + att_kvh) * h, h, xs + G * h + h, e, 1.f, -1);
          }
        } else if (ph == PH_OPROJ) {
          stage(a.o, a.H * h, xs, e, 1.f, k_tiles<WT>(a.H * h) * 4 * V);
        } else if (ph == PH_UP) {
          stage(a.xres, a.d, xraw, e, 1.f, -1);
        } else {
          stage(a.u, a.F, xs, e, 1.f, k_tiles<WT>(a.F) * 4 * V);
        }
        stamp(a, tr, layer, ph, 2);
        lds_barrier();                                   // B
        if (ph == PH_QKV) {
          if (first)                                       // rows of the residual stream this workgroup owns
            for (int i = et; i < 16 * nb_d; i += ET) {
              const int r = (wg + (i >> 4) * nwg) * 16 + (i & 15);
              own[i] = r < a.d ? xraw[r] : 0.f;
            }
          normalise(L.ln1_b);
        } else if (ph == PH_UP) {
          normalise(L.ln2_b);
        }
        lds_barrier();                                   // C
        if (si[L_ABORT]) return;
        stamp(a, tr, layer, ph, 3);
        if (ph == PH_ATTN) {
          // the newest position (not in the cache yet) as one more record, formed while the others stream
          const lds_float* kn = xs + G * h;
          const lds_float* vn = kn + h;
          for (int gi = ew; gi < G; gi += E) {
            lds_float* r = rec + (S * G + gi) * recsz;
            float s = 0.f;
            if (att_new) for (int i = lane; i < h; i += 64) s += xs[gi * h + i] * kn[i];
            s = wave_sum(s);
            for (int i = lane; i < h; i += 64) r[i] = att_new ? vn[i] : 0.f;
            if (lane == 0) { r[h] = att_new ? s : -1e30f; r[h + 1] = att_new ? 1.f : 0.f; }
          }
        }
        lds_barrier();                                   // A
        stamp(a, tr, layer, ph, 4);

        // ---- epilogue --------------------------------------------------------------------------
        if (ph == PH_ATTN) {
          for (int gi = ew; gi < G; gi += E) {
            const int head = att_hg * G + gi;
            float m = -1e30f;
            for (int w = 0; w <= S; ++w) m = fmaxf(m, rec[(w * G + gi) * recsz + h]);
            float l = 0.f;
            for (int w = 0; w <= S; ++w) { const lds_float* r = rec + (w * G + gi) * recsz; l += r[h + 1] * __expf(r[h] - m); }
            const bool single = a.n_splits == 1;
            tagged_t* pr = a.part + ((long)head * kMaxSplits + att_split) * recsz;
            for (int i = lane; i < h; i += 64) {
              float o = 0.f;
              for (int w = 0; w <= S; ++w) { const lds_float* r = rec + (w * G + gi) * recsz; o += r[i] * __expf(r[h] - m); }
              if (single) st_tag(a.o + (long)head * h + i, o / l, wtag); else st_tag(pr + i, o, wtag);
            }
            if (single) continue;
            if (lane == 0) { st_tag(pr + h, m, wtag); st_tag(pr + h + 1, l, wtag); }
            // the last workgroup of the head to arrive folds the splits in split order
            unsigned ticket = 0;
            if (lane == 0) ticket = __hip_atomic_fetch_add(a.tickets + head, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ticket = (unsigned)rfl((int)ticket);
            if (ticket != (unsigned)a.n_splits - 1) continue;
            const tagged_t* p0 = a.part + (long)head * kMaxSplits * recsz;
            for (int i = lane; i < h; i += 64) {
              float mm = -1e30f, ll = 0.f, oo = 0.f;
              for (int sp0 = 0; sp0 < a.n_splits; sp0 += 8) {
                tagged_t rm[8], rl[8], ro[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                  const bool ok = sp0 + k < a.n_splits;
                  const tagged_t* r = p0 + (sp0 + k) * recsz;
                  rm[k] = ok ? ld_raw(r + h) : 0ull; rl[k] = ok ? ld_raw(r + h + 1) : 0ull; ro[k] = ok ? ld_raw(r + i) : 0ull;
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                  if (sp0 + k < a.n_splits) {
                    const tagged_t* r = p0 + (sp0 + k) * recsz;
                    const float mk = settle(r + h, rm[k], wtag, watch);
                    const float lk = settle(r + h + 1, rl[k], wtag, watch);
                    const float ok_ = settle(r + i, ro[k], wtag, watch);
                    const float mn = fmaxf(mm, mk);
                    const float sa = __expf(mm - mn), sb = __expf(mk - mn);
                    ll = ll * sa + lk * sb;
                    oo = oo * sa + ok_ * sb;
                    mm = mn;
                  }
                }
              }
              st_tag(a.o + (long)head * h + i, oo / ll, wtag);
            }
            if (lane == 0) __hip_atomic_store(a.tickets + head, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        } else {
          const lds_int* go = gq + gemv_index(ph) * L_GEO_INTS;
          const int nb = rfl(go[G_NB]), rope_h = rfl(go[G_ROPE_H]), N = rfl(go[G_N]);
          for (int pl = et; pl < nb * 8; pl += ET) {            // pair pl & 7 of this workgroup's block pl >> 3
            const int bl = pl >> 3, pi = pl & 7;
            float v0 = 0.f, v1 = 0.f;
#pragma unroll
            for (int w = 0; w < S; ++w) {
              lds_float* slot = part + (bl * S + w) * 16 + 2 * pi;
              v0 += slot[0]; v1 += slot[1];
              slot[0] = 0.f; slot[1] = 0.f;
            }
            const int p = (wg + bl * nwg) * 8 + pi;
            if (2 * p >= N) continue;                            // rows that only fill up the last block
            const int r0 = geo_row(rope_h, p, 0), r1 = geo_row(rope_h, p, 1);
            if (ph == PH_QKV) {
              if (L.bqkv) { v0 += L.bqkv[r0]; v1 += L.bqkv[r1]; }
              const int head = r0 / h, i = r0 - head * h;
              if (a.rope && head < a.H + a.K) {
                const float2 cs = a.rope[i];
                const float t0 = v0 * cs.x - v1 * cs.y, t1 = v0 * cs.y + v1 * cs.x;
                v0 = t0; v1 = t1;
              }
              if (head < a.H) {
                st_tag(a.q + r0, v0, wtag); st_tag(a.q + r1, v1, wtag);
              } else {
                // the cache row is for later launches (plain stores); this launch's attention takes the
                // same rounded values from the tagged copy
                const bool is_v = head >= a.H + a.K;
                const int kvh = head - a.H - (is_v ? a.K : 0);
                WT* dst = (WT*)L.kv + a.kv_tok_off + (long)(kvh * 2 + (is_v ? 1 : 0)) * a.pt_h + i;
                Storage<WT>::put(dst, v0); Storage<WT>::put(dst + (h >> 1), v1);
                tagged_t* kn = a.knew + (long)(is_v ? a.K * h : 0) + kvh * h + i;
                st_tag(kn, Storage<WT>::get(dst), wtag); st_tag(kn + (h >> 1), Storage<WT>::get(dst + (h >> 1)), wtag);
              }
            } else if (ph == PH_UP) {
              if (a.mlp_kind == MDI_MLP_SWIGLU) {
                st_tag(a.u + p, silu_f(v0) * v1, wtag);              // rows (2f, 2f+1) = (gate_f, up_f)
              } else {
                if (L.bup) { v0 += L.bup[r0]; if (r1 < N) v1 += L.bup[r1]; }
                const bool tanh_form = a.mlp_kind == MDI_MLP_GELU_TANH;
                st_tag(a.u + r0, tanh_form ? gelu_tanh_f(v0) : gelu_erf_f(v0), wtag);
                if (r1 < N) st_tag(a.u + r1, tanh_form ? gelu_tanh_f(v1) : gelu_erf_f(v1), wtag);
              }
            } else {                                                  // residual phases
              const float* bias = ph == PH_OPROJ ? L.bo : L.bdown;
              const bool last = ph == PH_DOWN && layer == a.n_layer - 1;
              v0 += own[2 * pl] + (bias ? bias[r0] : 0.f);             // own[] is in block order: 16 * bl + 2 * pi = 2 * pl
              own[2 * pl] = v0;
              st_tag(a.xres + r0, v0, wtag);
              if (last) store_kind(a.act_out, a.act_kind, r0, v0);
              if (r1 < N) {
                v1 += own[2 * pl + 1] + (bias ? bias[r1] : 0.f);
                own[2 * pl + 1] = v1;
                st_tag(a.xres + r1, v1, wtag);
                if (last) store_kind(a.act_out, a.act_kind, r1, v1);
              }
            }
          }
        }
        stamp(a, tr, layer, ph, 5);
        // ---- publish: done with every phase before this workgroup's next one -------------------
        if (a.trace && layer == a.n_layer - 1 && ph == 4)
          for (int i = et; i < L_TRACE_INTS; i += ET)
            a.trace[(long)gridDim.x * a.n_layer * 40 + (long)blockIdx.x * L_TRACE_INTS + i] = (unsigned)si[L_TRACE + i];
        if (et == 0) {
          unsigned nxt = e_end;
          for (int q = ph + 1; q < 5 * (layer + 1 < a.n_layer ? 2 : 1); ++q)
            if (ntp[q % 5] > 0) { nxt = a.epoch0 + 5u * (unsigned)(layer + q / 5) + (unsigned)(q % 5); break; }
          __hip_atomic_store(a.flags + wg, nxt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  }
}

// Wavefront split and ring depth per GQA group size G.  The attention state of G query heads lives
// in registers next to the ring, and the ring's registers must never be spilled or copied (a load
// still in flight would land in a register the compiler has given to something else), so larger
// groups get fewer wavefronts with more registers each, and a shorter ring.
template <int G> struct Shape { static constexpr int S = 6, E = 2, NT = 4, D = 3; };     // 8 wavefronts, 256 registers each
template <> struct Shape<4> { static constexpr int S = 6, E = 2, NT = 3, D = 2; };

template <typename WT, int G>
void launch_g(hipStream_t s, int nwg, size_t lds, const Step2Args& a) {
  using Sh = Shape<G>;
  hipLaunchKernelGGL((k_step2<WT, G, Sh::S, Sh::E, Sh::NT, Sh::D>), dim3(nwg), dim3((Sh::S + Sh::E) * 64), lds, s, a);
}
template <typename WT, int G>
hipError_t allow_g(size_t lds) {
  using Sh = Shape<G>;
  return hipFuncSetAttribute((const void*)k_step2<WT, G, Sh::S, Sh::E, Sh::NT, Sh::D>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}
template <typename WT>
void launch_t(hipStream_t s, int G, int nwg, size_t lds, const Step2Args& a) {
  switch (G) {
    case 4: launch_g<WT, 4>(s, nwg, lds, a); break;
    case 2: launch_g<WT, 2>(s, nwg, lds, a); break;
    default: launch_g<WT, 1>(s, nwg, lds, a); break;
  }
}
template <typename WT>
hipError_t allow_t(int G, size_t lds) {
  switch (G) {
    case 4: return allow_g<WT, 4>(lds);
    case 2: return allow_g<WT, 2>(lds);
    default: return allow_g<WT, 1>(lds);
  }
}

}  // namespace

void step2_shape(int G, int* S, int* E) {
  switch (G) {
    case 4: *S = Shape<4>::S; *E = Shape<4>::E; break;
    case 2: *S = Shape<2>::S; *E = Shape<2>::E; break;
    default: *S = Shape<1>::S; *E = Shape<1>::E; break;
  }
}

bool step2_allow_lds(int dtype, int G, size_t lds) {
  return (dtype == MDI_BF16 ? allow_t<bf16_t>(G, lds) : allow_t<float>(G, lds)) == hipSuccess;
}

void launch_step2(hipStream_t s, int dtype, int G, int nwg, size_t lds, const Step2Args& a) {
  if (dtype == MDI_BF16) launch_t<bf16_t>(s, G, nwg, lds, a); else launch_t<float>(s, G, nwg, lds, a);
}

}  // namespace mdi
