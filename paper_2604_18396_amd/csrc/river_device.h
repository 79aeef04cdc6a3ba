// Device code of the early-exit decode step for gfx950 (CDNA4, 64-wide wavefronts).
//
// One decode step is a fixed sequence of phases (River-LLM method section,
// "Inference with Seamless Exit"): per block RMSNorm + QKV, attention (which also applies
// RoPE and writes this position's K/V), O-proj + residual, RMSNorm + gate/up + SwiGLU,
// down-proj + residual + the three sums of the Eq. 1 similarity; then the original final
// norm + LM head + argmax.  After a token has exited, the same phases run with the block's
// 4-bit river twin and write K/V into the same cache slot.  Every phase strides over its
// work with whatever grid it is given, so the same code serves the one-kernel-per-phase
// mode and the persistent one-kernel-per-token mode.
//
// Design points for MI355X:
//  * Weight streaming is HBM-bound at batch 1.  A wavefront owns whole rows; a "step" is up
//    to 8 non-temporal 16-byte loads per lane (8 KiB per wavefront, each load 1 KiB
//    contiguous), two register sets in flight, so 8 wavefronts keep 128 KiB per CU in flight.
//  * The first steps of the NEXT phase are issued before the device-wide barrier that
//    separates the phases: weights do not depend on activations, so the HBM pipe stays
//    busy while the workgroups synchronise and exchange the small activation vector.
//  * Activations cross workgroups (and XCDs, whose L2s are not coherent with each other)
//    through agent-scope relaxed atomic stores and sc1 buffer loads; no cache-wide
//    write-back / invalidate is ever issued (they cost ~6-15 us each on this part).
//  * All reductions have a fixed order: results do not depend on timing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace river {

constexpr int kBlock = 512;        // threads per workgroup (8 wavefronts), one workgroup per CU
constexpr int kWaves = kBlock / 64;
constexpr int kNL = 8;             // 16-byte loads per lane per step
constexpr int kMaxGrid = 512;      // upper bound on workgroups per launch (partial-result arrays)
constexpr int kMaxSplits = 8;     // split-K factor of decode attention
constexpr int kRecords = 4096;     // ring of per-step records

enum { M_WQ = 0, M_WK, M_WV, M_WO, M_GATE, M_UP, M_DOWN };

struct DevLayer {
  const void *attn_norm, *ffn_norm;
  const void *w[7];               // wq wk wv wo w_gate w_up w_down, [out, in] row-major
  const uint8_t *qc[7];           // river codes, two per byte
  const void *qsz[7];             // river (scale, zero) pairs per (row, group), packed at creation
};

struct DevState {
  int cur_token;                  // token produced by the last head phase
  int slot_river[2], slot_exit[2];// exit state of the current token, by block parity (one-kernel-per-phase mode)
  unsigned int head_cnt;
};

struct Dev {
  int L, d, nq, nkv, hd, ffn, vocab, max_seq, min_exit, group, spin_limit;
  int kv_f16;                     // the KV cache of a bf16 model holds IEEE half values instead of bf16
  int bar_vector_poll;            // the barrier block is ordinary (cached) device memory: poll it with vector loads
  int xcap;                       // floats of LDS reserved for the staged input vector
  float eps, tau;
  const void *tok_emb, *final_norm, *lm_head;
  const DevLayer *layers;
  void *kcache, *vcache;          // [L][max_seq][nkv*hd] in the cache dtype
  const float2 *rope;             // [max_seq][hd/2] (cos, sin)
  float *hidden;                  // [L+1][d]  h(0..L) of the current token
  float *qbuf, *obuf;             // [nq*hd]
  float *kvcur;                   // [2][nkv*hd] K and V of the current position (cache-rounded values)
  float *h1;                      // [d]
  float *abuf;                    // [ffn]
  float *logits;                  // [vocab]
  float *part_o;                  // [nq][kMaxSplits][hd] unnormalised partial outputs
  float *part_ml;                 // [nq][kMaxSplits][4] (running max, sum, -, -)
  float *cos_part;                // [kMaxGrid][4]
  float *amax_val;                // [kMaxGrid]
  int *amax_idx;                  // [kMaxGrid]
  DevState *st;
  unsigned long long *bar;        // barrier block (see barrier_arrive): 8 counters 128 B apart, error flag at byte 1024
  int *rec_token, *rec_exit;      // [kRecords]
  float *rec_sims;                // [kRecords][L]
  unsigned long long *trace;      // [5L][2][grid] barrier arrive / release times (RIVER_TRACE builds)
};

struct StepArgs {
  int pos;            // position this token is written to
  int token;          // >= 0: token to consume; < 0: DevState::cur_token
  int forced_e;       // < 0: Eq. 1 decides; else exit position to impose
  int want_head;      // 0: skip final norm + LM head (prompt positions but the last)
  int rec_slot;       // record ring slot of this step (< 0: no record)
  int n_splits;       // split-K factor for this step's attention
  unsigned long long bar_base;   // device-wide barriers completed before this launch
};

// The descriptor and the per-block weight tables are written once (at creation) and only
// read by kernels.  Device code reads them through the constant address space: scalar
// loads that the compiler may repeat or move freely, instead of vector loads it must order
// against the kernels' own stores.
#define RIVER_CONSTANT(T, p) ((const __attribute__((address_space(4))) T *)(p))
typedef const __attribute__((address_space(4))) Dev &DevRef;
typedef const __attribute__((address_space(4))) DevLayer &LayerRef;
__device__ __forceinline__ LayerRef layer_of(DevRef D, int l) { return *RIVER_CONSTANT(DevLayer, D.layers + l); }

// Exit state of the current token, identical in every workgroup (each derives it from the
// same published sums in the same order).
struct Ctl {
  bool river;         // the token has left the backbone: blocks run as river twins
  int exit_pos;
};

// ------------------------------------------------------------------ storage

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Pointers that were themselves loaded from memory (the per-block weight tables) are
// generic to the compiler; loads through them would be FLAT instructions, which also count
// on the LDS counter and would make every LDS wait drain the weight loads in flight.
// All of them point to device memory, so they are cast to the global address space.
#define RIVER_GLOBAL(T, p) ((const __attribute__((address_space(1))) T *)(p))

template <int DT> struct Store;   // DT 0: fp32, 1: bf16
template <> struct Store<0> {
  typedef float T;
  typedef float2 SZ;              // (scale, zero) of one river group
  static constexpr int EPL = 4;   // elements per 16-byte lane load
  static __device__ __forceinline__ float ld(const void *p, size_t i) { return RIVER_GLOBAL(float, p)[i]; }
  static __device__ __forceinline__ float rnd(float v) { return v; }
  static __device__ __forceinline__ void st(void *p, size_t i, float v) { ((float *)p)[i] = v; }
  static __device__ __forceinline__ void unpack(const u32x4 &w, float (&f)[4]) {
    f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
    f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
  }
  static __device__ __forceinline__ uint4 repack(const float (&f)[4]) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
  static __device__ __forceinline__ SZ ldsz(const void *p, size_t i) {
    return make_float2(RIVER_GLOBAL(float, p)[2 * i], RIVER_GLOBAL(float, p)[2 * i + 1]);
  }
  static __device__ __forceinline__ SZ pack(float s, float z) { return make_float2(s, z); }
  static __device__ __forceinline__ float scale(const SZ &v) { return v.x; }
  static __device__ __forceinline__ float zero(const SZ &v) { return v.y; }
};
template <> struct Store<1> {
  typedef uint16_t T;
  typedef uint32_t SZ;
  static constexpr int EPL = 8;
  static __device__ __forceinline__ float ld(const void *p, size_t i) {
    return __uint_as_float((uint32_t)RIVER_GLOBAL(uint16_t, p)[i] << 16);
  }
  // round-to-nearest-even fp32 -> bf16
  static __device__ __forceinline__ uint16_t rne(float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  }
  static __device__ __forceinline__ float rnd(float v) { return __uint_as_float((uint32_t)rne(v) << 16); }
  static __device__ __forceinline__ void st(void *p, size_t i, float v) { ((uint16_t *)p)[i] = rne(v); }
  static __device__ __forceinline__ void unpack(const u32x4 &w, float (&f)[8]) {
    f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
    f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
    f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
    f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
  }
  // exact for values that are already bf16-representable
  static __device__ __forceinline__ uint4 repack(const float (&f)[8]) {
    return make_uint4((__float_as_uint(f[0]) >> 16) | (__float_as_uint(f[1]) & 0xffff0000u),
                      (__float_as_uint(f[2]) >> 16) | (__float_as_uint(f[3]) & 0xffff0000u),
                      (__float_as_uint(f[4]) >> 16) | (__float_as_uint(f[5]) & 0xffff0000u),
                      (__float_as_uint(f[6]) >> 16) | (__float_as_uint(f[7]) & 0xffff0000u));
  }
  static __device__ __forceinline__ SZ ldsz(const void *p, size_t i) { return RIVER_GLOBAL(uint32_t, p)[i]; }
  static __device__ __forceinline__ SZ pack(float s, float z) {
    return (uint32_t)rne(s) | ((uint32_t)rne(z) << 16);
  }
  static __device__ __forceinline__ float scale(const SZ &v) { return __uint_as_float(v << 16); }
  static __device__ __forceinline__ float zero(const SZ &v) { return __uint_as_float(v & 0xffff0000u); }
};

// streaming (read-once) 16- and 8-byte loads of weights
// (16 bytes travel as the native vector type u32x4: arrays of the uint4 struct are not always
// kept in registers by the compiler, and a stray element in scratch memory puts a wait for all
// outstanding loads into the streaming loop.  A component of such a vector is copied into a scalar
// before it is bit-cast: a bit cast applied to the component expression itself reads component 0.)
__device__ __forceinline__ u32x4 ld_stream16(const void *p) {
  return __builtin_nontemporal_load(RIVER_GLOBAL(u32x4, p));
}
__device__ __forceinline__ u32x4 ld_stream8(const void *p) {
  const u32x2 v = __builtin_nontemporal_load(RIVER_GLOBAL(u32x2, p));
  return u32x4{v.x, v.y, 0u, 0u};
}

// ------------------------------------- activations shared between workgroups

// Values produced in this launch and read by other workgroups are published with
// agent-scope atomic stores (written through to the device coherence point) and read
// with agent-scope loads (sc1), so they never rely on a cache-wide flush.
__device__ __forceinline__ void pub(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float sub(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16-byte agent-coherent load of base[idx .. idx+3] (idx % 4 == 0)
__device__ __forceinline__ float4 sub4(const float *base, int idx) {
  const __amdgpu_buffer_rsrc_t r =
      __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, 0x7ffffff0, 0x00020000);
  const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, idx * 4, 0, 16));
  return make_float4(v.x, v.y, v.z, v.w);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for
// every outstanding global load of the wave, i.e. for the weight prefetch in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// Workgroup barrier after which everything this workgroup has published is device-visible.
__device__ __forceinline__ void publish_barrier() {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ------------------------------------------------------------ reductions


// Sum over the 16 lanes of a DPP row; every lane gets the result.  DPP lane permutations
// only (no LDS pipe traffic): two quad permutes, then the mirrors of a half row and of a
// row, which after the previous steps hold the other half's sum.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v = dpp_add<0xB1>(v);      // quad_perm [1,0,3,2]
  v = dpp_add<0x4E>(v);      // quad_perm [2,3,0,1]
  v = dpp_add<0x141>(v);     // row_half_mirror
  v = dpp_add<0x140>(v);     // row_mirror
  return v;
}

// Sum over the wavefront, the same value (a scalar) in every lane: row sums, then the last
// lane of row r added into row r + 1 (rows 1 and 3), then the last lane of row 1 into rows
// 2 and 3; lane 63 holds the total.  Lane permutations only -- the LDS-pipe exchange this
// replaces took several times as long per step, on the critical path of every task.
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142 /* row_bcast:15 */, 0xa, 0xf, false));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143 /* row_bcast:31 */, 0xc, 0xf, false));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Sum over the workgroup in a fixed order; every thread gets the result.
// red: LDS scratch of at least 16 floats.
__device__ __forceinline__ float block_sum(float v, float *red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  lds_barrier();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  lds_barrier();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

// K sums at once (one pair of workgroup barriers), each in the order block_sum uses.
// red: LDS scratch of at least 8 K floats.
template <int K>
__device__ __forceinline__ void block_sum_k(float (&v)[K], float *red) {
#pragma unroll
  for (int k = 0; k < K; ++k) v[k] = wave_sum(v[k]);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  lds_barrier();
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int k = 0; k < K; ++k) red[w * K + k] = v[k];
  }
  lds_barrier();
#pragma unroll
  for (int k = 0; k < K; ++k) {
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += red[i * K + k];
    v[k] = t;
  }
}

__device__ __forceinline__ void argmax_take(float &v, int &i, float v2, int i2) {
  if (v2 > v || (v2 == v && i2 < i)) { v = v2; i = i2; }   // lower index wins ties
}

// (value, index) maximum over the workgroup; every thread gets the result.
// red: LDS scratch of at least 32 floats.
__device__ __forceinline__ void block_argmax(float &v, int &i, float *red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float v2 = __shfl_xor(v, o);
    const int i2 = __shfl_xor(i, o);
    argmax_take(v, i, v2, i2);
  }
  int *redi = (int *)(red + 16);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  lds_barrier();
  if ((threadIdx.x & 63) == 0) { red[w] = v; redi[w] = i; }
  lds_barrier();
  v = red[0]; i = redi[0];
  for (int k = 1; k < nw; ++k) argmax_take(v, i, red[k], redi[k]);
}

// --------------------------------------------------------- device barrier

#define RIVER_AG __HIP_MEMORY_SCOPE_AGENT

// Device-wide barrier number k (1-based, counted over the life of the context) of the
// persistent kernel, in two halves so that work which does not depend on other
// workgroups (the next phase's weight prefetch) can be issued between arriving and
// waiting.  Workgroup i adds one to counter i % 8 (eight counters on separate cache lines
// keep the contention on one address low) and does not wait for the result; a waiting
// workgroup reads all eight with independent loads and is released when they add up to
// k * gridDim.x.  Counters are monotone, so nothing is ever reset and a sum of values read
// at slightly different times can only under-count.  The hand-over is thus one atomic that
// nobody waits on plus one round of loads; a hierarchy of counters with a published
// generation needs two dependent atomics with their results and a store before anybody can
// see the release.  Only relaxed agent-scope operations are used: published values are
// already device-coherent and publish_barrier() makes every wave wait for its own stores
// before the arrival.
// The wait is bounded: after spin_limit polls, or once another workgroup has flagged an
// error, the workgroup flags the error and goes on, so every wave reaches the end of the
// kernel whatever happens.
constexpr int kBarErrorByte = 1024;      // offset of the error flag in the barrier block
constexpr int kBarBytes = 2048;
__device__ __forceinline__ int *bar_error(unsigned long long *bar) { return (int *)((char *)bar + kBarErrorByte); }

__device__ __forceinline__ void barrier_arrive(unsigned long long *bar, unsigned long long k) {
  publish_barrier();
  if (threadIdx.x == 0)
    (void)__hip_atomic_fetch_add(&bar[(blockIdx.x & 7) * 16], 1ull, __ATOMIC_RELAXED, RIVER_AG);
}
// The barrier block lives in uncached device memory and is polled with scalar loads: vector
// loads of a wavefront return in order, so a vector poll would wait for the weight prefetch
// the same wavefront has just issued -- in the workgroups that arrive last, which then start
// the next phase last (measured: 2.6 % of a dense token).  glc makes the scalar loads miss the
// scalar cache; uncached memory keeps the counters out of the (per-XCD, mutually
// non-coherent) L2s.  The first wavefront polls; the others wait at the workgroup barrier.
__device__ __forceinline__ bool barrier_poll(const unsigned long long *bar, unsigned long long target, int &err) {
  unsigned long long c0, c1, c2, c3, c4, c5, c6, c7;
  asm volatile(
      "s_load_dwordx2 %0, %9, 0x0 glc\n\t"
      "s_load_dwordx2 %1, %9, 0x80 glc\n\t"
      "s_load_dwordx2 %2, %9, 0x100 glc\n\t"
      "s_load_dwordx2 %3, %9, 0x180 glc\n\t"
      "s_load_dwordx2 %4, %9, 0x200 glc\n\t"
      "s_load_dwordx2 %5, %9, 0x280 glc\n\t"
      "s_load_dwordx2 %6, %9, 0x300 glc\n\t"
      "s_load_dwordx2 %7, %9, 0x380 glc\n\t"
      "s_load_dword %8, %9, 0x400 glc\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(c0), "=&s"(c1), "=&s"(c2), "=&s"(c3), "=&s"(c4), "=&s"(c5), "=&s"(c6), "=&s"(c7), "=&s"(err)
      : "s"(bar)
      : "memory");
  return ((c0 + c1) + (c2 + c3)) + ((c4 + c5) + (c6 + c7)) >= target;
}
// The same poll for a barrier block in ordinary device memory (contexts whose barrier block
// lives in the library's static scratch): scalar loads could be served from a stale L2 line
// there, so the counters are read with device-coherent vector loads.  These return behind the
// weight prefetch the polling wavefront has issued, which costs a few percent of a token.
__device__ __forceinline__ bool barrier_poll_vector(const unsigned long long *bar, unsigned long long target, int &err) {
  unsigned long long c = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) c += __hip_atomic_load(bar + i * 16, __ATOMIC_RELAXED, RIVER_AG);
  err = __hip_atomic_load(bar_error((unsigned long long *)bar), __ATOMIC_RELAXED, RIVER_AG);
  return c >= target;
}
__device__ __forceinline__ void barrier_wait(unsigned long long *bar, unsigned long long k, int spin_limit,
                                             int vector_poll = 0) {
  if (__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) == 0) {
    const unsigned long long target = k * gridDim.x;
    int spins = 0;
    for (;;) {
      int err;
      if (vector_poll ? barrier_poll_vector(bar, target, err) : barrier_poll(bar, target, err)) break;
      if (++spins > spin_limit || err != 0) {
        if ((threadIdx.x & 63) == 0) __hip_atomic_store(bar_error(bar), 1, __ATOMIC_RELAXED, RIVER_AG);
        break;
      }
      __builtin_amdgcn_s_sleep(2);
    }
  }
  lds_barrier();
}

// "Last workgroup to arrive" ticket: the caller's workgroup has published its partial
// result; returns true in every thread of the one workgroup that arrives last among
// `expected`, which may then read all partials (with agent-coherent loads).
__device__ __forceinline__ bool last_arriver(unsigned int *cnt, unsigned int expected, int *flag_lds) {
  publish_barrier();
  if (threadIdx.x == 0) {
    const unsigned int t = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, RIVER_AG);
    const int last = (t == expected - 1);
    if (last) __hip_atomic_store(cnt, 0u, __ATOMIC_RELAXED, RIVER_AG);
    *flag_lds = last;
  }
  lds_barrier();
  return *flag_lds != 0;
}

// ------------------------------------------------------------- LDS layout

// [0, xcap) staged vector in fp32 (or the attention merge area); then xcap/2 words for the
// staged vector as half pairs and xcap/32 floats for its per-run sums (4-bit phases of a
// bf16 model, see W4); then 32 floats of reduction scratch and the last-arriver flag.
__host__ __device__ inline int lds_half_floats(int xcap) { return xcap / 2 + xcap / 32; }
__device__ __forceinline__ float *lds_half(DevRef D, float *lds) { return lds + D.xcap; }
__device__ __forceinline__ float *lds_red(DevRef D, float *lds) { return lds + D.xcap + lds_half_floats(D.xcap); }
__device__ __forceinline__ int *lds_flag(DevRef D, float *lds) { return (int *)(lds_red(D, lds) + 32); }

// wave-uniform by construction; readfirstlane tells the compiler, so that task indices and
// row pointers live in scalar registers
__device__ __forceinline__ int wave_in_wg() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }
__device__ __forceinline__ int wave_id() { return blockIdx.x * (blockDim.x >> 6) + wave_in_wg(); }
__device__ __forceinline__ int wave_count() { return gridDim.x * (blockDim.x >> 6); }

// -------------------------------------------------------------- staging x

// The staged vector is not stored in column order.  A lane of the streaming engine owns a
// run of P = 2^lp consecutive columns per lane load (4 or 8 dense elements, 16 or 32
// codes) and reads them as P/4 float4; in column order the 64 lanes of a wavefront would
// hit the same few LDS banks (lane stride P floats).  So, within each granule of 64 P
// columns, float4 number q of every lane's run is stored lane after lane:
//   column c -> granule base + (e / 4) * 256 + lane * 4 + e % 4,  lane = (c % 64P) / P, e = c % P
// and a wavefront's read of float4 q covers 1 KB of consecutive addresses.
__device__ __forceinline__ int x_slot(int c, int lp) {
  const int P = 1 << lp;
  return ((c >> (6 + lp)) << (6 + lp)) + (((c & (P - 1)) >> 2) << 8) + (((c >> lp) & 63) << 2) + (c & 3);
}

// xl = h * rsqrt(mean(h^2) + eps) * gain   (fused RMSNorm prologue), stored for runs of
// 2^lp; h published by other workgroups, n % 4 == 0.
// `mid` is called once, after the first global loads of the vector have been issued and before
// their data is used: loads issued there (a late part of the weight prefetch) are in flight
// while the vector arrives, and cannot delay it (a wavefront's loads return in order).
#define RIVER_PIN_ORDER() __builtin_amdgcn_sched_barrier(0)
template <int DT, class Mid>
__device__ __forceinline__ void stage_norm(const float *h, const void *gain, int n, float eps, int lp,
                                           float *xl, float *red, Mid mid) {
  float ss = 0.f;
  const int stride = blockDim.x * 4;
  bool first = true;
  for (int i0 = threadIdx.x * 4; i0 < n || first; i0 += 4 * stride) {
    float4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + k * stride;
      v[k] = i < n ? sub4(h, i) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (first) {
      RIVER_PIN_ORDER();
      mid();
      RIVER_PIN_ORDER();
      first = false;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + k * stride;
      if (i < n) {
        *(float4 *)(xl + x_slot(i, lp)) = v[k];
        ss += (v[k].x * v[k].x + v[k].y * v[k].y) + (v[k].z * v[k].z + v[k].w * v[k].w);
      }
    }
  }
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)n + eps);
  for (int i = threadIdx.x * 4; i < n; i += blockDim.x * 4) {
    float4 v = *(float4 *)(xl + x_slot(i, lp));
    v.x = v.x * r * Store<DT>::ld(gain, i);
    v.y = v.y * r * Store<DT>::ld(gain, i + 1);
    v.z = v.z * r * Store<DT>::ld(gain, i + 2);
    v.w = v.w * r * Store<DT>::ld(gain, i + 3);
    *(float4 *)(xl + x_slot(i, lp)) = v;
  }
  lds_barrier();
}

// Same, the source being row `tok` of the embedding table (block 1 of a token); also
// publishes h(0) (each workgroup a slice) for the residual adds and the similarity.
// lp < 0: the half layout, written to xh (see half_store8; defined further down).
__device__ __forceinline__ void half_store8(float *xh, int n, int c, const float (&v)[8]);
template <int DT>
__device__ __forceinline__ void stage_norm_embed(DevRef D, int tok, const void *gain, int lp, float *xl,
                                                 float *xh, float *red) {
  const int n = D.d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const float v = Store<DT>::ld(D.tok_emb, (size_t)tok * n + i);
    xl[lp < 0 ? i : x_slot(i, lp)] = v;
    ss += v * v;
  }
  const int per = (n + gridDim.x - 1) / gridDim.x;
  for (int i = blockIdx.x * per + threadIdx.x; i < min(n, (int)(blockIdx.x + 1) * per); i += blockDim.x)
    pub(D.hidden + i, Store<DT>::ld(D.tok_emb, (size_t)tok * n + i));
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)n + D.eps);
  if (lp < 0) {
    for (int i = threadIdx.x * 8; i < n; i += blockDim.x * 8) {
      float v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = xl[i + k] * r * Store<DT>::ld(gain, i + k);
      half_store8(xh, n, i, v);
    }
  } else {
    for (int i = threadIdx.x; i < n; i += blockDim.x) xl[x_slot(i, lp)] = xl[x_slot(i, lp)] * r * Store<DT>::ld(gain, i);
  }
  lds_barrier();
}

template <class Mid>
__device__ __forceinline__ void stage_copy(const float *src, int n, int lp, float *xl, Mid mid) {
  lds_barrier();
  const int stride = blockDim.x * 4;
  bool first = true;
  for (int i0 = threadIdx.x * 4; i0 < n || first; i0 += 4 * stride) {
    float4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + k * stride;
      v[k] = i < n ? sub4(src, i) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (first) {
      RIVER_PIN_ORDER();
      mid();
      RIVER_PIN_ORDER();
      first = false;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + k * stride;
      if (i < n) *(float4 *)(xl + x_slot(i, lp)) = v[k];
    }
  }
  lds_barrier();
}

// The staged vector for the 4-bit phases of a bf16 model (columns a multiple of 32): rounded
// to half precision -- the river is a weight-only 4-bit format with 16-bit activations --
// and stored as the pairs the packed dot product consumes.  A lane load is 32 codes in four
// words; word w holds codes of columns 8w .. 8w+7, and its nibble pairs (k, k+4) are
// extracted two at a time, so the vector is stored as half2 (x[8w+k], x[8w+k+4]), k < 4:
// one uint4 per (lane, word), lane after lane per word (conflict-free as in x_slot):
//   uint4 (granule g, word w, lane) at word offset g * 1024 + w * 256 + lane * 4.
// Behind the pairs, sums[g * 64 + lane] = sum of the lane's 32 rounded values.
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_half2(float a, float b) {
  const half2_t h = {(_Float16)a, (_Float16)b};
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ int half_sums_offset(int n) { return ((n + 2047) >> 11) * 1024; }

// Store eight consecutive values v[0..7] (columns c .. c+7, c % 8 == 0) of the half layout
// and add their rounded sum into the run sum; the four threads that hold one lane's run
// are neighbours (c / 8 consecutive), so the run sum is a quad reduction.
__device__ __forceinline__ void half_store8(float *xh, int n, int c, const float (&v)[8]) {
  const int g = c >> 11, lane = (c >> 5) & 63, w = (c >> 3) & 3;
  uint4 o;
  o.x = pack_half2(v[0], v[4]); o.y = pack_half2(v[1], v[5]);
  o.z = pack_half2(v[2], v[6]); o.w = pack_half2(v[3], v[7]);
  *(uint4 *)((uint32_t *)xh + g * 1024 + w * 256 + lane * 4) = o;
  float sr = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) sr += (float)(_Float16)v[k];
  sr = dpp_add<0xB1>(sr);       // quad_perm [1,0,3,2]
  sr = dpp_add<0x4E>(sr);       // quad_perm [2,3,0,1]
  if (w == 0) xh[half_sums_offset(n) + g * 64 + lane] = sr;
}

// xh = half layout of h * rsqrt(mean(h^2) + eps) * gain; n % 32 == 0.  `xl` (n floats)
// holds h between the two passes.
template <int DT, class Mid>
__device__ __forceinline__ void stage_norm_half(const float *h, const void *gain, int n, float eps,
                                                float *xl, float *xh, float *red, Mid mid) {
  float ss = 0.f;
  const int stride = blockDim.x * 4;
  bool first = true;
  for (int i0 = threadIdx.x * 4; i0 < n || first; i0 += 4 * stride) {
    float4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + k * stride;
      v[k] = i < n ? sub4(h, i) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (first) {
      RIVER_PIN_ORDER();
      mid();
      RIVER_PIN_ORDER();
      first = false;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + k * stride;
      if (i < n) {
        *(float4 *)(xl + i) = v[k];
        ss += (v[k].x * v[k].x + v[k].y * v[k].y) + (v[k].z * v[k].z + v[k].w * v[k].w);
      }
    }
  }
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)n + eps);
  // whole quads of threads run the loop together (n % 32 == 0), as the run sums need
  for (int i = threadIdx.x * 8; i < n; i += blockDim.x * 8) {
    const float4 a = *(float4 *)(xl + i), b = *(float4 *)(xl + i + 4);
    float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = v[k] * r * Store<DT>::ld(gain, i + k);
    half_store8(xh, n, i, v);
  }
  lds_barrier();
}

template <class Mid>
__device__ __forceinline__ void stage_copy_half(const float *src, int n, float *xh, Mid mid) {
  lds_barrier();
  const int stride = blockDim.x * 8;
  bool first = true;
  for (int i0 = threadIdx.x * 8; i0 < n || first; i0 += 2 * stride) {
    float4 a[2], b[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int i = i0 + k * stride;
      a[k] = i < n ? sub4(src, i) : make_float4(0.f, 0.f, 0.f, 0.f);
      b[k] = i < n ? sub4(src, i + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (first) {
      RIVER_PIN_ORDER();
      mid();
      RIVER_PIN_ORDER();
      first = false;
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int i = i0 + k * stride;
      if (i < n) {                                   // whole quads of threads: n % 32 == 0
        const float v[8] = {a[k].x, a[k].y, a[k].z, a[k].w, b[k].x, b[k].y, b[k].z, b[k].w};
        half_store8(xh, n, i, v);
      }
    }
  }
  lds_barrier();
}

// ------------------------------------------------- weight streaming engine

template <int V> struct IC { static constexpr int value = V; };   // compile-time value as a tag

// Registers of one step: kNL lane loads (codes or dense weights) and, for river rows,
// the (scale, zero) pair of the group each lane load falls in.
template <int DT> struct Regs {
  u32x4 w[kNL];
  typename Store<DT>::SZ sz[kNL];
};

// The R rows of one task of a wavefront.
template <int R> struct Rows {
  const char *p[R];        // dense row / codes row
  const char *sz[R];       // (scale, zero) row (river only)
};

// Dense format: a step covers R rows x U column granules of 64 lanes x 16 bytes (R*U <= kNL).
template <int DT, int R, int U> struct Dense {
  static_assert(R * U <= kNL, "a step holds at most kNL lane loads");
  static constexpr int EPL = Store<DT>::EPL;
  static constexpr int SUB = (R * U * 2 <= kNL) ? 2 : 1;      // steps that fit one register set
  static __device__ __forceinline__ int steps(int cols) {
    const int row_bytes = cols * (int)sizeof(typename Store<DT>::T);
    return (row_bytes + U * 1024 - 1) / (U * 1024);
  }
  // `base`: first load slot of the register set to use (0, or kNL/2 for the second half)
  static __device__ __forceinline__ void issue(Regs<DT> &g, int base, const Rows<R> &rw, int cols, int group,
                                               int step, int lane) {
    const int row_bytes = cols * (int)sizeof(typename Store<DT>::T);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int off = (step * U + u) * 1024 + lane * 16;
#pragma unroll
      for (int r = 0; r < R; ++r)
        // lanes beyond the row load its last 16 bytes (fma does not use them): no load sits behind a
        // branch on the lane's column
        g.w[base + r * U + u] = ld_stream16(rw.p[r] + min(off, row_bytes - 16));
    }
  }
  static __device__ __forceinline__ void fma(const Regs<DT> &g, int base, int cols, int group, int step,
                                             const float *xl, float (&acc)[R], int lane) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int gb = (step * U + u) * 64 * EPL;            // granule base; see x_slot
      const int c = gb + lane * EPL;
      if (c < cols) {
        float x[EPL];
#pragma unroll
        for (int e = 0; e < EPL; e += 4) {
          const float4 t = *(const float4 *)(xl + gb + e * 64 + lane * 4);
          x[e] = t.x; x[e + 1] = t.y; x[e + 2] = t.z; x[e + 3] = t.w;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
          float f[EPL];
          Store<DT>::unpack(g.w[base + r * U + u], f);
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[r] = fmaf(f[e], x[e], acc[r]);
        }
      }
    }
  }
};

// River format: 4-bit codes, CPL codes per lane load (32: 16-byte loads, 16: 8-byte loads
// for column counts that are not a multiple of 32), weight = (code - zero) * scale per
// group.  Per lane load the sum over its columns is factored as
// scale * (sum code*x - zero * sum x).  group % CPL == 0, so a lane load never straddles
// a group.
template <int DT, int R, int U, int CPL> struct W4 {
  static_assert(R * U <= kNL, "a step holds at most kNL lane loads");
  static constexpr int SUB = (R * U * 2 <= kNL) ? 2 : 1;      // steps that fit one register set
  static __device__ __forceinline__ int steps(int cols) {
    return (cols + U * 64 * CPL - 1) / (U * 64 * CPL);
  }
  static __device__ __forceinline__ void issue(Regs<DT> &g, int base, const Rows<R> &rw, int cols, int group,
                                               int step, int lane) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // (lanes beyond the row load its last codes, which fma does not use: no load behind a branch)
      const int c = min(((step * U + u) * 64 + lane) * CPL, cols - CPL);
      const int gi = c / group;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        g.w[base + r * U + u] = CPL == 32 ? ld_stream16(rw.p[r] + (c >> 1)) : ld_stream8(rw.p[r] + (c >> 1));
        g.sz[base + r * U + u] = Store<DT>::ldsz(rw.sz[r], gi);
      }
    }
  }
  static __device__ __forceinline__ float dot8(uint32_t v, const float *x) {
    // byte j of v holds column 2j in the low nibble and column 2j+1 in the high nibble
    const uint32_t lo = v & 0x0f0f0f0fu, hi = (v >> 4) & 0x0f0f0f0fu;
    float a = (float)(lo & 0xffu) * x[0];
    a = fmaf((float)(hi & 0xffu), x[1], a);
    a = fmaf((float)((lo >> 8) & 0xffu), x[2], a);
    a = fmaf((float)((hi >> 8) & 0xffu), x[3], a);
    a = fmaf((float)((lo >> 16) & 0xffu), x[4], a);
    a = fmaf((float)((hi >> 16) & 0xffu), x[5], a);
    a = fmaf((float)(lo >> 24), x[6], a);
    a = fmaf((float)(hi >> 24), x[7], a);
    return a;
  }
  // Half-precision activations (bf16 models, 32 codes per lane load): xl points to the half
  // layout (see half_store8).  A code nibble n is turned into the half value 1024 + n by
  // OR-ing it into the mantissa of 1024.0, two nibbles (k, k+4) of a word at a time; the
  // packed dot product accumulates in fp32, and the 1024 offsets leave with the zero point:
  // sum (code - zero) x = sum (1024 + code) x - (zero + 1024) sum x.
  static constexpr bool HALF = DT == 1 && CPL == 32;
  static __device__ __forceinline__ float dot8h(uint32_t v, const u32x4 &xv, float a) {
    const uint32_t m = 0x000f000fu, one = 0x64006400u;
    const struct { uint32_t x, y, z, w; } xw = {xv.x, xv.y, xv.z, xv.w};    // (scalars: see ld_stream16)
    a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, (v & m) | one), __builtin_bit_cast(half2_t, xw.x), a, false);
    a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, ((v >> 4) & m) | one), __builtin_bit_cast(half2_t, xw.y), a, false);
    a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, ((v >> 8) & m) | one), __builtin_bit_cast(half2_t, xw.z), a, false);
    a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, ((v >> 12) & m) | one), __builtin_bit_cast(half2_t, xw.w), a, false);
    return a;
  }
  static __device__ __forceinline__ void fma_half(const Regs<DT> &g, int base, int cols, int step,
                                                  const float *xl, float (&acc)[R], int lane) {
    const float *sums = xl + half_sums_offset(cols);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int gi = step * U + u;                         // granule
      if ((gi * 64 + lane) * 32 < cols) {
        const uint32_t *xp = (const uint32_t *)xl + gi * 1024 + lane * 4;
        const u32x4 x0 = *(const u32x4 *)xp, x1 = *(const u32x4 *)(xp + 256);
        const u32x4 x2 = *(const u32x4 *)(xp + 512), x3 = *(const u32x4 *)(xp + 768);
        const float sx = sums[gi * 64 + lane];
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const u32x4 &w = g.w[base + r * U + u];
          const float aq = dot8h(w.w, x3, dot8h(w.z, x2, dot8h(w.y, x1, dot8h(w.x, x0, 0.f))));
          const float s = Store<DT>::scale(g.sz[base + r * U + u]), z = Store<DT>::zero(g.sz[base + r * U + u]);
          acc[r] = fmaf(s, aq - (z + 1024.0f) * sx, acc[r]);
        }
      }
    }
  }
  static __device__ __forceinline__ void fma(const Regs<DT> &g, int base, int cols, int group, int step,
                                             const float *xl, float (&acc)[R], int lane) {
    if constexpr (HALF) {
      fma_half(g, base, cols, step, xl, acc, lane);
      return;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int gb = (step * U + u) * 64 * CPL;            // granule base; see x_slot
      const int c = gb + lane * CPL;
      if (c < cols) {
        float x[CPL];
        float sx = 0.f;
#pragma unroll
        for (int e = 0; e < CPL; e += 4) {
          const float4 t = *(const float4 *)(xl + gb + e * 64 + lane * 4);
          x[e] = t.x; x[e + 1] = t.y; x[e + 2] = t.z; x[e + 3] = t.w;
          sx += (t.x + t.y) + (t.z + t.w);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const u32x4 &w = g.w[base + r * U + u];
          float aq = dot8(w.x, x) + dot8(w.y, x + 8);
          if constexpr (CPL == 32) aq += dot8(w.z, x + 16) + dot8(w.w, x + 24);
          const float s = Store<DT>::scale(g.sz[base + r * U + u]), z = Store<DT>::zero(g.sz[base + r * U + u]);
          acc[r] = fmaf(s, aq - z * sx, acc[r]);
        }
      }
    }
  }
};

// The register sets of the streaming pipeline.  The (task, step) pairs of a wavefront
// form one sequence j = 0, 1, 2, ...: task wave_id() + (j / NS) * wave_count(), step j % NS.
// An element occupies one "slot": a whole register set, or half of one for formats whose
// step needs at most kNL / 2 loads (F::SUB == 2) -- then twice as many elements are in
// flight for the same registers.  While one slot is consumed the others are in flight.
// The slots of the first sets are issued before the barrier in front of the phase, the
// last set's once the barrier has been passed (a larger burst in flight delays the barrier
// itself), so that its latency is covered by the staging of the input vector.
// `lane` is the lane id passed through an empty asm: with all phases of all blocks inlined
// into one kernel the compiler would otherwise derive every lane-offset variant once at
// kernel entry and keep (spill) them all; this way they are re-derived per phase.
__device__ __forceinline__ int fresh_lane() {
  int t = threadIdx.x & 63;
  asm volatile("" : "+v"(t));
  return t;
}
#ifndef RIVER_SETS
#define RIVER_SETS 2
#endif
constexpr int kSets = RIVER_SETS;  // register sets of the streaming pipeline (a third one only delayed the phases)
template <int DT> struct Pre {
  Regs<DT> set[kSets];
  float rh[2], r1[2];      // residual inputs of this wavefront's first two tasks (O, down phases)
  int lane;
  __device__ __forceinline__ Pre() : lane(fresh_lane()) {}
};

// Issue element j of this wavefront's sequence into slot j % (kSets * F::SUB) (nothing if
// the sequence is shorter).
template <class F, int DT, int R, class RowsOf>
__device__ __forceinline__ void issue_seq(int j, int slot, int n_tasks, int cols, int group, Pre<DT> &pre,
                                          RowsOf rows_of) {
  const int NS = F::steps(cols);
  const int t = wave_id() + (j / NS) * wave_count();
  if (t < n_tasks) {
    Rows<R> rw;
    rows_of(t, rw);
    F::issue(pre.set[slot / F::SUB], (slot % F::SUB) * (kNL / F::SUB), rw, cols, group, j % NS, pre.lane);
  }
}
// The first elements into their slots.  part 0: the slots to fill before the barrier in
// front of the phase; part 1: the rest, issued once the barrier has been passed; part 2: all.
#ifndef RIVER_EARLY_SETS
#define RIVER_EARLY_SETS 2
#endif
template <class F, int DT, int R, class RowsOf>
__device__ __forceinline__ void issue_first(int part, int n_tasks, int cols, int group, Pre<DT> &pre,
                                            RowsOf rows_of) {
  constexpr int NSLOT = kSets * F::SUB;
  constexpr int EARLY = RIVER_EARLY_SETS * F::SUB;
#pragma unroll
  for (int q = 0; q < NSLOT; ++q)
    if (part == 2 || (part == 0) == (q < EARLY)) issue_seq<F, DT, R>(q, q, n_tasks, cols, group, pre, rows_of);
}

// Runs all tasks of this wavefront of one GEMV phase.  The slots must already hold the first
// elements of the sequence (issue_first, called by the caller, possibly before the
// preceding barrier).  rows_of(task, Rows&) gives the rows of a task; epi(task, acc)
// receives the R finished dot products (identical in all lanes).
template <class F, int DT, int R, class RowsOf, class Epi>
__device__ __forceinline__ void stream_tasks(int n_tasks, int cols, int group, const float *xl,
                                             Pre<DT> &pre, RowsOf rows_of, Epi epi) {
  constexpr int NSLOT = kSets * F::SUB;
  const int nw = wave_count(), w = wave_id();
  if (w >= n_tasks) return;
  const int NS = F::steps(cols);
  const int J = ((n_tasks - w + nw - 1) / nw) * NS;      // length of this wavefront's sequence
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
  int s = 0, t = w;                                       // step and task being consumed
  for (int j = 0; j < J; j += NSLOT) {
#pragma unroll
    for (int q = 0; q < NSLOT; ++q) {
      if (j + q < J) {
        F::fma(pre.set[q / F::SUB], (q % F::SUB) * (kNL / F::SUB), cols, group, s, xl, acc, pre.lane);
        if (++s == NS) {
#pragma unroll
          for (int r = 0; r < R; ++r) acc[r] = wave_sum(acc[r]);
          epi(t, acc);
#pragma unroll
          for (int r = 0; r < R; ++r) acc[r] = 0.f;
          s = 0;
          t += nw;
        }
        if (j + q + NSLOT < J) issue_seq<F, DT, R>(j + q + NSLOT, q, n_tasks, cols, group, pre, rows_of);
      }
    }
  }
}

// ------------------------------------------------- task -> rows, per phase

enum { PH_QKV = 0, PH_O, PH_GU, PH_DOWN };

// Every GEMV phase works on a linear row space:
//   QKV   n in [0, qd + 2 kvd): rows of W_q, then W_k, then W_v
//   O     n in [0, d)
//   GU    n in [0, 2 ffn): n = 2 i is gate row i, n = 2 i + 1 is up row i
//   DOWN  n in [0, d)
// A task is R consecutive rows; R and the column granules per step U are chosen per phase
// and format so that (for the 8B shape) the tasks divide evenly over the 2048 wavefronts
// and a step fills the load slots:   dense  QKV 1x8  O 1x8  GU 2x4  DOWN 2x4
//                                    river  QKV 3x2  O 2x2  GU 2x2  DOWN 1x7
template <int PH, bool RIVER> struct Shape;
template <> struct Shape<PH_QKV, false> { static constexpr int R = 1, U = 8; };
template <> struct Shape<PH_O, false> { static constexpr int R = 1, U = 8; };
template <> struct Shape<PH_GU, false> { static constexpr int R = 2, U = 4; };
template <> struct Shape<PH_DOWN, false> { static constexpr int R = 2, U = 4; };
template <> struct Shape<PH_QKV, true> { static constexpr int R = 3, U = 2; };
template <> struct Shape<PH_O, true> { static constexpr int R = 2, U = 2; };
template <> struct Shape<PH_GU, true> { static constexpr int R = 2, U = 2; };
template <> struct Shape<PH_DOWN, true> { static constexpr int R = 1, U = 7; };

// Layout of the staged vector for the format a phase runs in: log2 of the columns a lane
// owns per lane load (x_slot), or -1 for the half layout (4-bit phases of a bf16 model
// whose column count is a multiple of 32).
template <int DT>
__device__ __forceinline__ int run_log2(bool river, int cols) {
  if (!river) return Store<DT>::EPL == 8 ? 3 : 2;
  if ((cols & 31) != 0) return 4;
  return DT == 1 ? -1 : 5;
}
// where the streaming engine finds the staged vector of that layout
__device__ __forceinline__ const float *x_area(DevRef D, float *lds, int lp) {
  return lp < 0 ? lds_half(D, lds) : lds;
}
__device__ __forceinline__ int phase_nrows(DevRef D, int ph) {
  return ph == PH_QKV ? (D.nq + 2 * D.nkv) * D.hd : ph == PH_GU ? 2 * D.ffn : D.d;
}
__device__ __forceinline__ int phase_cols(DevRef D, int ph) {
  return ph == PH_O ? D.nq * D.hd : ph == PH_DOWN ? D.ffn : D.d;
}

// linear row n of a phase -> matrix and row in it
template <int PH>
__device__ __forceinline__ void phase_row(DevRef D, int n, int &m, int &row) {
  if (PH == PH_QKV) {
    const int qd = D.nq * D.hd, kvd = D.nkv * D.hd;
    if (n < qd) { m = M_WQ; row = n; }
    else if (n < qd + kvd) { m = M_WK; row = n - qd; }
    else { m = M_WV; row = n - qd - kvd; }
  } else if (PH == PH_GU) {
    m = (n & 1) ? M_UP : M_GATE;
    row = n >> 1;
  } else {
    m = PH == PH_O ? M_WO : M_DOWN;
    row = n;
  }
}

// Row pointers of task t (rows t*R .. t*R+R-1, clamped to the last row of the phase).
template <int DT, int PH, bool RIVER, int R>
__device__ __forceinline__ void phase_rows(DevRef D, LayerRef Lw, int t, Rows<R> &rw) {
  const int cols = phase_cols(D, PH), last = phase_nrows(D, PH) - 1;
  const int gpr = (cols + D.group - 1) / D.group;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    int m, row;
    phase_row<PH>(D, min(t * R + r, last), m, row);
    if (!RIVER) {
      rw.p[r] = (const char *)Lw.w[m] + (size_t)row * cols * sizeof(typename Store<DT>::T);
      rw.sz[r] = nullptr;
    } else {
      rw.p[r] = (const char *)Lw.qc[m] + (size_t)row * (cols >> 1);
      rw.sz[r] = (const char *)Lw.qsz[m] + (size_t)row * gpr * sizeof(typename Store<DT>::SZ);
    }
  }
}

// f(Format type tag) is called with the streaming format of (PH, river, column count).
template <class F> struct Tag { typedef F type; };
template <int DT, int PH, class Fn>
__device__ __forceinline__ void with_format(DevRef D, bool river, Fn f) {
  if (!river) {
    f(Tag<Dense<DT, Shape<PH, false>::R, Shape<PH, false>::U>>(), IC<false>(), IC<Shape<PH, false>::R>());
  } else if ((phase_cols(D, PH) & 31) == 0) {
    f(Tag<W4<DT, Shape<PH, true>::R, Shape<PH, true>::U, 32>>(), IC<true>(), IC<Shape<PH, true>::R>());
  } else {
    f(Tag<W4<DT, Shape<PH, true>::R, Shape<PH, true>::U, 16>>(), IC<true>(), IC<Shape<PH, true>::R>());
  }
}

// Issue the first elements of this wavefront's sequence of phase PH of block l (dense or
// river), one per slot.
template <int DT, int PH>
__device__ __forceinline__ void prefetch_phase_t(DevRef D, int l, bool river, Pre<DT> &g, int part) {
  LayerRef Lw = layer_of(D, l);
  with_format<DT, PH>(D, river, [&](auto ftag, auto rv, auto rr) {
    typedef typename decltype(ftag)::type F;
    constexpr bool RV = decltype(rv)::value;
    constexpr int R = decltype(rr)::value;
    auto rows_of = [&](int t, Rows<R> &rw) { phase_rows<DT, PH, RV, R>(D, Lw, t, rw); };
    const int n = (phase_nrows(D, PH) + R - 1) / R, cols = phase_cols(D, PH);
    issue_first<F, DT, R>(part, n, cols, D.group, g, rows_of);
    // The residual inputs of the phases that add to the hidden state (h for O and down, h1
    // for down) were published at least one barrier ago: fetch them for the first two tasks
    // now, so that the epilogue does not wait for them.
    if ((PH == PH_O || PH == PH_DOWN) && part != 1) {
      const float *hin = D.hidden + (size_t)l * D.d;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row = (wave_id() + j * wave_count()) * R + g.lane;
        const bool ok = g.lane < R && row < D.d;
        g.rh[j] = ok ? sub(hin + row) : 0.f;
        if (PH == PH_DOWN) g.r1[j] = ok ? sub(D.h1 + row) : 0.f;
      }
    }
  });
}
template <int DT>
__device__ __forceinline__ void prefetch_phase(DevRef D, int l, int ph, bool river, Pre<DT> &g, int part = 2) {
  switch (ph) {
    case PH_QKV: prefetch_phase_t<DT, PH_QKV>(D, l, river, g, part); break;
    case PH_O: prefetch_phase_t<DT, PH_O>(D, l, river, g, part); break;
    case PH_GU: prefetch_phase_t<DT, PH_GU>(D, l, river, g, part); break;
    default: prefetch_phase_t<DT, PH_DOWN>(D, l, river, g, part); break;
  }
}

// Run phase PH of block l over the staged vector.  epi(n0, acc) is called once per task with
// its first linear row n0 and the R finished dot products (lane-uniform); rows >= the row
// count of the phase (a ragged last task) must be ignored by it.
template <int DT, int PH, class Epi>
__device__ __forceinline__ void run_phase(DevRef D, int l, bool river, const float *xl,
                                          Pre<DT> &pre, Epi epi) {
  LayerRef Lw = layer_of(D, l);
  with_format<DT, PH>(D, river, [&](auto ftag, auto rv, auto rr) {
    typedef typename decltype(ftag)::type F;
    constexpr bool RV = decltype(rv)::value;
    constexpr int R = decltype(rr)::value;
    auto rows_of = [&](int t, Rows<R> &rw) { phase_rows<DT, PH, RV, R>(D, Lw, t, rw); };
    auto e = [&](int t, float (&acc)[R]) { epi(t * R, acc); };
    stream_tasks<F, DT, R>((phase_nrows(D, PH) + R - 1) / R, phase_cols(D, PH), D.group, xl, pre, rows_of, e);
  });
}

// value of acc[lane] for lane < R.  Register arrays cannot be indexed by a lane id, and a chain of
// selects is turned back into such an index by the compiler (which then keeps the accumulators of
// the streaming loop in scratch memory): the value is put together from masked bit patterns.
template <int R>
__device__ __forceinline__ float pick(const float (&acc)[R], int lane) {
  uint32_t bits = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) bits |= __float_as_uint(acc[r]) & (uint32_t)-(int)(lane == r);
  return __uint_as_float(bits);
}

// diagnostics build: workgroup 0 stamps the 100 MHz wall clock at marked points of the
// last block's phases (after the barrier stamps in Dev::trace)
#ifdef RIVER_TRACE
#define RIVER_MARK(D, id)                                                                    \
  do {                                                                                        \
    if (blockIdx.x == 0 && threadIdx.x == 0)                                                  \
      (D).trace[(size_t)5 * (D).L * 2 * gridDim.x + (id)] = wall_clock64();                   \
  } while (0)
#define RIVER_MARK_SYNC(D, id)                                                               \
  do {                                                                                        \
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");                               \
    RIVER_MARK(D, id);                                                                        \
  } while (0)
#else
#define RIVER_MARK(D, id)
#define RIVER_MARK_SYNC(D, id)
#endif

// ------------------------------------------------------------------ phases

// Eq. 1 for block l1 = l (1-based) from the sums the down-projection phase of that block
// published; every workgroup computes the same value in the same order.  Returns s.
__device__ __forceinline__ float similarity_from_partials(DevRef D, float *red) {
  float pab = 0.f, paa = 0.f, pbb = 0.f;
  for (int i = threadIdx.x; i < (int)gridDim.x; i += blockDim.x) {
    const float4 v = sub4(D.cos_part, i * 4);
    pab += v.x; paa += v.y; pbb += v.z;
  }
  float p3[3] = {pab, paa, pbb};
  block_sum_k<3>(p3, red);
  pab = p3[0]; paa = p3[1]; pbb = p3[2];
  float s = 0.f;
  if (paa > 0.f && pbb > 0.f) {
    s = pab / (sqrtf(paa) * sqrtf(pbb));
    s = fminf(1.0f, fmaxf(-1.0f, s));
  }
  return s;
}

// Exit test after backbone block l1 (1-based), Eq. 1: first hit at or above L_s, never at
// L, strict '>'; a forced exit position overrides the threshold.  With a forced position the
// decision needs no similarity, so the reduction is kept off the path of every workgroup:
// the similarity is then computed for the record only, by one workgroup that has nothing to
// do in the attention phase (record_similarity).
__device__ __forceinline__ void exit_test(DevRef D, const StepArgs &A, int l1, Ctl &ctl, float *lds) {
  if (ctl.river) return;
  const bool may = l1 >= D.min_exit && l1 < D.L;
  if (A.forced_e >= 0) {
    if (may && A.forced_e == l1) { ctl.river = true; ctl.exit_pos = l1; }
    return;
  }
  const float s = similarity_from_partials(D, lds_red(D, lds));
  if (blockIdx.x == 0 && threadIdx.x == 0 && A.rec_slot >= 0)
    pub(D.rec_sims + (size_t)A.rec_slot * D.L + (l1 - 1), s);
  if (may && s > D.tau) {
    ctl.river = true;
    ctl.exit_pos = l1;
  }
}
// The similarity of backbone block l1 for the record of a forced-exit step (see exit_test).
// ctl is the exit state AFTER the test that followed block l1.  Called by every workgroup in
// the attention phase of the next block; the last workgroup does the work (the per-workgroup
// sums it reads stay valid until the next down-projection).
__device__ __forceinline__ void record_similarity(DevRef D, const StepArgs &A, int l1, const Ctl &ctl, float *lds) {
  if (l1 < 1 || A.forced_e < 0 || A.rec_slot < 0 || blockIdx.x != gridDim.x - 1) return;
  if (ctl.river && ctl.exit_pos < l1) return;          // block l1 ran as a river block: no similarity
  const float s = similarity_from_partials(D, lds_red(D, lds));
  // device-coherent stores: the record row is written by workgroups of different XCDs
  if (threadIdx.x == 0) pub(D.rec_sims + (size_t)A.rec_slot * D.L + (l1 - 1), s);
}

// Which format will block l1 + 1 run in, as far as can be known before block l1's
// similarity is reduced (used to pick what to prefetch across the block boundary).
__device__ __forceinline__ bool guess_river_after(const StepArgs &A, const Ctl &ctl, int l1) {
  return ctl.river || A.forced_e == l1;
}

// a0 + a1: (block 1: h(0) = E[token]); x = RMSNorm(h) * g1; [q;k;v] = W x, published raw.
// RoPE, the rounding of k, v to the cache dtype and the write of slot (l, pos) happen in the
// attention phase (a2 there), which frees the row-to-wavefront assignment here: single rows,
// three per wavefront at the 8B shape.
template <int DT, class Late>
__device__ __forceinline__ void phase_qkv(DevRef D, const StepArgs &A, int l, bool river, float *lds, Pre<DT> &pre,
                                          Late late) {
  RIVER_MARK(D, 16);
  LayerRef Lw = layer_of(D, l);
  if (l == 0) {
    int tok = A.token >= 0 ? A.token : D.st->cur_token;
    tok = min(max(tok, 0), D.vocab - 1);       // a NaN-poisoned argmax must not index out of range
    late();
    stage_norm_embed<DT>(D, tok, Lw.attn_norm, run_log2<DT>(river, D.d), lds, lds_half(D, lds), lds_red(D, lds));
  } else if (run_log2<DT>(river, D.d) < 0) {
    stage_norm_half<DT>(D.hidden + (size_t)l * D.d, Lw.attn_norm, D.d, D.eps, lds, lds_half(D, lds), lds_red(D, lds),
                        late);
  } else {
    stage_norm<DT>(D.hidden + (size_t)l * D.d, Lw.attn_norm, D.d, D.eps, run_log2<DT>(river, D.d), lds,
                   lds_red(D, lds), late);
  }
  RIVER_MARK(D, 17);
  const int qd = D.nq * D.hd, nrows = qd + 2 * D.nkv * D.hd;
  const int lane = pre.lane;
  auto epi = [&](int n0, auto &acc) {
    constexpr int R = sizeof(acc) / sizeof(float);
    const int n = n0 + lane;
    if (lane < R && n < nrows) {
      const float v = pick<R>(acc, lane);
      if (n < qd) pub(D.qbuf + n, v);
      else pub(D.kvcur + (n - qd), v);          // [k (kvd); v (kvd)]
    }
  };
  run_phase<DT, PH_QKV>(D, l, river, x_area(D, lds, run_log2<DT>(river, D.d)), pre, epi);
  RIVER_MARK(D, 18);
}

// a2 for the 16 lanes that share one head vector (lane dl holds elements dl*EL .. dl*EL+EL-1):
// the rotation partner i +- hd/2 of every element sits in lane dl ^ 8 at the same register
// index, so one DPP row rotation by 8 fetches it.  cs[e] = (cos, sin) of pair (dl & 7)*EL + e.
template <int EL>
__device__ __forceinline__ void rope_rotate(float (&x)[EL], const float2 (&cs)[EL], bool upper) {
#pragma unroll
  for (int e = 0; e < EL; ++e) {
    const float o = __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x[e]), 0x128 /* row_ror:8 */, 0xf, 0xf, false));
    // lower half: x c - o s;  upper half: x c + o s   (o = the partner element)
    x[e] = upper ? o * cs[e].y + x[e] * cs[e].x : x[e] * cs[e].x - o * cs[e].y;
  }
}

// a3: split-K decode attention, one workgroup per (query head, split).  Sixteen lanes
// share a cached position (EL = hd/16 elements each), so a wavefront load covers 4
// positions and the workgroup's 32 lane groups 32 positions; a chunk is RU such rounds.
// Two chunks are in flight per lane; both are issued BEFORE the device-wide barrier in
// front of the phase (old cache rows do not depend on this block's QKV) and re-issued
// alternately while the other is consumed.  The query heads of a kv head run in different
// workgroups of the same XCD (item index = kv head + nkv * ...; consecutive workgroup ids
// go round the XCDs), so the repeated K/V reads meet in that XCD's L2.  Each lane group
// keeps an online softmax (base 2, the scores carry log2 e) rescaled once per chunk; the
// four lane groups of a wavefront are merged with lane exchanges, the eight wavefronts in
// LDS in a fixed order, and the splits (if more than one) by the consumer, in split order
// -- the result is independent of timing.
// This token's own K/V come from the exchange buffer and seed the running softmax of the
// lane group that owns the current position.
#ifndef RIVER_ATTN_POS_PER_SPLIT
#define RIVER_ATTN_POS_PER_SPLIT 256
#endif
constexpr int kAttnPosPerSplit = RIVER_ATTN_POS_PER_SPLIT;   // positions a workgroup should cover before the host adds a split
constexpr float kNegBig = -1.0e30f;     // "no position yet": finite, so differences never give NaN

// LDS floats of the merge area: per wavefront hd outputs and (max, sum).
__host__ __device__ inline int attn_lds_floats(int hd) { return kWaves * (hd + 2); }

template <int DT, int EL> struct KV {                  // raw cache words of one lane: EL elements
  static constexpr int NW = EL * (int)sizeof(typename Store<DT>::T) / 4;
  uint32_t w[NW];
  __device__ __forceinline__ void load(const char *p) {
    if constexpr (NW == 2) {
      const u32x2 v = *RIVER_GLOBAL(u32x2, p);
      w[0] = v.x; w[1] = v.y;
    } else {
#pragma unroll
      for (int i = 0; i < NW; i += 4) {
        const u32x4 v = *RIVER_GLOBAL(u32x4, p + i * 4);
        w[i] = v.x; w[i + 1] = v.y; w[i + 2] = v.z; w[i + 3] = v.w;
      }
    }
  }
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int i = 0; i < NW; ++i) w[i] = 0;
  }
  // round EL values to the cache's storage type (nearest even); F16: IEEE half in a 16-bit cache
  template <bool F16 = false>
  __device__ __forceinline__ void from(const float (&f)[EL]) {
    if constexpr (DT == 1 && F16) {
#pragma unroll
      for (int i = 0; i < NW; ++i) w[i] = pack_half2(f[2 * i], f[2 * i + 1]);
    } else if constexpr (DT == 1) {
#pragma unroll
      for (int i = 0; i < NW; ++i)
        w[i] = (uint32_t)Store<1>::rne(f[2 * i]) | ((uint32_t)Store<1>::rne(f[2 * i + 1]) << 16);
    } else {
#pragma unroll
      for (int i = 0; i < NW; ++i) w[i] = __float_as_uint(f[i]);
    }
  }
  __device__ __forceinline__ void store(char *p) const {
    if constexpr (NW == 2) {
      *(uint2 *)p = make_uint2(w[0], w[1]);
    } else {
#pragma unroll
      for (int i = 0; i < NW; i += 4) *(uint4 *)(p + i * 4) = make_uint4(w[i], w[i + 1], w[i + 2], w[i + 3]);
    }
  }
  template <bool F16 = false>
  __device__ __forceinline__ void unpack(float (&f)[EL]) const {
    if constexpr (DT == 1 && F16) {
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        const half2_t h = __builtin_bit_cast(half2_t, w[i]);
        f[2 * i] = (float)h[0];
        f[2 * i + 1] = (float)h[1];
      }
    } else if constexpr (DT == 1) {
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NW; ++i) f[i] = __uint_as_float(w[i]);
    }
  }
};

// Rounds per chunk: 64 registers of K and V per chunk (two chunks are held), at most 8.
template <int DT, int EL> struct AttnShape {
  static constexpr int NW = KV<DT, EL>::NW;
  static constexpr int RU = 32 / NW > 8 ? 8 : 32 / NW;
  static constexpr int NENT = kWaves * 4;              // lane groups per workgroup
  static constexpr int CH = NENT * RU;                 // positions per chunk
};
template <int DT, int EL> struct KVChunk {
  KV<DT, EL> k[AttnShape<DT, EL>::RU], v[AttnShape<DT, EL>::RU];
};
template <int DT, int EL> struct AttnPre {             // what is fetched ahead of the barrier
  KVChunk<DT, EL> a, b;
  float2 cs[EL];                                       // RoPE (cos, sin) of the current position
};

// Geometry of the item (query head, split) a workgroup serves.
struct AttnItem { int h, kvh, sp, p0, p1; };
__device__ __forceinline__ AttnItem attn_item(DevRef D, const StepArgs &A, int item) {
  const int S = A.n_splits, T = A.pos + 1;
  const int chunk = (T + S - 1) / S;
  const int gq = D.nq / D.nkv;
  AttnItem it;
  it.kvh = item % D.nkv;
  const int r = item / D.nkv;
  it.h = it.kvh * gq + r % gq;
  it.sp = r / gq;
  it.p0 = it.sp * chunk; it.p1 = min(T, it.p0 + chunk);
  return it;
}

// Issue the loads of one chunk: positions pb + u*32 + slot for u < RU (pb already includes
// this wavefront's offset).  The current position is never read from the cache.
template <int DT, int EL>
__device__ __forceinline__ void attn_load_chunk(DevRef D, const StepArgs &A, int l, const AttnItem &it,
                                                int pb, int lane, KVChunk<DT, EL> &c) {
  typedef AttnShape<DT, EL> SH;
  const int slot = lane >> 4, dl = lane & 15;
  const int kvd = D.nkv * D.hd;
  const size_t es = sizeof(typename Store<DT>::T);
  const size_t base = ((size_t)l * D.max_seq * kvd + (size_t)it.kvh * D.hd + dl * EL) * es;
#pragma unroll
  for (int u = 0; u < SH::RU; ++u) {
    const int p = pb + u * SH::NENT + slot;
    if (p < it.p1 && p != A.pos) {
      const size_t off = base + (size_t)p * kvd * es;
      c.k[u].load((const char *)D.kcache + off);
      c.v[u].load((const char *)D.vcache + off);
    } else {
      c.k[u].zero();
      c.v[u].zero();
    }
  }
}

// What does not depend on this block's QKV, for item `item` of this workgroup: the first
// two chunks of cached K/V and the rotation table row of the current position.
template <int DT, int EL>
__device__ __forceinline__ void attn_prefetch(DevRef D, const StepArgs &A, int l, int item, int lane,
                                              AttnPre<DT, EL> &c) {
  typedef AttnShape<DT, EL> SH;
  if (item < D.nq * A.n_splits) {
    const int dl = lane & 15;
    const float *rt = (const float *)D.rope + ((size_t)A.pos * (D.hd >> 1) + (dl & 7) * EL) * 2;
#pragma unroll
    for (int e = 0; e < EL; e += 2) {
      const f32x4 t = *RIVER_GLOBAL(f32x4, rt + e * 2);
      c.cs[e] = make_float2(t.x, t.y); c.cs[e + 1] = make_float2(t.z, t.w);
    }
    const AttnItem it = attn_item(D, A, item);
    const int pb = it.p0 + wave_in_wg() * 4;
    attn_load_chunk<DT, EL>(D, A, l, it, pb, lane, c.a);
    attn_load_chunk<DT, EL>(D, A, l, it, pb + SH::CH, lane, c.b);
  }
}

// Merge the S <= kMaxSplits published split partials of query head h, elements e8 .. e8+7,
// in split order (independent of timing); all loads go out before the first is used.
__device__ __forceinline__ void combine_splits8(DevRef D, int S, int h, int e8, float (&out)[8]) {
  const size_t p_base = (size_t)h * kMaxSplits;
  float4 ml[kMaxSplits], pa[kMaxSplits], pb[kMaxSplits];
#pragma unroll
  for (int j = 0; j < kMaxSplits; ++j) {
    if (j < S) {                                       // uniform
      ml[j] = sub4(D.part_ml, (int)((p_base + j) * 4));
      pa[j] = sub4(D.part_o, (int)((p_base + j) * D.hd + e8));
      pb[j] = sub4(D.part_o, (int)((p_base + j) * D.hd + e8 + 4));
    } else {
      ml[j] = pa[j] = pb[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  float M = kNegBig;
#pragma unroll
  for (int j = 0; j < kMaxSplits; ++j) M = fmaxf(M, j < S ? ml[j].x : kNegBig);
  float Lsum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) out[e] = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxSplits; ++j) {
    const float cj = j < S ? __builtin_amdgcn_exp2f(ml[j].x - M) : 0.f;
    Lsum = fmaf(ml[j].y, cj, Lsum);
    out[0] = fmaf(pa[j].x, cj, out[0]); out[1] = fmaf(pa[j].y, cj, out[1]);
    out[2] = fmaf(pa[j].z, cj, out[2]); out[3] = fmaf(pa[j].w, cj, out[3]);
    out[4] = fmaf(pb[j].x, cj, out[4]); out[5] = fmaf(pb[j].y, cj, out[5]);
    out[6] = fmaf(pb[j].z, cj, out[6]); out[7] = fmaf(pb[j].w, cj, out[7]);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) out[e] /= Lsum;
}

// Stage the attention output for the output projection: a copy of the finished vector
// (one split), or the merge of the split partials, done by every workgroup for itself --
// that costs the consumers some more loads but no extra hand-over between workgroups.
template <class Mid>
__device__ __forceinline__ void stage_attn_out(DevRef D, const StepArgs &A, int lp, float *xl, float *xh, Mid mid) {
  const int S = A.n_splits, n = D.nq * D.hd;
  if (S == 1) {
    if (lp < 0) stage_copy_half(D.obuf, n, xh, mid);
    else stage_copy(D.obuf, n, lp, xl, mid);
    return;
  }
  mid();
  lds_barrier();
  for (int i = threadIdx.x * 8; i < n; i += blockDim.x * 8) {
    float v[8];
    combine_splits8(D, S, i / D.hd, i % D.hd, v);
    if (lp < 0) {
      half_store8(xh, n, i, v);
    } else {
      *(float4 *)(xl + x_slot(i, lp)) = make_float4(v[0], v[1], v[2], v[3]);
      *(float4 *)(xl + x_slot(i + 4, lp)) = make_float4(v[4], v[5], v[6], v[7]);
    }
  }
  lds_barrier();
}

template <int DT, int EL, bool F16>
__device__ __forceinline__ void attn_items(DevRef D, const StepArgs &A, int l, float *lds, int lane,
                                           AttnPre<DT, EL> &c) {
  typedef AttnShape<DT, EL> SH;
  constexpr int RU = SH::RU, NENT = SH::NENT, CH = SH::CH;
  const int hd = D.hd;                               // == 16 * EL
  const int S = A.n_splits;
  const int wv = wave_in_wg();
  const int slot = lane >> 4, dl = lane & 15;
  const int kvd = D.nkv * hd;
  const float qs = 1.4426950408889634f / sqrtf((float)hd);    // log2(e) / sqrt(hd)
  float *mo_o = lds;                                 // [kWaves][hd]
  float *mo_ml = lds + (size_t)kWaves * hd;          // [kWaves][2]
  for (int item = blockIdx.x; item < D.nq * S; item += gridDim.x) {
    const AttnItem it = attn_item(D, A, item);
    int pb = it.p0 + wv * 4;
    if (item != (int)blockIdx.x) attn_prefetch<DT, EL>(D, A, l, item, lane, c);   // not fetched ahead
    RIVER_MARK(D, 0);
    // q of the head and this token's own k, v (one lane group of the split that holds the
    // current position): a2's rotation at this position, then k, v rounded to the cache
    // dtype.  The first query head of a kv head also stores them in slot (l, pos) -- the
    // same slot for backbone and river -- for the tokens to come.  The own position then
    // seeds that lane group's running softmax, so the loop over cached positions has no
    // special case.
    const bool own = A.pos >= it.p0 && A.pos < it.p1 && ((A.pos - it.p0) & (NENT - 1)) == wv * 4 + slot;
    float q[EL], o[EL], m, ls;
    float kf0[EL], vf0[EL];
#pragma unroll
    for (int e = 0; e < EL; e += 4) {
      const float4 t = sub4(D.qbuf, it.h * hd + dl * EL + e);
      q[e] = t.x; q[e + 1] = t.y; q[e + 2] = t.z; q[e + 3] = t.w;
    }
    if (own) {
#pragma unroll
      for (int e = 0; e < EL; e += 4) {
        const float4 t = sub4(D.kvcur, it.kvh * hd + dl * EL + e);
        kf0[e] = t.x; kf0[e + 1] = t.y; kf0[e + 2] = t.z; kf0[e + 3] = t.w;
        const float4 u = sub4(D.kvcur, kvd + it.kvh * hd + dl * EL + e);
        vf0[e] = u.x; vf0[e + 1] = u.y; vf0[e + 2] = u.z; vf0[e + 3] = u.w;
      }
    }
    rope_rotate<EL>(q, c.cs, dl >= 8);
#pragma unroll
    for (int e = 0; e < EL; ++e) q[e] *= qs;
    m = kNegBig; ls = 0.f;
#pragma unroll
    for (int e = 0; e < EL; ++e) o[e] = 0.f;
    if (own) {
      rope_rotate<EL>(kf0, c.cs, dl >= 8);
      KV<DT, EL> tk, tv;
      tk.template from<F16>(kf0); tk.template unpack<F16>(kf0);
      tv.template from<F16>(vf0); tv.template unpack<F16>(vf0);
      if (it.h % (D.nq / D.nkv) == 0) {
        // byte offset of this lane's elements in cache slot (l, pos) of the kv head
        const size_t slot_off = (((size_t)l * D.max_seq + A.pos) * kvd + (size_t)it.kvh * hd + dl * EL) *
                                sizeof(typename Store<DT>::T);
        tk.store((char *)D.kcache + slot_off);
        tv.store((char *)D.vcache + slot_off);
      }
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EL; ++e) d = fmaf(q[e], kf0[e], d);
      m = row16_sum(d);
      ls = 1.f;
#pragma unroll
      for (int e = 0; e < EL; ++e) o[e] = vf0[e];
    }
    RIVER_MARK_SYNC(D, 5);
    // one chunk: scores of its RU positions, one rescale, then the weighted V rows
    auto consume = [&](const KVChunk<DT, EL> &ck, int pbase) {
      float sc[RU];
      float mn = m;
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const int p = pbase + u * NENT + slot;
        const bool ok = p < it.p1 && p != A.pos;       // the own position is already in (m, ls, o)
        float kf[EL];
        ck.k[u].template unpack<F16>(kf);
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < EL; ++e) d = fmaf(q[e], kf[e], d);
        d = row16_sum(d);
        sc[u] = ok ? d : kNegBig;
        mn = fmaxf(mn, sc[u]);
      }
      const float cg = __builtin_amdgcn_exp2f(m - mn);    // <= 1; 1 while nothing seen
      ls *= cg;
#pragma unroll
      for (int e = 0; e < EL; ++e) o[e] *= cg;
      m = mn;
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const float pg = sc[u] > 0.5f * kNegBig ? __builtin_amdgcn_exp2f(sc[u] - mn) : 0.f;
        ls += pg;
        float vf[EL];
        ck.v[u].template unpack<F16>(vf);
#pragma unroll
        for (int e = 0; e < EL; ++e) o[e] = fmaf(pg, vf[e], o[e]);
      }
    };
    for (; pb < it.p1; pb += 2 * CH) {
      consume(c.a, pb);
      if (pb + 2 * CH < it.p1) attn_load_chunk<DT, EL>(D, A, l, it, pb + 2 * CH, lane, c.a);
      if (pb + CH < it.p1) {
        consume(c.b, pb + CH);
        if (pb + 3 * CH < it.p1) attn_load_chunk<DT, EL>(D, A, l, it, pb + 3 * CH, lane, c.b);
      }
    }
    RIVER_MARK(D, 1);
    // the four lane groups of the wavefront -> one (lanes 16, 32 apart hold the same elements)
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float m2 = __shfl_xor(m, off), l2 = __shfl_xor(ls, off);
      const float mn = fmaxf(m, m2);
      const float c1 = __builtin_amdgcn_exp2f(m - mn), c2 = __builtin_amdgcn_exp2f(m2 - mn);
      ls = ls * c1 + l2 * c2;
#pragma unroll
      for (int e = 0; e < EL; ++e) o[e] = o[e] * c1 + __shfl_xor(o[e], off) * c2;
      m = mn;
    }
    lds_barrier();                        // merge area free (previous item fully consumed)
    if (slot == 0) {
      float *w = mo_o + wv * hd + dl * EL;
#pragma unroll
      for (int e = 0; e < EL; e += 4) *(float4 *)(w + e) = make_float4(o[e], o[e + 1], o[e + 2], o[e + 3]);
      if (dl == 0) *(float2 *)(mo_ml + wv * 2) = make_float2(m, ls);
    }
    RIVER_MARK(D, 2);
    lds_barrier();
    RIVER_MARK(D, 3);
    // the wavefronts -> one partial per (head, split), fixed order
    if ((int)threadIdx.x < hd) {
      const int e = threadIdx.x;
      float2 ml[kWaves];
      float ov[kWaves];
      float M = kNegBig;
#pragma unroll
      for (int j = 0; j < kWaves; ++j) {
        ml[j] = *(const float2 *)(mo_ml + j * 2);
        ov[j] = mo_o[j * hd + e];
        M = fmaxf(M, ml[j].x);
      }
      float Lsum = 0.f, O = 0.f;
#pragma unroll
      for (int j = 0; j < kWaves; ++j) {
        const float cj = __builtin_amdgcn_exp2f(ml[j].x - M);       // entries that saw nothing have sum 0
        Lsum = fmaf(ml[j].y, cj, Lsum);
        O = fmaf(ov[j], cj, O);
      }
      if (S == 1) {
        pub(D.obuf + it.h * hd + e, O / Lsum);
      } else {
        const size_t pi = (size_t)it.h * kMaxSplits + it.sp;
        pub(D.part_o + pi * hd + e, O);
        if (e == 0) { pub(D.part_ml + pi * 4, M); pub(D.part_ml + pi * 4 + 1, Lsum); }
      }
    }
    RIVER_MARK(D, 4);
  }
}

// The attention phase with the device-wide barrier in front of it (in the one-kernel-per-
// phase mode arrive and wait do nothing): what can be fetched ahead is issued between
// arriving and waiting.  Register arrays are sized by the elements per lane (head_dim 64
// or 128).
template <int DT, bool F16, class Arrive, class Wait>
__device__ __forceinline__ void phase_attn(DevRef D, const StepArgs &A, int l, const Ctl &ctl, float *lds,
                                           Arrive arrive, Wait wait) {
  const int lane = fresh_lane();
  auto run = [&](auto el) {
    constexpr int EL = decltype(el)::value;
    AttnPre<DT, EL> c;
    arrive();
    attn_prefetch<DT, EL>(D, A, l, blockIdx.x, lane, c);
    wait();
    attn_items<DT, EL, F16>(D, A, l, lds, lane, c);
  };
  if (D.hd == 128) run(IC<8>()); else run(IC<4>());
  lds_barrier();                                   // the merge area of the last item is read
  record_similarity(D, A, l, ctl, lds);
}

// a4: h1 = h + W_o o
template <int DT, class Late>
__device__ __forceinline__ void phase_oproj(DevRef D, const StepArgs &A, int l, bool river, float *lds, Pre<DT> &pre,
                                            Late late) {
  RIVER_MARK(D, 20);
  const int lp = run_log2<DT>(river, D.nq * D.hd);
  stage_attn_out(D, A, lp, lds, lds_half(D, lds), late);
  RIVER_MARK(D, 21);
  const float *hin = D.hidden + (size_t)l * D.d;
  const int lane = pre.lane;
  int ord = 0;                          // ordinal of the task among this wavefront's
  auto epi = [&](int n0, auto &acc) {
    constexpr int R = sizeof(acc) / sizeof(float);
    const int n = n0 + lane;
    if (lane < R && n < D.d) {
      const float h0 = ord == 0 ? pre.rh[0] : ord == 1 ? pre.rh[1] : sub(hin + n);
      pub(D.h1 + n, h0 + pick<R>(acc, lane));
    }
    ++ord;
  };
  run_phase<DT, PH_O>(D, l, river, x_area(D, lds, lp), pre, epi);
  RIVER_MARK(D, 22);
}

// a5: y = RMSNorm(h1) * g2; a = silu(W_g y) * (W_u y); rows come as (gate i, up i) pairs
template <int DT, class Late>
__device__ __forceinline__ void phase_gateup(DevRef D, const StepArgs &A, int l, bool river, float *lds, Pre<DT> &pre,
                                             Late late) {
  RIVER_MARK(D, 24);
  const int lp = run_log2<DT>(river, D.d);
  if (lp < 0)
    stage_norm_half<DT>(D.h1, layer_of(D, l).ffn_norm, D.d, D.eps, lds, lds_half(D, lds), lds_red(D, lds), late);
  else stage_norm<DT>(D.h1, layer_of(D, l).ffn_norm, D.d, D.eps, lp, lds, lds_red(D, lds), late);
  RIVER_MARK(D, 25);
  const int lane = pre.lane;
  auto epi = [&](int n0, auto &acc) {
    constexpr int R = sizeof(acc) / sizeof(float);
    static_assert(R % 2 == 0, "gate/up tasks hold whole (gate, up) pairs");
    float gv = acc[0], uv = acc[1];
#pragma unroll
    for (int k = 1; k < R / 2; ++k) { gv = lane == k ? acc[2 * k] : gv; uv = lane == k ? acc[2 * k + 1] : uv; }
    const int i = (n0 >> 1) + lane;
    if (lane < R / 2 && i < D.ffn) pub(D.abuf + i, gv / (1.0f + expf(-gv)) * uv);
  };
  run_phase<DT, PH_GU>(D, l, river, x_area(D, lds, lp), pre, epi);
  RIVER_MARK(D, 26);
}

// a6: h2 = h1 + W_d a, published as h(l+1); on backbone blocks also the three sums of
// Eq. 1's similarity <h,h2>, <h,h>, <h2,h2> reduced over this workgroup's rows.  The
// reduction over workgroups and the exit decision are taken by every workgroup at the
// start of the next block (exit_test), so no workgroup waits for another here.
template <int DT, class Late>
__device__ __forceinline__ void phase_down(DevRef D, const StepArgs &A, int l, bool river, float *lds, Pre<DT> &pre,
                                           Late late) {
  RIVER_MARK(D, 28);
  const int lp = run_log2<DT>(river, D.ffn);
  if (lp < 0) stage_copy_half(D.abuf, D.ffn, lds_half(D, lds), late);
  else stage_copy(D.abuf, D.ffn, lp, lds, late);
  RIVER_MARK(D, 29);
  const float *hin = D.hidden + (size_t)l * D.d;
  float *hout = D.hidden + (size_t)(l + 1) * D.d;
  const int lane = pre.lane;
  float ab = 0.f, aa = 0.f, bb = 0.f;
  int ord = 0;                          // ordinal of the task among this wavefront's
  auto epi = [&](int n0, auto &acc) {
    constexpr int R = sizeof(acc) / sizeof(float);
    const int n = n0 + lane;
    if (lane < R && n < D.d) {
      const float h0 = ord == 0 ? pre.rh[0] : ord == 1 ? pre.rh[1] : sub(hin + n);
      const float h1 = ord == 0 ? pre.r1[0] : ord == 1 ? pre.r1[1] : sub(D.h1 + n);
      const float h2 = h1 + pick<R>(acc, lane);
      pub(hout + n, h2);
      ab = fmaf(h0, h2, ab); aa = fmaf(h0, h0, aa); bb = fmaf(h2, h2, bb);
    }
    ++ord;
  };
  run_phase<DT, PH_DOWN>(D, l, river, x_area(D, lds, lp), pre, epi);
  RIVER_MARK(D, 30);
  if (river) return;                    // river blocks take no exit test
  float *red = lds_red(D, lds);
  float p3[3] = {ab, aa, bb};
  block_sum_k<3>(p3, red);
  if (threadIdx.x == 0) {
    pub(D.cos_part + blockIdx.x * 4 + 0, p3[0]);
    pub(D.cos_part + blockIdx.x * 4 + 1, p3[1]);
    pub(D.cos_part + blockIdx.x * 4 + 2, p3[2]);
  }
}

// a9 + a10: logits = W_head RMSNorm(h(L)) * g_f; greedy token (lowest index on ties);
// the step's record.
constexpr int kRD = 2, kUD = 4;      // LM head: two rows x four granules per step
template <int DT>
__device__ __forceinline__ void head_rows(DevRef D, int t, Rows<kRD> &rw) {
#pragma unroll
  for (int r = 0; r < kRD; ++r) {
    rw.p[r] = (const char *)D.lm_head +
              (size_t)min(t * kRD + r, D.vocab - 1) * D.d * sizeof(typename Store<DT>::T);
    rw.sz[r] = nullptr;
  }
}
template <int DT>
__device__ __forceinline__ void prefetch_head(DevRef D, Pre<DT> &g, int part = 2) {
  auto rows_of = [&](int t, Rows<kRD> &rw) { head_rows<DT>(D, t, rw); };
  const int n = (D.vocab + kRD - 1) / kRD;
  issue_first<Dense<DT, kRD, kUD>, DT, kRD>(part, n, D.d, D.group, g, rows_of);
}
template <int DT, class Late>
__device__ __forceinline__ void phase_head(DevRef D, const StepArgs &A, const Ctl &ctl, float *lds, Pre<DT> &pre,
                                           Late late) {
  float *red = lds_red(D, lds);
  if (!ctl.river && A.rec_slot >= 0) {      // similarity of the last backbone block: recorded, never tested
    const float s = similarity_from_partials(D, red);
    if (blockIdx.x == 0 && threadIdx.x == 0) pub(D.rec_sims + (size_t)A.rec_slot * D.L + (D.L - 1), s);
  }
  stage_norm<DT>(D.hidden + (size_t)D.L * D.d, D.final_norm, D.d, D.eps, run_log2<DT>(false, D.d), lds, red, late);
  const int lane = pre.lane;
  float best = -INFINITY;
  int besti = 0x7fffffff;
  auto rows_of = [&](int t, Rows<kRD> &rw) { head_rows<DT>(D, t, rw); };
  auto epi = [&](int t, float (&acc)[kRD]) {
#pragma unroll
    for (int r = 0; r < kRD; ++r) {
      const int row = t * kRD + r;
      if (row < D.vocab) {
        if (lane == 0) D.logits[row] = acc[r];
        argmax_take(best, besti, acc[r], row);
      }
    }
  };
  stream_tasks<Dense<DT, kRD, kUD>, DT, kRD>((D.vocab + kRD - 1) / kRD, D.d, D.group, lds, pre, rows_of, epi);
  block_argmax(best, besti, red);
  if (threadIdx.x == 0) {
    pub(D.amax_val + blockIdx.x, best);
    pub((float *)D.amax_idx + blockIdx.x, __int_as_float(besti));
  }
  if (last_arriver(&D.st->head_cnt, gridDim.x, lds_flag(D, lds))) {
    float b = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += blockDim.x)
      argmax_take(b, bi, sub(D.amax_val + i), __float_as_int(sub((const float *)D.amax_idx + i)));
    block_argmax(b, bi, red);
    if (threadIdx.x == 0) {
      D.st->cur_token = bi;
      if (A.rec_slot >= 0) {
        D.rec_token[A.rec_slot] = bi;
        D.rec_exit[A.rec_slot] = ctl.exit_pos;
      }
    }
  }
}

// Start-of-token state: exit position 0 (everything in the river) only when forced.
__device__ __forceinline__ Ctl ctl_init(DevRef D, const StepArgs &A) {
  Ctl c;
  c.river = (A.forced_e == 0);
  c.exit_pos = c.river ? 0 : D.L;
  return c;
}

// NaN in the record for blocks that run as river twins (no similarity there).
__device__ __forceinline__ void record_init(DevRef D, const StepArgs &A) {
  if (blockIdx.x == 0 && A.rec_slot >= 0)
    for (int i = threadIdx.x; i < D.L; i += blockDim.x)
      pub(D.rec_sims + (size_t)A.rec_slot * D.L + i, __uint_as_float(0x7fc00000u));
}

}  // namespace river
