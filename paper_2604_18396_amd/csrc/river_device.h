// Device code of the early-exit decode step for gfx950 (CDNA4, 64-wide wavefronts).
//
// One decode step is a fixed sequence of phases (River-LLM method section,
// "Inference with Seamless Exit"): per block RMSNorm+QKV+RoPE+KV write, split-K GQA
// attention, O-proj + residual, RMSNorm + gate/up + SwiGLU, down-proj + residual +
// the three sums of the Eq. 1 similarity; then the original final norm + LM head +
// argmax.  After a token has exited, the same phases run with the block's 4-bit river
// twin and write K/V into the same cache slot.  Every phase strides over its work with
// whatever grid it is given, so the same code serves the one-kernel-per-phase mode and
// the persistent one-kernel-per-token mode.
//
// Design points for MI355X:
//  * Weight streaming is HBM-bound at batch 1.  A wavefront owns whole rows; a "step" is
//    16 non-temporal 16-byte loads per lane (16 KiB per wavefront, fully coalesced 1 KiB
//    rows of loads), double buffered, so 8 wavefronts keep >= 128 KiB per CU in flight.
//  * The first step of the NEXT phase is issued before the device-wide barrier that
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
constexpr int kMaxSplits = 32;     // split-K factor of decode attention
constexpr int kMaxKvHeads = 64;
constexpr int kRecords = 4096;     // ring of per-step records

enum { M_WQ = 0, M_WK, M_WV, M_WO, M_GATE, M_UP, M_DOWN };

struct DevLayer {
  const void *attn_norm, *ffn_norm;
  const void *w[7];               // wq wk wv wo w_gate w_up w_down, [out, in] row-major
  const uint8_t *qc[7];           // river codes, two per byte
  const void *qsz[7];             // river (scale, zero) pairs per (row, group), packed at creation
};

struct DevState {
  unsigned long long grp[8 * 16]; // first-level barrier counters, one per group of workgroups, padded
  unsigned long long top;         // second-level barrier counter
  unsigned long long gen;         // index of the last completed barrier
  int error;                      // set when a bounded wait gave up
  int cur_token;                  // token produced by the last head phase
  int slot_river[2], slot_exit[2];// exit state of the current token, by block parity (one-kernel-per-phase mode)
  unsigned int head_cnt;
  unsigned int attn_cnt[kMaxKvHeads];
};

struct Dev {
  int L, d, nq, nkv, hd, ffn, vocab, max_seq, min_exit, group, spin_limit;
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
  float *part_o;                  // [nkv][kMaxSplits][G][hd] unnormalised partial outputs
  float *part_ml;                 // [nkv][kMaxSplits][G][2] (running max, sum)
  float *cos_part;                // [kMaxGrid][4]
  float *amax_val;                // [kMaxGrid]
  int *amax_idx;                  // [kMaxGrid]
  DevState *st;
  int *rec_token, *rec_exit;      // [kRecords]
  float *rec_sims;                // [kRecords][L]
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
  static __device__ __forceinline__ void unpack(const uint4 &w, float (&f)[4]) {
    f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
    f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
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
  static __device__ __forceinline__ void unpack(const uint4 &w, float (&f)[8]) {
    f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
    f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
    f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
    f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
  }
  static __device__ __forceinline__ SZ ldsz(const void *p, size_t i) { return RIVER_GLOBAL(uint32_t, p)[i]; }
  static __device__ __forceinline__ SZ pack(float s, float z) {
    return (uint32_t)rne(s) | ((uint32_t)rne(z) << 16);
  }
  static __device__ __forceinline__ float scale(const SZ &v) { return __uint_as_float(v << 16); }
  static __device__ __forceinline__ float zero(const SZ &v) { return __uint_as_float(v & 0xffff0000u); }
};

// streaming (read-once) 16- and 8-byte loads of weights
__device__ __forceinline__ uint4 ld_stream16(const void *p) {
  const u32x4 v = __builtin_nontemporal_load(RIVER_GLOBAL(u32x4, p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 ld_stream8(const void *p) {
  const u32x2 v = __builtin_nontemporal_load(RIVER_GLOBAL(u32x2, p));
  return make_uint4(v.x, v.y, 0, 0);
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

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
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
// waiting.  Two levels keep the contention on one address low: workgroup i adds to counter
// i % 8; the last of each group adds to the top counter; the last of those publishes k in
// `gen`, which everybody polls.  Counters are monotone, so nothing is ever reset.  Only
// relaxed agent-scope atomics are used: published values are already device-coherent and
// publish_barrier() makes every wave wait for its own stores before the arrival.
// The wait is bounded: after spin_limit polls, or once another workgroup has flagged an
// error, the workgroup flags the error and goes on, so every wave reaches the end of the
// kernel whatever happens.  gridDim.x must be a multiple of 8.
__device__ __forceinline__ void barrier_arrive(DevState *st, unsigned long long k) {
  publish_barrier();
  if (threadIdx.x == 0) {
    const unsigned long long per = gridDim.x >> 3;
    const unsigned long long t =
        __hip_atomic_fetch_add(&st->grp[(blockIdx.x & 7) * 16], 1ull, __ATOMIC_RELAXED, RIVER_AG);
    if (t == k * per - 1) {
      const unsigned long long t2 = __hip_atomic_fetch_add(&st->top, 1ull, __ATOMIC_RELAXED, RIVER_AG);
      if (t2 == k * 8 - 1) __hip_atomic_store(&st->gen, k, __ATOMIC_RELAXED, RIVER_AG);
    }
  }
}
__device__ __forceinline__ void barrier_wait(DevState *st, unsigned long long k, int spin_limit) {
  if (threadIdx.x == 0) {
    int spins = 0;
    while (__hip_atomic_load(&st->gen, __ATOMIC_RELAXED, RIVER_AG) < k) {
      if (++spins > spin_limit || __hip_atomic_load(&st->error, __ATOMIC_RELAXED, RIVER_AG) != 0) {
        __hip_atomic_store(&st->error, 1, __ATOMIC_RELAXED, RIVER_AG);
        break;
      }
      __builtin_amdgcn_s_sleep(8);
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

// [0, xcap) staged vector (or the attention merge area), [xcap, xcap+32) reduction
// scratch, [xcap+32] last-arriver flag.
__device__ __forceinline__ float *lds_red(const Dev &D, float *lds) { return lds + D.xcap; }
__device__ __forceinline__ int *lds_flag(const Dev &D, float *lds) { return (int *)(lds + D.xcap + 32); }

// wave-uniform by construction; readfirstlane tells the compiler, so that task indices and
// row pointers live in scalar registers
__device__ __forceinline__ int wave_in_wg() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }
__device__ __forceinline__ int wave_id() { return blockIdx.x * (blockDim.x >> 6) + wave_in_wg(); }
__device__ __forceinline__ int wave_count() { return gridDim.x * (blockDim.x >> 6); }

// -------------------------------------------------------------- staging x

// xl[0..n) = h * rsqrt(mean(h^2) + eps) * gain   (fused RMSNorm prologue); h published
// by other workgroups, n % 4 == 0.
template <int DT>
__device__ __forceinline__ void stage_norm(const float *h, const void *gain, int n, float eps,
                                           float *xl, float *red) {
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < n; i += blockDim.x * 4) {
    const float4 v = sub4(h, i);
    *(float4 *)(xl + i) = v;
    ss += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
  }
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)n + eps);
  for (int i = threadIdx.x * 4; i < n; i += blockDim.x * 4) {
    float4 v = *(float4 *)(xl + i);
    v.x = v.x * r * Store<DT>::ld(gain, i);
    v.y = v.y * r * Store<DT>::ld(gain, i + 1);
    v.z = v.z * r * Store<DT>::ld(gain, i + 2);
    v.w = v.w * r * Store<DT>::ld(gain, i + 3);
    *(float4 *)(xl + i) = v;
  }
  lds_barrier();
}

// Same, the source being row `tok` of the embedding table (block 1 of a token); also
// publishes h(0) (each workgroup a slice) for the residual adds and the similarity.
template <int DT>
__device__ __forceinline__ void stage_norm_embed(const Dev &D, int tok, const void *gain, float *xl,
                                                 float *red) {
  const int n = D.d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const float v = Store<DT>::ld(D.tok_emb, (size_t)tok * n + i);
    xl[i] = v;
    ss += v * v;
  }
  const int per = (n + gridDim.x - 1) / gridDim.x;
  for (int i = blockIdx.x * per + threadIdx.x; i < min(n, (int)(blockIdx.x + 1) * per); i += blockDim.x)
    pub(D.hidden + i, Store<DT>::ld(D.tok_emb, (size_t)tok * n + i));
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)n + D.eps);
  for (int i = threadIdx.x; i < n; i += blockDim.x) xl[i] = xl[i] * r * Store<DT>::ld(gain, i);
  lds_barrier();
}

__device__ __forceinline__ void stage_copy(const float *src, int n, float *xl) {
  lds_barrier();
  for (int i = threadIdx.x * 4; i < n; i += blockDim.x * 4) *(float4 *)(xl + i) = sub4(src, i);
  lds_barrier();
}

// ------------------------------------------------- weight streaming engine

// Registers of one step: kNL lane loads (codes or dense weights) and, for river rows,
// the (scale, zero) pair of the group each lane load falls in.
template <int DT> struct Regs {
  uint4 w[kNL];
  typename Store<DT>::SZ sz[kNL];
};

// The R rows of one task of a wavefront.
template <int R> struct Rows {
  const char *p[R];        // dense row / codes row
  const char *sz[R];       // (scale, zero) row (river only)
};

// Dense format: a step covers R rows x U = kNL / R column granules of 64 lanes x 16 bytes.
template <int DT, int R> struct Dense {
  static constexpr int U = kNL / R;
  static constexpr int EPL = Store<DT>::EPL;
  static __device__ __forceinline__ int steps(int cols) {
    const int row_bytes = cols * (int)sizeof(typename Store<DT>::T);
    return (row_bytes + U * 1024 - 1) / (U * 1024);
  }
  static __device__ __forceinline__ void issue(Regs<DT> &g, const Rows<R> &rw, int cols, int group, int step) {
    const int row_bytes = cols * (int)sizeof(typename Store<DT>::T);
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int off = (step * U + u) * 1024 + lane * 16;
#pragma unroll
      for (int r = 0; r < R; ++r)
        g.w[r * U + u] = off < row_bytes ? ld_stream16(rw.p[r] + off) : make_uint4(0, 0, 0, 0);
    }
  }
  static __device__ __forceinline__ void fma(const Regs<DT> &g, int cols, int group, int step,
                                             const float *xl, float (&acc)[R]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = ((step * U + u) * 64 + lane) * EPL;
      if (c < cols) {
        float x[EPL];
#pragma unroll
        for (int e = 0; e < EPL; e += 4) {
          const float4 t = *(const float4 *)(xl + c + e);
          x[e] = t.x; x[e + 1] = t.y; x[e + 2] = t.z; x[e + 3] = t.w;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
          float f[EPL];
          Store<DT>::unpack(g.w[r * U + u], f);
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
template <int DT, int R, int CPL> struct W4 {
  static constexpr int U = kNL / R;
  static __device__ __forceinline__ int steps(int cols) {
    return (cols + U * 64 * CPL - 1) / (U * 64 * CPL);
  }
  static __device__ __forceinline__ void issue(Regs<DT> &g, const Rows<R> &rw, int cols, int group, int step) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = ((step * U + u) * 64 + lane) * CPL;
      const int gi = c / group;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (c < cols) {
          g.w[r * U + u] = CPL == 32 ? ld_stream16(rw.p[r] + (c >> 1)) : ld_stream8(rw.p[r] + (c >> 1));
          g.sz[r * U + u] = Store<DT>::ldsz(rw.sz[r], gi);
        } else {
          g.w[r * U + u] = make_uint4(0, 0, 0, 0);
          g.sz[r * U + u] = Store<DT>::pack(0.f, 0.f);
        }
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
  static __device__ __forceinline__ void fma(const Regs<DT> &g, int cols, int group, int step,
                                             const float *xl, float (&acc)[R]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = ((step * U + u) * 64 + lane) * CPL;
      if (c < cols) {
        float x[CPL];
        float sx = 0.f;
#pragma unroll
        for (int e = 0; e < CPL; e += 4) {
          const float4 t = *(const float4 *)(xl + c + e);
          x[e] = t.x; x[e + 1] = t.y; x[e + 2] = t.z; x[e + 3] = t.w;
          sx += (t.x + t.y) + (t.z + t.w);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const uint4 &w = g.w[r * U + u];
          float aq = dot8(w.x, x) + dot8(w.y, x + 8);
          if constexpr (CPL == 32) aq += dot8(w.z, x + 16) + dot8(w.w, x + 24);
          const float s = Store<DT>::scale(g.sz[r * U + u]), z = Store<DT>::zero(g.sz[r * U + u]);
          acc[r] = fmaf(s, aq - z * sx, acc[r]);
        }
      }
    }
  }
};

// Runs all tasks of this wavefront (task ids wave_id(), + wave_count(), ...) of one GEMV
// phase.  `cur` must already hold step 0 of the first task (issued by the caller, possibly
// before the preceding barrier).  rows_of(task, Rows&) gives the rows of a task; epi(task,
// acc) receives the R finished dot products (identical in all lanes).
template <class F, int DT, int R, class RowsOf, class Epi>
__device__ __forceinline__ void stream_tasks(int n_tasks, int cols, int group, const float *xl,
                                             Regs<DT> &cur, RowsOf rows_of, Epi epi) {
  const int nw = wave_count();
  int t = wave_id();
  if (t >= n_tasks) return;
  const int NS = F::steps(cols);
  Rows<R> rw;
  rows_of(t, rw);
  int s = 0;
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
  while (true) {
    int s2 = s + 1, t2 = t;
    if (s2 == NS) { s2 = 0; t2 = t + nw; }
    const bool more = t2 < n_tasks;
    Regs<DT> nxt;
    Rows<R> rw2 = rw;
    if (more) {
      if (t2 != t) rows_of(t2, rw2);
      F::issue(nxt, rw2, cols, group, s2);
    }
    F::fma(cur, cols, group, s, xl, acc);
    if (s == NS - 1) {
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] = wave_sum(acc[r]);
      epi(t, acc);
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] = 0.f;
    }
    if (!more) break;
    cur = nxt;
    rw = rw2;
    t = t2;
    s = s2;
  }
}

// Row pointers of a task from (matrix, row) pairs.
template <int DT, int R>
__device__ __forceinline__ void set_rows(Rows<R> &rw, const DevLayer &Lw, bool river, const int (&m)[R],
                                         const int (&row)[R], int cols, int group) {
  if (!river) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      rw.p[r] = (const char *)Lw.w[m[r]] + (size_t)row[r] * cols * sizeof(typename Store<DT>::T);
      rw.sz[r] = nullptr;
    }
  } else {
    const int gpr = (cols + group - 1) / group;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      rw.p[r] = (const char *)Lw.qc[m[r]] + (size_t)row[r] * (cols >> 1);
      rw.sz[r] = (const char *)Lw.qsz[m[r]] + (size_t)row[r] * gpr * sizeof(typename Store<DT>::SZ);
    }
  }
}

// Rows per task: 2 for dense rows (2 x 8 granules per step), 4 for river rows.
constexpr int kRD = 2, kRQ = 4;

// ------------------------------------------------- task -> rows, per phase

enum { PH_QKV = 0, PH_O, PH_GU, PH_DOWN };

// number of tasks of a phase for R rows per task
template <int R>
__device__ __forceinline__ int phase_tasks(const Dev &D, int ph) {
  switch (ph) {
    case PH_QKV: return (D.nq + 2 * D.nkv) * (D.hd >> 1) * 2 / R;   // rotation pairs (2 rows each)
    case PH_O: return D.d / R;
    case PH_GU: return D.ffn * 2 / R;                               // (gate, up) row pairs
    default: return D.d / R;
  }
}
__device__ __forceinline__ int phase_cols(const Dev &D, int ph) {
  return ph == PH_O ? D.nq * D.hd : ph == PH_DOWN ? D.ffn : D.d;
}

// QKV pair index -> matrix, head, first row
__device__ __forceinline__ void qkv_pair(const Dev &D, int pair, int &m, int &hh, int &i) {
  const int half = D.hd >> 1;
  const int head = pair / half;
  i = pair % half;
  if (head < D.nq) { m = M_WQ; hh = head; }
  else if (head < D.nq + D.nkv) { m = M_WK; hh = head - D.nq; }
  else { m = M_WV; hh = head - D.nq - D.nkv; }
}

template <int DT, int R>
__device__ __forceinline__ void phase_rows(const Dev &D, const DevLayer &Lw, int ph, bool river, int t,
                                           Rows<R> &rw) {
  int m[R], row[R];
  const int cols = phase_cols(D, ph);
  if (ph == PH_QKV) {
    const int half = D.hd >> 1;
#pragma unroll
    for (int k = 0; k < R / 2; ++k) {
      int mm, hh, i;
      qkv_pair(D, t * (R / 2) + k, mm, hh, i);
      m[2 * k] = mm; m[2 * k + 1] = mm;
      row[2 * k] = hh * D.hd + i; row[2 * k + 1] = hh * D.hd + i + half;
    }
  } else if (ph == PH_GU) {
#pragma unroll
    for (int k = 0; k < R / 2; ++k) {
      m[2 * k] = M_GATE; m[2 * k + 1] = M_UP;
      row[2 * k] = t * (R / 2) + k; row[2 * k + 1] = t * (R / 2) + k;
    }
  } else {
#pragma unroll
    for (int r = 0; r < R; ++r) { m[r] = ph == PH_O ? M_WO : M_DOWN; row[r] = t * R + r; }
  }
  set_rows<DT, R>(rw, Lw, river, m, row, cols, D.group);
}

// Issue step 0 of this wavefront's first task of phase `ph` of block l (dense or river).
template <int DT>
__device__ __forceinline__ void prefetch_phase(const Dev &D, int l, int ph, bool river, Regs<DT> &g) {
  const DevLayer &Lw = D.layers[l];
  const int cols = phase_cols(D, ph);
  const int t = wave_id();
  if (!river) {
    if (t < phase_tasks<kRD>(D, ph)) {
      Rows<kRD> rw;
      phase_rows<DT, kRD>(D, Lw, ph, false, t, rw);
      Dense<DT, kRD>::issue(g, rw, cols, D.group, 0);
    }
  } else {
    if (t < phase_tasks<kRQ>(D, ph)) {
      Rows<kRQ> rw;
      phase_rows<DT, kRQ>(D, Lw, ph, true, t, rw);
      if ((cols & 31) == 0) W4<DT, kRQ, 32>::issue(g, rw, cols, D.group, 0);
      else W4<DT, kRQ, 16>::issue(g, rw, cols, D.group, 0);
    }
  }
}

// Run a block phase over the staged vector; epi2(row-slot k, task, acc[2k], acc[2k+1])
// is called for every pair of rows of a task (lane-uniform values).
template <int DT, class Epi>
__device__ __forceinline__ void run_phase(const Dev &D, int l, int ph, bool river, const float *xl,
                                          Regs<DT> &pre, Epi epi) {
  const DevLayer &Lw = D.layers[l];
  const int cols = phase_cols(D, ph);
  if (!river) {
    auto rows_of = [&](int t, Rows<kRD> &rw) { phase_rows<DT, kRD>(D, Lw, ph, false, t, rw); };
    auto e = [&](int t, float (&acc)[kRD]) { epi(t, acc[0], acc[1]); };
    stream_tasks<Dense<DT, kRD>, DT, kRD>(phase_tasks<kRD>(D, ph), cols, D.group, xl, pre, rows_of, e);
  } else {
    auto rows_of = [&](int t, Rows<kRQ> &rw) { phase_rows<DT, kRQ>(D, Lw, ph, true, t, rw); };
    auto e = [&](int t, float (&acc)[kRQ]) {
      epi(2 * t, acc[0], acc[1]);
      epi(2 * t + 1, acc[2], acc[3]);
    };
    if ((cols & 31) == 0)
      stream_tasks<W4<DT, kRQ, 32>, DT, kRQ>(phase_tasks<kRQ>(D, ph), cols, D.group, xl, pre, rows_of, e);
    else
      stream_tasks<W4<DT, kRQ, 16>, DT, kRQ>(phase_tasks<kRQ>(D, ph), cols, D.group, xl, pre, rows_of, e);
  }
}

// ------------------------------------------------------------------ phases

// Eq. 1 for block l1 = l (1-based) from the sums the down-projection phase of that block
// published; every workgroup computes the same value in the same order.  Returns s.
__device__ __forceinline__ float similarity_from_partials(const Dev &D, float *red) {
  float pab = 0.f, paa = 0.f, pbb = 0.f;
  for (int i = threadIdx.x; i < (int)gridDim.x; i += blockDim.x) {
    const float4 v = sub4(D.cos_part, i * 4);
    pab += v.x; paa += v.y; pbb += v.z;
  }
  pab = block_sum(pab, red); paa = block_sum(paa, red); pbb = block_sum(pbb, red);
  float s = 0.f;
  if (paa > 0.f && pbb > 0.f) {
    s = pab / (sqrtf(paa) * sqrtf(pbb));
    s = fminf(1.0f, fmaxf(-1.0f, s));
  }
  return s;
}

// Exit test after backbone block l1 (1-based), Eq. 1: first hit at or above L_s, never at
// L, strict '>'; a forced exit position overrides the threshold.
__device__ __forceinline__ void exit_test(const Dev &D, const StepArgs &A, int l1, Ctl &ctl, float *lds) {
  if (ctl.river) return;
  const float s = similarity_from_partials(D, lds_red(D, lds));
  if (blockIdx.x == 0 && threadIdx.x == 0 && A.rec_slot >= 0)
    D.rec_sims[(size_t)A.rec_slot * D.L + (l1 - 1)] = s;
  if (l1 >= D.min_exit && l1 < D.L && ((A.forced_e < 0 && s > D.tau) || A.forced_e == l1)) {
    ctl.river = true;
    ctl.exit_pos = l1;
  }
}

// Which format will block l1 + 1 run in, as far as can be known before block l1's
// similarity is reduced (used to pick what to prefetch across the block boundary).
__device__ __forceinline__ bool guess_river_after(const StepArgs &A, const Ctl &ctl, int l1) {
  return ctl.river || A.forced_e == l1;
}

// a0 + a1 + a2: (block 1: h(0) = E[token]); x = RMSNorm(h) * g1; [q;k;v] = W x; RoPE on
// q, k at this position; k, v rounded to the cache dtype and stored in slot (l, pos) --
// the same slot for backbone and river ("identical KV Cache addressing scheme").  A task
// owns rotation pairs (rows i and i + hd/2 of a head), so the rotation needs no exchange.
template <int DT>
__device__ __forceinline__ void phase_qkv(const Dev &D, const StepArgs &A, int l, bool river, float *lds, Regs<DT> &pre) {
  const DevLayer &Lw = D.layers[l];
  if (l == 0) {
    int tok = A.token >= 0 ? A.token : D.st->cur_token;
    tok = min(max(tok, 0), D.vocab - 1);       // a NaN-poisoned argmax must not index out of range
    stage_norm_embed<DT>(D, tok, Lw.attn_norm, lds, lds_red(D, lds));
  } else {
    stage_norm<DT>(D.hidden + (size_t)l * D.d, Lw.attn_norm, D.d, D.eps, lds, lds_red(D, lds));
  }
  const int half = D.hd >> 1;
  const int kvd = D.nkv * D.hd;
  const int lane = threadIdx.x & 63;
  auto epi = [&](int pair, float a, float b) {
    if (lane != 0) return;
    int m, hh, i;
    qkv_pair(D, pair, m, hh, i);
    if (m != M_WV) {
      const size_t ri = ((size_t)A.pos * half + i) * 2;
      const float2 cs = make_float2(RIVER_GLOBAL(float, D.rope)[ri], RIVER_GLOBAL(float, D.rope)[ri + 1]);
      const float ra = a * cs.x - b * cs.y, rb = a * cs.y + b * cs.x;
      a = ra; b = rb;
    }
    if (m == M_WQ) {
      pub(D.qbuf + hh * D.hd + i, a);
      pub(D.qbuf + hh * D.hd + i + half, b);
    } else {
      void *cache = (m == M_WK) ? D.kcache : D.vcache;
      const size_t base = ((size_t)l * D.max_seq + A.pos) * kvd + (size_t)hh * D.hd;
      Store<DT>::st(cache, base + i, a);             // for later tokens (later launches)
      Store<DT>::st(cache, base + i + half, b);
      float *cur = D.kvcur + (m == M_WK ? 0 : kvd) + hh * D.hd;
      pub(cur + i, Store<DT>::rnd(a));               // for this token's attention
      pub(cur + i + half, Store<DT>::rnd(b));
    }
  };
  run_phase<DT>(D, l, PH_QKV, river, lds, pre, epi);
}

// a3: split-K GQA decode attention.  A workgroup owns (kv head, split): its wavefronts
// stream that split's K and V rows once (16 bytes per lane, hd/EPL lanes per position)
// and serve all G query heads of the group from registers, with an online softmax per
// lane group.  Partials (max, sum, unnormalised output) are merged in a fixed order:
// lane groups, wavefronts (through LDS), then splits (by the last workgroup of the kv
// head to arrive), so the result is independent of timing.  The current position's K/V
// come from the exchange buffer; older positions from the cache.
template <int DT, int G>
__device__ __forceinline__ void attn_items(const Dev &D, const StepArgs &A, int l, float *lds) {
  constexpr int EPL = Store<DT>::EPL;
  const int hd = D.hd, LPP = hd / EPL, PPW = 64 / LPP;
  const int S = A.n_splits, T = A.pos + 1;
  const int chunk = (T + S - 1) / S;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int slot = lane / LPP, dl = lane % LPP;
  const int kvd = D.nkv * hd;
  const float inv = 1.0f / sqrtf((float)hd);
  const float NEG = -INFINITY;
  float *mo = lds;                          // merge area: per wavefront G * (hd + 2) floats
  // A kv head with more than 4 query heads is served as several "virtual" kv heads of G
  // query heads each (they stream the same K/V rows again).
  const int npass = (D.nq / D.nkv) / G;
  for (int item = blockIdx.x; item < D.nkv * npass * S; item += gridDim.x) {
    const int vh = item / S, sp = item % S;   // virtual head: query heads vh*G .. vh*G+G-1
    const int kvh = vh / npass;
    const int p0 = sp * chunk, p1 = min(T, p0 + chunk);
    float q[G][EPL], o[G][EPL], m[G], ls[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = NEG; ls[g] = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; e += 4) {
        const float4 t = sub4(D.qbuf, (vh * G + g) * hd + dl * EPL + e);
        q[g][e] = t.x * inv; q[g][e + 1] = t.y * inv; q[g][e + 2] = t.z * inv; q[g][e + 3] = t.w * inv;
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[g][e] = 0.f;
    }
    const size_t es = sizeof(typename Store<DT>::T);
    const char *Kb = (const char *)D.kcache + ((size_t)l * D.max_seq * kvd + (size_t)kvh * hd + dl * EPL) * es;
    const char *Vb = (const char *)D.vcache + ((size_t)l * D.max_seq * kvd + (size_t)kvh * hd + dl * EPL) * es;
    for (int pb = p0 + wv * PPW; pb < p1; pb += nw * PPW) {
      const int p = pb + slot;
      const bool ok = p < p1;
      float kf[EPL], vf[EPL];
      if (ok && p == A.pos) {
#pragma unroll
        for (int e = 0; e < EPL; e += 4) {
          const float4 tk = sub4(D.kvcur, kvh * hd + dl * EPL + e);
          const float4 tv = sub4(D.kvcur, kvd + kvh * hd + dl * EPL + e);
          kf[e] = tk.x; kf[e + 1] = tk.y; kf[e + 2] = tk.z; kf[e + 3] = tk.w;
          vf[e] = tv.x; vf[e + 1] = tv.y; vf[e + 2] = tv.z; vf[e + 3] = tv.w;
        }
      } else {
        const size_t off = (size_t)(ok ? p : p0) * kvd * es;
        const u32x4 kx = *RIVER_GLOBAL(u32x4, Kb + off), vx = *RIVER_GLOBAL(u32x4, Vb + off);
        const uint4 kw = make_uint4(kx.x, kx.y, kx.z, kx.w), vw = make_uint4(vx.x, vx.y, vx.z, vx.w);
        Store<DT>::unpack(kw, kf);
        Store<DT>::unpack(vw, vf);
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float sc = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) sc = fmaf(q[g][e], kf[e], sc);
        for (int s = 1; s < LPP; s <<= 1) sc += __shfl_xor(sc, s);
        if (ok) {
          const float mn = fmaxf(m[g], sc);
          const float corr = expf(m[g] - mn);       // exp(-inf) = 0 on the first position
          const float pe = expf(sc - mn);
          ls[g] = ls[g] * corr + pe;
#pragma unroll
          for (int e = 0; e < EPL; ++e) o[g][e] = o[g][e] * corr + pe * vf[e];
          m[g] = mn;
        }
      }
    }
    // merge the lane groups of this wavefront (fixed xor order); slot 0 ends with the total
    for (int s = LPP; s < 64; s <<= 1) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float m2 = __shfl_xor(m[g], s), l2 = __shfl_xor(ls[g], s);
        const float mn = fmaxf(m[g], m2);
        const float c1 = (m[g] == NEG) ? 0.f : expf(m[g] - mn);
        const float c2 = (m2 == NEG) ? 0.f : expf(m2 - mn);
        ls[g] = ls[g] * c1 + l2 * c2;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const float o2 = __shfl_xor(o[g][e], s);
          o[g][e] = o[g][e] * c1 + o2 * c2;
        }
        m[g] = mn;
      }
    }
    lds_barrier();                      // merge area free (previous item fully consumed)
    if (slot == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float *w = mo + ((size_t)wv * G + g) * (hd + 2);
#pragma unroll
        for (int e = 0; e < EPL; ++e) w[2 + dl * EPL + e] = o[g][e];
        if (dl == 0) { w[0] = m[g]; w[1] = ls[g]; }
      }
    }
    lds_barrier();
    // wavefronts -> one partial per (kv head, split, g), fixed order
    for (int idx = threadIdx.x; idx < G * hd; idx += blockDim.x) {
      const int g = idx / hd, e = idx % hd;
      float M = NEG;
      for (int w = 0; w < nw; ++w) M = fmaxf(M, mo[((size_t)w * G + g) * (hd + 2)]);
      float Lsum = 0.f, O = 0.f;
      for (int w = 0; w < nw; ++w) {
        const float *src = mo + ((size_t)w * G + g) * (hd + 2);
        const float c = (src[0] == NEG) ? 0.f : expf(src[0] - M);
        Lsum += src[1] * c;
        O += src[2 + e] * c;
      }
      const size_t pi = ((size_t)vh * kMaxSplits + sp) * G + g;
      pub(D.part_o + pi * hd + e, O);
      if (e == 0) { pub(D.part_ml + pi * 2, M); pub(D.part_ml + pi * 2 + 1, Lsum); }
    }
    // splits -> final output, by whichever workgroup of this kv head finishes last
    if (last_arriver(&D.st->attn_cnt[vh], (unsigned)S, lds_flag(D, lds))) {
      for (int idx = threadIdx.x; idx < G * hd; idx += blockDim.x) {
        const int g = idx / hd, e = idx % hd;
        const size_t p_base = ((size_t)vh * kMaxSplits) * G + g;
        float M = NEG;
        for (int s2 = 0; s2 < S; ++s2) M = fmaxf(M, sub(D.part_ml + (p_base + (size_t)s2 * G) * 2));
        float Lsum = 0.f, O = 0.f;
        for (int s2 = 0; s2 < S; ++s2) {
          const size_t pi = p_base + (size_t)s2 * G;
          const float pm = sub(D.part_ml + pi * 2), pl = sub(D.part_ml + pi * 2 + 1);
          const float c = (pm == NEG) ? 0.f : expf(pm - M);
          Lsum += pl * c;
          O += sub(D.part_o + pi * hd + e) * c;
        }
        pub(D.obuf + (vh * G + g) * hd + e, O / Lsum);
      }
    }
  }
}

template <int DT>
__device__ __forceinline__ void phase_attn(const Dev &D, const StepArgs &A, int l, float *lds) {
  switch (D.nq / D.nkv) {
    case 1: attn_items<DT, 1>(D, A, l, lds); break;
    case 2: attn_items<DT, 2>(D, A, l, lds); break;
    default: attn_items<DT, 4>(D, A, l, lds); break;   // 4, or a multiple of 4 in passes
  }
}

// a4: h1 = h + W_o o
template <int DT>
__device__ __forceinline__ void phase_oproj(const Dev &D, const StepArgs &A, int l, bool river, float *lds, Regs<DT> &pre) {
  stage_copy(D.obuf, D.nq * D.hd, lds);
  const float *hin = D.hidden + (size_t)l * D.d;
  const int lane = threadIdx.x & 63;
  auto epi = [&](int k, float a, float b) {
    if (lane < 2) {
      const int r = 2 * k + lane;
      pub(D.h1 + r, sub(hin + r) + (lane ? b : a));
    }
  };
  run_phase<DT>(D, l, PH_O, river, lds, pre, epi);
}

// a5: y = RMSNorm(h1) * g2; a = silu(W_g y) * (W_u y)
template <int DT>
__device__ __forceinline__ void phase_gateup(const Dev &D, const StepArgs &A, int l, bool river, float *lds, Regs<DT> &pre) {
  stage_norm<DT>(D.h1, D.layers[l].ffn_norm, D.d, D.eps, lds, lds_red(D, lds));
  const int lane = threadIdx.x & 63;
  auto epi = [&](int r, float g, float u) {
    if (lane == 0) pub(D.abuf + r, g / (1.0f + expf(-g)) * u);
  };
  run_phase<DT>(D, l, PH_GU, river, lds, pre, epi);
}

// a6: h2 = h1 + W_d a, published as h(l+1); on backbone blocks also the three sums of
// Eq. 1's similarity <h,h2>, <h,h>, <h2,h2> reduced over this workgroup's rows.  The
// reduction over workgroups and the exit decision are taken by every workgroup at the
// start of the next block (exit_test), so no workgroup waits for another here.
template <int DT>
__device__ __forceinline__ void phase_down(const Dev &D, const StepArgs &A, int l, bool river, float *lds, Regs<DT> &pre) {
  stage_copy(D.abuf, D.ffn, lds);
  const float *hin = D.hidden + (size_t)l * D.d;
  float *hout = D.hidden + (size_t)(l + 1) * D.d;
  const int lane = threadIdx.x & 63;
  float ab = 0.f, aa = 0.f, bb = 0.f;
  auto epi = [&](int k, float a, float b) {
    if (lane < 2) {
      const int r = 2 * k + lane;
      const float h0 = sub(hin + r);
      const float h2 = sub(D.h1 + r) + (lane ? b : a);
      pub(hout + r, h2);
      ab = fmaf(h0, h2, ab); aa = fmaf(h0, h0, aa); bb = fmaf(h2, h2, bb);
    }
  };
  run_phase<DT>(D, l, PH_DOWN, river, lds, pre, epi);
  if (river) return;                    // river blocks take no exit test
  float *red = lds_red(D, lds);
  ab = block_sum(ab, red); aa = block_sum(aa, red); bb = block_sum(bb, red);
  if (threadIdx.x == 0) {
    pub(D.cos_part + blockIdx.x * 4 + 0, ab);
    pub(D.cos_part + blockIdx.x * 4 + 1, aa);
    pub(D.cos_part + blockIdx.x * 4 + 2, bb);
  }
}

// a9 + a10: logits = W_head RMSNorm(h(L)) * g_f; greedy token (lowest index on ties);
// the step's record.
template <int DT>
__device__ __forceinline__ void head_rows(const Dev &D, int t, Rows<kRD> &rw) {
#pragma unroll
  for (int r = 0; r < kRD; ++r) {
    rw.p[r] = (const char *)D.lm_head +
              (size_t)min(t * kRD + r, D.vocab - 1) * D.d * sizeof(typename Store<DT>::T);
    rw.sz[r] = nullptr;
  }
}
template <int DT>
__device__ __forceinline__ void prefetch_head(const Dev &D, Regs<DT> &g) {
  const int t = wave_id();
  if (t < (D.vocab + kRD - 1) / kRD) {
    Rows<kRD> rw;
    head_rows<DT>(D, t, rw);
    Dense<DT, kRD>::issue(g, rw, D.d, D.group, 0);
  }
}
template <int DT>
__device__ __forceinline__ void phase_head(const Dev &D, const StepArgs &A, const Ctl &ctl, float *lds, Regs<DT> &pre) {
  float *red = lds_red(D, lds);
  if (!ctl.river && A.rec_slot >= 0) {      // similarity of the last backbone block: recorded, never tested
    const float s = similarity_from_partials(D, red);
    if (blockIdx.x == 0 && threadIdx.x == 0) D.rec_sims[(size_t)A.rec_slot * D.L + (D.L - 1)] = s;
  }
  stage_norm<DT>(D.hidden + (size_t)D.L * D.d, D.final_norm, D.d, D.eps, lds, red);
  const int lane = threadIdx.x & 63;
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
  stream_tasks<Dense<DT, kRD>, DT, kRD>((D.vocab + kRD - 1) / kRD, D.d, D.group, lds, pre, rows_of, epi);
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
__device__ __forceinline__ Ctl ctl_init(const Dev &D, const StepArgs &A) {
  Ctl c;
  c.river = (A.forced_e == 0);
  c.exit_pos = c.river ? 0 : D.L;
  return c;
}

// NaN in the record for blocks that run as river twins (no similarity there).
__device__ __forceinline__ void record_init(const Dev &D, const StepArgs &A) {
  if (blockIdx.x == 0 && A.rec_slot >= 0)
    for (int i = threadIdx.x; i < D.L; i += blockDim.x)
      D.rec_sims[(size_t)A.rec_slot * D.L + i] = __uint_as_float(0x7fc00000u);
}

}  // namespace river
