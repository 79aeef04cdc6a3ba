// Device code of the early-exit decode step for gfx950 (CDNA4, 64-wide wavefronts).
//
// One decode step is a fixed sequence of phases (River-LLM method section,
// "Inference with Seamless Exit"): embedding, then per block RMSNorm+QKV+RoPE+
// KV write, split-K GQA attention, O-proj + residual, RMSNorm + gate/up + SwiGLU,
// down-proj + residual + the Eq. 1 similarity and exit decision, and finally the
// original final norm + LM head + argmax.  After a token has exited, the same
// phases run with the block's 4-bit river twin, writing K/V into the same cache
// slot.  Every phase is a __device__ function that strides over its work with
// whatever grid it is given, so the same code serves the one-kernel-per-phase
// mode and the persistent one-kernel-per-token mode.
//
// Weight streaming is HBM-bound at batch 1: a wavefront owns whole rows, each
// lane reads 16 contiguous bytes per load (1 KiB per wavefront load, fully
// coalesced), accumulates in fp32 and the 64 lanes are summed with xor shuffles
// in a fixed order, so results do not depend on timing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace river {

constexpr int kMaxGrid = 1024;     // upper bound on workgroups per launch (partial-result arrays)
constexpr int kMaxSplits = 32;     // split-K factor of decode attention
constexpr int kPosPerSplit = 64;   // positions per split before another split is added
constexpr int kMaxKvHeads = 64;
constexpr int kRecords = 4096;     // ring of per-step records

struct DevLayer {
  const void *attn_norm, *ffn_norm;
  const void *w[7];               // wq wk wv wo w_gate w_up w_down
  const uint8_t *qc[7];           // river codes
  const void *qs[7], *qz[7];      // river scale, zero
};

struct DevState {
  unsigned long long bar_count;   // arrivals at device-wide barriers since creation
  int exited;                     // 1 once the current token left the backbone
  int exit_pos;                   // exit position e of the current token
  int cur_token;                  // token produced by the last head phase
  int error;                      // set when a bounded wait gave up
  unsigned int cos_cnt, head_cnt;
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
  float *h1;                      // [d]
  float *abuf;                    // [ffn]
  float *logits;                  // [vocab]
  float *part_o;                  // [nkv][kMaxSplits][G][hd] unnormalised partial outputs
  float2 *part_ml;                // [nkv][kMaxSplits][G] (running max, sum)
  float *cos_part;                // [kMaxGrid][3]
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
  unsigned long long bar_base;   // DevState::bar_count when this launch starts
};

// ------------------------------------------------------------------ storage

template <int DT> struct Store;   // DT 0: fp32, 1: bf16
template <> struct Store<0> {
  typedef float T;
  static constexpr int EPL = 4;   // elements per 16-byte lane load
  static __device__ __forceinline__ float ld(const void *p, size_t i) { return ((const float *)p)[i]; }
  static __device__ __forceinline__ void st(void *p, size_t i, float v) { ((float *)p)[i] = v; }
  static __device__ __forceinline__ void unpack(const uint4 &w, float (&f)[4]) {
    f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
    f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
  }
};
template <> struct Store<1> {
  typedef uint16_t T;
  static constexpr int EPL = 8;
  static __device__ __forceinline__ float ld(const void *p, size_t i) {
    return __uint_as_float((uint32_t)((const uint16_t *)p)[i] << 16);
  }
  // round-to-nearest-even fp32 -> bf16
  static __device__ __forceinline__ uint16_t rne(float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  }
  static __device__ __forceinline__ void st(void *p, size_t i, float v) { ((uint16_t *)p)[i] = rne(v); }
  static __device__ __forceinline__ void unpack(const uint4 &w, float (&f)[8]) {
    f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
    f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
    f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
    f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
  }
};

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
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
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
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { red[w] = v; redi[w] = i; }
  __syncthreads();
  v = red[0]; i = redi[0];
  for (int k = 1; k < nw; ++k) argmax_take(v, i, red[k], redi[k]);
}

// --------------------------------------------------------- device barrier

// Device-wide barrier of the persistent kernel.  Every workgroup adds one to a
// monotone 64-bit counter (release, agent scope) and polls it (acquire) until
// `target` arrivals are in.  The wait is bounded: after spin_limit polls, or once
// another workgroup has flagged an error, the workgroup flags the error and goes
// on, so every wave reaches the end of the kernel whatever happens.
__device__ __forceinline__ void grid_barrier(DevState *st, unsigned long long target, int spin_limit) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(&st->bar_count, 1ull, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    int spins = 0;
    while (__hip_atomic_load(&st->bar_count, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < target) {
      if (++spins > spin_limit ||
          __hip_atomic_load(&st->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
        __hip_atomic_store(&st->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(2);
    }
  }
  __syncthreads();
}

// "Last workgroup to arrive" ticket: the caller's workgroup has finished writing
// its partial result; returns true in every thread of the one workgroup that
// arrives last among `expected`, after which that workgroup may read all partials.
__device__ __forceinline__ bool last_arriver(unsigned int *cnt, unsigned int expected, int *flag_lds) {
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned int t = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    int last = (t == expected - 1);
    if (last) __hip_atomic_store(cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag_lds = last;
  }
  __syncthreads();
  return *flag_lds != 0;
}

// -------------------------------------------------------------- staging x

// xl[0..n) = h * rsqrt(mean(h^2) + eps) * gain   (fused RMSNorm prologue)
template <int DT>
__device__ __forceinline__ void stage_norm(const float *h, const void *gain, int n, float eps,
                                           float *xl, float *red) {
  float ss = 0.f;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    float v = h[i];
    xl[i] = v;
    ss += v * v;
  }
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)n + eps);
  for (int i = threadIdx.x; i < n; i += blockDim.x) xl[i] = xl[i] * r * Store<DT>::ld(gain, i);
  __syncthreads();
}

__device__ __forceinline__ void stage_copy(const float *src, int n, float *xl) {
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += blockDim.x) xl[i] = src[i];
  __syncthreads();
}

// ------------------------------------------------------------- GEMV cores

// R dot products of dense rows with the vector in LDS, per wavefront.
// rowp[r]: byte pointer to row r (16-byte aligned), cols % EPL == 0.
template <int DT, int R, int U>
__device__ __forceinline__ void wave_gemv(const char *const (&rowp)[R], int cols, const float *xl,
                                          float (&acc)[R]) {
  constexpr int EPL = Store<DT>::EPL;
  constexpr int STEP = 64 * EPL;
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
  for (int c0 = lane * EPL; c0 < cols; c0 += STEP * U) {
    uint4 w[U][R];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = c0 + u * STEP;
#pragma unroll
      for (int r = 0; r < R; ++r)
        w[u][r] = (c < cols) ? *(const uint4 *)(rowp[r] + (size_t)c * sizeof(typename Store<DT>::T))
                             : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = c0 + u * STEP;
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
          Store<DT>::unpack(w[u][r], f);
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[r] = fmaf(f[e], x[e], acc[r]);
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = wave_sum(acc[r]);
}

// Same for river rows: codes are 4-bit, CPL codes per lane load (16: 8-byte load,
// 32: 16-byte load), weight = (code - zero) * scale per group.  Per lane load the
// sum over its columns is factored as scale * (sum code*x - zero * sum x).
// qrow[r]: codes of row r; srow/zrow[r]: scale/zero of row r; cols % CPL == 0,
// group % CPL == 0 so one lane load never straddles a group.
template <int DT, int R, int CPL>
__device__ __forceinline__ void wave_gemv_w4(const uint8_t *const (&qrow)[R],
                                             const void *const (&srow)[R],
                                             const void *const (&zrow)[R], int cols, int group,
                                             const float *xl, float (&acc)[R]) {
  constexpr int NW = CPL / 8;       // 32-bit words of codes per lane load
  constexpr int STEP = 64 * CPL;
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
  for (int c = lane * CPL; c < cols; c += STEP) {
    uint32_t w[R][NW];
    float s[R], z[R];
    const int g = c / group;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if constexpr (NW == 4) {
        const uint4 t = *(const uint4 *)(qrow[r] + (c >> 1));
        w[r][0] = t.x; w[r][1] = t.y; w[r][2] = t.z; w[r][3] = t.w;
      } else {
        const uint2 t = *(const uint2 *)(qrow[r] + (c >> 1));
        w[r][0] = t.x; w[r][1] = t.y;
      }
      s[r] = Store<DT>::ld(srow[r], g);
      z[r] = Store<DT>::ld(zrow[r], g);
    }
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
      float aq = 0.f;
#pragma unroll
      for (int k = 0; k < NW; ++k) {
        const uint32_t v = w[r][k];
        const uint32_t lo = v & 0x0f0f0f0fu, hi = (v >> 4) & 0x0f0f0f0fu;
        // byte j of v holds columns 2j (low nibble) and 2j+1 (high nibble)
        aq = fmaf((float)(lo & 0xffu), x[8 * k + 0], aq);
        aq = fmaf((float)(hi & 0xffu), x[8 * k + 1], aq);
        aq = fmaf((float)((lo >> 8) & 0xffu), x[8 * k + 2], aq);
        aq = fmaf((float)((hi >> 8) & 0xffu), x[8 * k + 3], aq);
        aq = fmaf((float)((lo >> 16) & 0xffu), x[8 * k + 4], aq);
        aq = fmaf((float)((hi >> 16) & 0xffu), x[8 * k + 5], aq);
        aq = fmaf((float)(lo >> 24), x[8 * k + 6], aq);
        aq = fmaf((float)(hi >> 24), x[8 * k + 7], aq);
      }
      acc[r] = fmaf(s[r], aq - z[r] * sx, acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = wave_sum(acc[r]);
}

// R dot products against rows rows[r] of matrices mats[r] of one block, dense
// (backbone) or river twin; all R matrices have `cols` columns.
template <int DT, int R>
__device__ __forceinline__ void rows_dot(const DevLayer &Lw, const int (&mats)[R], bool use_river,
                                         const int (&rows)[R], int cols, int group, const float *xl,
                                         float (&acc)[R]) {
  if (!use_river) {
    const char *rp[R];
#pragma unroll
    for (int r = 0; r < R; ++r)
      rp[r] = (const char *)Lw.w[mats[r]] + (size_t)rows[r] * cols * sizeof(typename Store<DT>::T);
    wave_gemv<DT, R, 2>(rp, cols, xl, acc);
  } else {
    const int gpr = (cols + group - 1) / group;
    const uint8_t *qp[R];
    const void *sp[R], *zp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      qp[r] = Lw.qc[mats[r]] + (size_t)rows[r] * (cols >> 1);
      sp[r] = (const char *)Lw.qs[mats[r]] + (size_t)rows[r] * gpr * sizeof(typename Store<DT>::T);
      zp[r] = (const char *)Lw.qz[mats[r]] + (size_t)rows[r] * gpr * sizeof(typename Store<DT>::T);
    }
    if ((cols & 31) == 0) wave_gemv_w4<DT, R, 32>(qp, sp, zp, cols, group, xl, acc);
    else wave_gemv_w4<DT, R, 16>(qp, sp, zp, cols, group, xl, acc);
  }
}

// ------------------------------------------------------------------ phases

// a0: h(0) = E[token]; reset the per-token exit state and this step's record.
template <int DT>
__device__ void phase_embed(const Dev &D, const StepArgs &A) {
  int tok = A.token >= 0 ? A.token : D.st->cur_token;
  tok = min(max(tok, 0), D.vocab - 1);       // a NaN-poisoned argmax must not index out of range
  const int n = gridDim.x * blockDim.x;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < D.d; i += n)
    D.hidden[i] = Store<DT>::ld(D.tok_emb, (size_t)tok * D.d + i);
  if (blockIdx.x == 0) {
    if (threadIdx.x == 0) {
      D.st->exited = (A.forced_e == 0);
      D.st->exit_pos = (A.forced_e == 0) ? 0 : D.L;
    }
    if (A.rec_slot >= 0)
      for (int i = threadIdx.x; i < D.L; i += blockDim.x)
        D.rec_sims[(size_t)A.rec_slot * D.L + i] = __uint_as_float(0x7fc00000u);
  }
}

// LDS layout of every phase: [0, xcap) staged vector (or the attention merge area),
// [xcap, xcap+32) reduction scratch, [xcap+32] last-arriver flag.
__device__ __forceinline__ float *lds_red(const Dev &D, float *lds) { return lds + D.xcap; }
__device__ __forceinline__ int *lds_flag(const Dev &D, float *lds) { return (int *)(lds + D.xcap + 32); }

__device__ __forceinline__ int wave_id() { return blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6); }
__device__ __forceinline__ int wave_count() { return gridDim.x * (blockDim.x >> 6); }

// a1 + a2: x = RMSNorm(h) * g1; [q;k;v] = W x; RoPE on q, k at this position; k, v rounded
// to the cache dtype and stored in slot (l, pos) -- the same slot for backbone and river
// ("identical KV Cache addressing scheme").  A wavefront owns two rotation pairs
// (rows i and i + hd/2 of a head) at a time, so the rotation needs no exchange.
template <int DT>
__device__ void phase_qkv(const Dev &D, const StepArgs &A, int l, float *lds) {
  const DevLayer &Lw = D.layers[l];
  const bool rv = D.st->exited != 0;
  float *xl = lds;
  stage_norm<DT>(D.hidden + (size_t)l * D.d, Lw.attn_norm, D.d, D.eps, xl, lds_red(D, lds));
  const int half = D.hd >> 1;
  const int heads = D.nq + 2 * D.nkv;
  const int units = heads * half;            // rotation pairs (v rows are paired the same way)
  const int kvd = D.nkv * D.hd;
  const int lane = threadIdx.x & 63;
  for (int u0 = wave_id() * 2; u0 < units; u0 += wave_count() * 2) {
    // both pairs of a task lie in the same head because half is even
    const int head = u0 / half, i0 = u0 % half;
    int m, hh;                                // matrix index and head within it
    if (head < D.nq) { m = 0; hh = head; }
    else if (head < D.nq + D.nkv) { m = 1; hh = head - D.nq; }
    else { m = 2; hh = head - D.nq - D.nkv; }
    const int rows[4] = {hh * D.hd + i0, hh * D.hd + i0 + half, hh * D.hd + i0 + 1,
                         hh * D.hd + i0 + 1 + half};
    const int mats[4] = {m, m, m, m};
    float acc[4];
    rows_dot<DT, 4>(Lw, mats, rv, rows, D.d, D.group, xl, acc);
    if (lane < 2) {
      const int i = i0 + lane;
      float a = lane ? acc[2] : acc[0], b = lane ? acc[3] : acc[1];
      if (m < 2) {
        const float2 cs = D.rope[(size_t)A.pos * half + i];
        const float ra = a * cs.x - b * cs.y, rb = a * cs.y + b * cs.x;
        a = ra; b = rb;
      }
      if (m == 0) {
        D.qbuf[hh * D.hd + i] = a;
        D.qbuf[hh * D.hd + i + half] = b;
      } else {
        void *cache = (m == 1) ? D.kcache : D.vcache;
        const size_t base = ((size_t)l * D.max_seq + A.pos) * kvd + (size_t)hh * D.hd;
        Store<DT>::st(cache, base + i, a);
        Store<DT>::st(cache, base + i + half, b);
      }
    }
  }
}

// a3: split-K GQA decode attention.  A workgroup owns (kv head, split): its wavefronts
// stream that split's K and V rows once (16 bytes per lane, hd/EPL lanes per position)
// and serve all G query heads of the group from registers, with an online softmax per
// lane group.  Partials (max, sum, unnormalised output) are merged in a fixed order:
// lane groups, wavefronts (through LDS), then splits (by the last workgroup of the kv
// head to arrive), so the result is independent of timing.
template <int DT, int G>
__device__ void attn_items(const Dev &D, const StepArgs &A, int l, float *lds) {
  constexpr int EPL = Store<DT>::EPL;
  const int hd = D.hd, LPP = hd / EPL, PPW = 64 / LPP;
  const int S = A.n_splits, T = A.pos + 1;
  const int chunk = (T + S - 1) / S;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int slot = lane / LPP, dl = lane % LPP;
  const int kvd = D.nkv * hd;
  const float inv = 1.0f / sqrtf((float)hd);
  const float NEG = -INFINITY;
  // LDS merge area: per wavefront G * (hd + 2) floats
  float *mo = lds;
  for (int item = blockIdx.x; item < D.nkv * S; item += gridDim.x) {
    const int kvh = item / S, sp = item % S;
    const int p0 = sp * chunk, p1 = min(T, p0 + chunk);
    float q[G][EPL], o[G][EPL], m[G], ls[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = NEG; ls[g] = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        q[g][e] = D.qbuf[(kvh * G + g) * hd + dl * EPL + e] * inv;
        o[g][e] = 0.f;
      }
    }
    const char *Kb = (const char *)D.kcache + ((size_t)l * D.max_seq * kvd + (size_t)kvh * hd + dl * EPL) * sizeof(typename Store<DT>::T);
    const char *Vb = (const char *)D.vcache + ((size_t)l * D.max_seq * kvd + (size_t)kvh * hd + dl * EPL) * sizeof(typename Store<DT>::T);
    for (int pb = p0 + wv * PPW; pb < p1; pb += nw * PPW) {
      const int p = pb + slot;
      const bool ok = p < p1;
      const size_t off = (size_t)(ok ? p : p0) * kvd * sizeof(typename Store<DT>::T);
      const uint4 kw = *(const uint4 *)(Kb + off);
      const uint4 vw = *(const uint4 *)(Vb + off);
      float kf[EPL], vf[EPL];
      Store<DT>::unpack(kw, kf);
      Store<DT>::unpack(vw, vf);
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
    __syncthreads();                      // merge area free (previous item fully consumed)
    if (slot == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float *w = mo + ((size_t)wv * G + g) * (hd + 2);
#pragma unroll
        for (int e = 0; e < EPL; ++e) w[2 + dl * EPL + e] = o[g][e];
        if (dl == 0) { w[0] = m[g]; w[1] = ls[g]; }
      }
    }
    __syncthreads();
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
      const size_t pi = ((size_t)kvh * kMaxSplits + sp) * G + g;
      D.part_o[pi * hd + e] = O;
      if (e == 0) D.part_ml[pi] = make_float2(M, Lsum);
    }
    // splits -> final output, by whichever workgroup of this kv head finishes last
    if (last_arriver(&D.st->attn_cnt[kvh], (unsigned)S, lds_flag(D, lds))) {
      for (int idx = threadIdx.x; idx < G * hd; idx += blockDim.x) {
        const int g = idx / hd, e = idx % hd;
        const size_t p_base = ((size_t)kvh * kMaxSplits) * G + g;
        float M = NEG;
        for (int s2 = 0; s2 < S; ++s2) M = fmaxf(M, D.part_ml[p_base + (size_t)s2 * G].x);
        float Lsum = 0.f, O = 0.f;
        for (int s2 = 0; s2 < S; ++s2) {
          const float2 ml = D.part_ml[p_base + (size_t)s2 * G];
          const float c = (ml.x == NEG) ? 0.f : expf(ml.x - M);
          Lsum += ml.y * c;
          O += D.part_o[(p_base + (size_t)s2 * G) * hd + e] * c;
        }
        D.obuf[(kvh * G + g) * hd + e] = O / Lsum;
      }
    }
  }
}

template <int DT>
__device__ void phase_attn(const Dev &D, const StepArgs &A, int l, float *lds) {
  switch (D.nq / D.nkv) {
    case 1: attn_items<DT, 1>(D, A, l, lds); break;
    case 2: attn_items<DT, 2>(D, A, l, lds); break;
    case 4: attn_items<DT, 4>(D, A, l, lds); break;
    default: attn_items<DT, 8>(D, A, l, lds); break;
  }
}

// a4: h1 = h + W_o o
template <int DT>
__device__ void phase_oproj(const Dev &D, const StepArgs &A, int l, float *lds) {
  const DevLayer &Lw = D.layers[l];
  const bool rv = D.st->exited != 0;
  const int n = D.nq * D.hd;
  stage_copy(D.obuf, n, lds);
  const float *hin = D.hidden + (size_t)l * D.d;
  const int lane = threadIdx.x & 63;
  for (int r0 = wave_id() * 4; r0 < D.d; r0 += wave_count() * 4) {
    const int rows[4] = {r0, r0 + 1, r0 + 2, r0 + 3};
    const int mats[4] = {3, 3, 3, 3};
    float acc[4];
    rows_dot<DT, 4>(Lw, mats, rv, rows, n, D.group, lds, acc);
    if (lane < 4) {
      const float v = lane == 0 ? acc[0] : lane == 1 ? acc[1] : lane == 2 ? acc[2] : acc[3];
      D.h1[r0 + lane] = hin[r0 + lane] + v;
    }
  }
}

// a5: y = RMSNorm(h1) * g2; a = silu(W_g y) * (W_u y)
template <int DT>
__device__ void phase_gateup(const Dev &D, const StepArgs &A, int l, float *lds) {
  const DevLayer &Lw = D.layers[l];
  const bool rv = D.st->exited != 0;
  stage_norm<DT>(D.h1, Lw.ffn_norm, D.d, D.eps, lds, lds_red(D, lds));
  const int lane = threadIdx.x & 63;
  for (int r0 = wave_id() * 2; r0 < D.ffn; r0 += wave_count() * 2) {
    const int rows[4] = {r0, r0, r0 + 1, r0 + 1};
    const int mats[4] = {4, 5, 4, 5};
    float acc[4];
    rows_dot<DT, 4>(Lw, mats, rv, rows, D.d, D.group, lds, acc);
    if (lane < 2) {
      const float gv = lane ? acc[2] : acc[0], uv = lane ? acc[3] : acc[1];
      D.abuf[r0 + lane] = gv / (1.0f + expf(-gv)) * uv;
    }
  }
}

// a6: h2 = h1 + W_d a, stored as h(l+1); on backbone blocks also the three sums of
// Eq. 1's similarity, reduced per workgroup, then over workgroups by the last one to
// arrive, which takes the exit decision for block l+1 (1-based) and publishes it in
// DevState for the next block's kernels to pick backbone or river weights.
template <int DT>
__device__ void phase_down(const Dev &D, const StepArgs &A, int l, float *lds) {
  const DevLayer &Lw = D.layers[l];
  const bool rv = D.st->exited != 0;
  stage_copy(D.abuf, D.ffn, lds);
  const float *hin = D.hidden + (size_t)l * D.d;
  float *hout = D.hidden + (size_t)(l + 1) * D.d;
  const int lane = threadIdx.x & 63;
  float ab = 0.f, aa = 0.f, bb = 0.f;
  for (int r0 = wave_id() * 4; r0 < D.d; r0 += wave_count() * 4) {
    const int rows[4] = {r0, r0 + 1, r0 + 2, r0 + 3};
    const int mats[4] = {6, 6, 6, 6};
    float acc[4];
    rows_dot<DT, 4>(Lw, mats, rv, rows, D.ffn, D.group, lds, acc);
    if (lane < 4) {
      const float v = lane == 0 ? acc[0] : lane == 1 ? acc[1] : lane == 2 ? acc[2] : acc[3];
      const float h0 = hin[r0 + lane];
      const float h2 = D.h1[r0 + lane] + v;
      hout[r0 + lane] = h2;
      ab = fmaf(h0, h2, ab); aa = fmaf(h0, h0, aa); bb = fmaf(h2, h2, bb);
    }
  }
  if (rv) return;                       // river blocks take no exit test
  float *red = lds_red(D, lds);
  ab = block_sum(ab, red); aa = block_sum(aa, red); bb = block_sum(bb, red);
  if (threadIdx.x == 0) {
    D.cos_part[blockIdx.x * 3 + 0] = ab;
    D.cos_part[blockIdx.x * 3 + 1] = aa;
    D.cos_part[blockIdx.x * 3 + 2] = bb;
  }
  if (last_arriver(&D.st->cos_cnt, gridDim.x, lds_flag(D, lds))) {
    float pab = 0.f, paa = 0.f, pbb = 0.f;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += blockDim.x) {
      pab += D.cos_part[i * 3 + 0]; paa += D.cos_part[i * 3 + 1]; pbb += D.cos_part[i * 3 + 2];
    }
    pab = block_sum(pab, red); paa = block_sum(paa, red); pbb = block_sum(pbb, red);
    if (threadIdx.x == 0) {
      float s = 0.f;
      if (paa > 0.f && pbb > 0.f) {
        s = pab / (sqrtf(paa) * sqrtf(pbb));
        s = fminf(1.0f, fmaxf(-1.0f, s));
      }
      const int l1 = l + 1;
      if (A.rec_slot >= 0) D.rec_sims[(size_t)A.rec_slot * D.L + l] = s;
      if (l1 >= D.min_exit && l1 < D.L &&
          ((A.forced_e < 0 && s > D.tau) || A.forced_e == l1)) {
        D.st->exited = 1;
        D.st->exit_pos = l1;
      }
    }
  }
}

// a9 + a10: logits = W_head RMSNorm(h(L)) * g_f; greedy token (lowest index on ties);
// the step's record.
template <int DT>
__device__ void phase_head(const Dev &D, const StepArgs &A, float *lds) {
  stage_norm<DT>(D.hidden + (size_t)D.L * D.d, D.final_norm, D.d, D.eps, lds, lds_red(D, lds));
  const int lane = threadIdx.x & 63;
  float best = -INFINITY;
  int besti = 0x7fffffff;
  for (int r0 = wave_id() * 4; r0 < D.vocab; r0 += wave_count() * 4) {
    const char *rp[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
      rp[r] = (const char *)D.lm_head +
              (size_t)min(r0 + r, D.vocab - 1) * D.d * sizeof(typename Store<DT>::T);
    float acc[4];
    wave_gemv<DT, 4, 2>(rp, D.d, lds, acc);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (r0 + r < D.vocab) {
        if (lane == 0) D.logits[r0 + r] = acc[r];
        if (acc[r] > best) { best = acc[r]; besti = r0 + r; }   // rows ascend: first maximum kept
      }
    }
  }
  float *red = lds_red(D, lds);
  block_argmax(best, besti, red);
  if (threadIdx.x == 0) {
    D.amax_val[blockIdx.x] = best;
    D.amax_idx[blockIdx.x] = besti;
  }
  if (last_arriver(&D.st->head_cnt, gridDim.x, lds_flag(D, lds))) {
    float b = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += blockDim.x)
      argmax_take(b, bi, D.amax_val[i], D.amax_idx[i]);
    block_argmax(b, bi, red);
    if (threadIdx.x == 0) {
      D.st->cur_token = bi;
      if (A.rec_slot >= 0) {
        D.rec_token[A.rec_slot] = bi;
        D.rec_exit[A.rec_slot] = D.st->exit_pos;
      }
    }
  }
}

}  // namespace river
