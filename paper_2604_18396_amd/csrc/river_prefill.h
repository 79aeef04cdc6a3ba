// Prefill phase with sequence-level exit (River-LLM method section, "Inference with Seamless
// Exit", list of phases): the whole prompt is processed at one unified depth e_p, blocks
// 1..e_p with the backbone matrices, blocks e_p+1..L with their 4-bit river twins, every
// block writing K/V of every prompt position into the shared cache slot.  Unlike a decode
// step this is dense matrix-matrix work, so it runs on the matrix cores: the prompt is cut
// into chunks of up to kChunk tokens and each block is a sequence of MFMA GEMMs over the
// chunk (fp16 operands, fp32 accumulation) with small element-wise kernels between them:
//
//   embed -> [ rmsnorm -> GEMM(Wq;Wk;Wv) -> rope + cache store -> causal attention
//              -> GEMM(Wo) += h -> rmsnorm -> GEMM(Wg;Wu) -> swiglu -> GEMM(Wd) += h1 ] x L
//
// Operand types: activations are rounded to half precision (fp16) when they enter a GEMM or
// the attention; backbone weights (bf16) are converted to fp16 while a tile is staged in LDS
// (exact but for magnitudes below 2^-14); river weights are dequantised, (code - zero) * scale
// in fp32, and rounded to fp16 while staged; cached K/V (bf16) are converted the same way.
// The residual stream stays fp32 in HBM.  Only bf16 models take this path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "river_device.h"

namespace river {
namespace pf {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kChunk = 1024;          // prompt tokens per pass (rows of the activation buffers)
constexpr int TM = 128, TN = 128, TK = 64;
constexpr int LDK = TK + 8;           // LDS row stride in halfs: 144 B, rows 4 banks apart
constexpr int kGemmLdsBytes = 2 * (TM + TN) * LDK * 2;     // k_pf_gemm: two buffers each of the A and B tiles

// v_mfma_f32_32x32x16_f16: D[32x32] += A[32x16] B[16x32].  Lane l supplies row l % 32 of A and
// column l % 32 of B, eight K values each (those of lane group l / 32; which eight is the same
// for A and B, so any fixed assignment gives the right sum).  D: register r of lane l is
// row (r / 4) * 8 + (l / 32) * 4 + r % 4, column l % 32.
__device__ __forceinline__ f32x16 mfma16(half8 a, half8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ int c_row(int r, int lane) { return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// eight bf16 values (16 bytes) -> eight fp16 values
__device__ __forceinline__ half8 bf16x8_to_half8(const uint4 &w) {
  half8 h;
  h[0] = (_Float16)bf16_lo(w.x); h[1] = (_Float16)bf16_hi(w.x);
  h[2] = (_Float16)bf16_lo(w.y); h[3] = (_Float16)bf16_hi(w.y);
  h[4] = (_Float16)bf16_lo(w.z); h[5] = (_Float16)bf16_hi(w.z);
  h[6] = (_Float16)bf16_lo(w.w); h[7] = (_Float16)bf16_hi(w.w);
  return h;
}

// A 16-bit KV cache holds bf16 values, or IEEE half values when the context keeps its cache in
// FP16 (kv_f16): store one element / fetch eight as fp16 / fetch one as fp32.
__device__ __forceinline__ void cache_store(void *cache, size_t i, float v, int kv_f16) {
  if (kv_f16) ((_Float16 *)cache)[i] = (_Float16)v;
  else Store<1>::st(cache, i, v);
}
__device__ __forceinline__ half8 cache_half8(const uint4 &w, int kv_f16) {
  return kv_f16 ? __builtin_bit_cast(half8, w) : bf16x8_to_half8(w);
}
__device__ __forceinline__ float cache_lo(uint32_t w, int kv_f16) {
  return kv_f16 ? (float)__builtin_bit_cast(half2v, w)[0] : bf16_lo(w);
}
__device__ __forceinline__ float cache_hi(uint32_t w, int kv_f16) {
  return kv_f16 ? (float)__builtin_bit_cast(half2v, w)[1] : bf16_hi(w);
}

// ------------------------------------------------------------------ GEMM
//
// C[M, N] (+)= A[M, K] B^T, B = up to three matrices stacked along N (rows of W_q, W_k, W_v;
// of W_gate, W_up), each [rows, K] row-major: dense bf16, or 4-bit codes with one packed
// (scale, zero) pair per (row, group of `group` columns).  One workgroup of four wavefronts
// per 128 x 128 tile of C, each wavefront a 64 x 64 quarter (2 x 2 MFMA blocks); K in tiles of
// 64 staged through LDS, the next tile's global loads in flight while the current one is
// multiplied.  M must be a multiple of 128 (the activation buffers are; rows beyond the
// prompt hold don't-care values); N is guarded; K % 64 == 0, group % 64 == 0.
struct GemmB {
  const void *w[3];
  const void *sz[3];
  int rows[3];
};

__device__ __forceinline__ void gemm_b_row(const GemmB &B, int n, int N, int &mat, int &row) {
  n = min(n, N - 1);
  mat = 0;
  if (n >= B.rows[0]) { n -= B.rows[0]; mat = 1; }
  if (mat == 1 && n >= B.rows[1]) { n -= B.rows[1]; mat = 2; }
  row = n;
}

template <bool W4, bool ADD>
__global__ __launch_bounds__(256, 2) void k_pf_gemm(const _Float16 *__restrict__ A, int lda, GemmB B, int N, int K,
                                                 int group, float *C, int ldc, int m_tiles) {
  extern __shared__ __attribute__((aligned(16))) _Float16 pf_lds[];   // kGemmLdsBytes: two buffers each of A and B
  _Float16 *const As = pf_lds, *const Bs = pf_lds + 2 * TM * LDK;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  // Workgroup -> tile of C.  Consecutive workgroup ids go round the 8 XCDs; the workgroups of one
  // XCD take all M tiles of a column of N tiles before the next column, so the workgroups resident
  // on an XCD at a time cover all M tiles of a few N tiles: a B tile is fetched from HBM once (its
  // XCD's L2 serves the other M tiles) and the A tiles stay in every L2.
  // (one-dimensional grid of 8 * ceil(N tiles / 8) * m_tiles workgroups)
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int n_tile = (j / m_tiles) * 8 + xcd, m_tile = j % m_tiles;
  if (n_tile * TN >= N) return;
  const int m0 = m_tile * TM, n0 = n_tile * TN;
  const int wm = wv >> 1, wn = wv & 1;

  // what this thread stages per K tile: four 16-byte segments of A; of B four 16-byte
  // segments (dense) or one 16-byte run of 32 codes with its (scale, zero) pair (river)
  const char *a_src[4];
  int a_dst[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int seg = tid + 256 * i, row = seg >> 3, ks = seg & 7;
    a_src[i] = (const char *)(A + (size_t)(m0 + row) * lda + ks * 8);
    a_dst[i] = row * LDK + ks * 8;
  }
  const char *b_src[W4 ? 1 : 4];
  const char *b_sz = nullptr;
  int b_dst[W4 ? 1 : 4];
  if constexpr (W4) {
    const int row = tid >> 1, hf = tid & 1;
    int mat, r;
    gemm_b_row(B, n0 + row, N, mat, r);
    b_src[0] = (const char *)B.w[mat] + (size_t)r * (K >> 1) + hf * 16;
    b_sz = (const char *)B.sz[mat] + (size_t)r * (K / group) * 4;
    b_dst[0] = row * LDK + hf * 32;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int seg = tid + 256 * i, row = seg >> 3, ks = seg & 7;
      int mat, r;
      gemm_b_row(B, n0 + row, N, mat, r);
      b_src[i] = (const char *)B.w[mat] + ((size_t)r * K + ks * 8) * 2;
      b_dst[i] = row * LDK + ks * 8;
    }
  }

  // a K tile on its way from global memory to LDS
  u32x4 fa[4], fb[W4 ? 1 : 4];                  // (native vectors: as structs they are kept in scratch memory)
  uint32_t fsz = 0;
  const int nk = K / TK;
  auto load = [&](int kt) {
    const int k0 = kt * TK;
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = *(const u32x4 *)(a_src[i] + (size_t)k0 * 2);
    if constexpr (W4) {
      fb[0] = *(const u32x4 *)(b_src[0] + (k0 >> 1));
      fsz = *(const uint32_t *)(b_sz + (size_t)(k0 / group) * 4);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) fb[i] = *(const u32x4 *)(b_src[i] + (size_t)k0 * 2);
    }
  };
  auto stage = [&](int buf) {
    _Float16 *const As = pf_lds + buf * TM * LDK, *const Bs = pf_lds + 2 * TM * LDK + buf * TN * LDK;
#pragma unroll
    for (int i = 0; i < 4; ++i) *(u32x4 *)(As + a_dst[i]) = fa[i];
    if constexpr (W4) {
      // weight = (code - zero) * scale in fp32, then fp16; byte j of the run holds column 2j
      // in its low nibble and column 2j + 1 in its high nibble
      const float s = bf16_lo(fsz), z = bf16_hi(fsz);
      const uint32_t wds[4] = {fb[0].x, fb[0].y, fb[0].z, fb[0].w};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        half8 h;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const uint32_t byte = (wds[w] >> (8 * b)) & 0xffu;
          h[2 * b] = (_Float16)(((float)(byte & 15u) - z) * s);
          h[2 * b + 1] = (_Float16)(((float)(byte >> 4) - z) * s);
        }
        *(half8 *)(Bs + b_dst[0] + w * 8) = h;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) *(half8 *)(Bs + b_dst[i]) = bf16x8_to_half8(make_uint4(fb[i].x, fb[i].y, fb[i].z, fb[i].w));
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int r32 = lane & 31, g8 = (lane >> 5) * 8;
  // Tile kt is multiplied from LDS buffer kt % 2 while tile kt + 1 (fetched during the previous
  // iteration) is written into the other buffer and tile kt + 2 is fetched: one workgroup barrier
  // per K tile.
  load(0);
  stage(0);
  if (nk > 1) load(1);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) stage(cur ^ 1);
    if (kt + 2 < nk) load(kt + 2);
    const _Float16 *const Ac = As + cur * TM * LDK, *const Bc = Bs + cur * TN * LDK;
#pragma unroll
    for (int ks = 0; ks < TK / 16; ++ks) {
      half8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = *(const half8 *)(Ac + (wm * 64 + i * 32 + r32) * LDK + ks * 16 + g8);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = *(const half8 *)(Bc + (wn * 64 + j * 32 + r32) * LDK + ks * 16 + g8);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma16(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn * 64 + j * 32 + r32;
      if (col < N) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float *p = C + (size_t)(m0 + wm * 64 + i * 32 + c_row(r, lane)) * ldc + col;
          if constexpr (ADD) *p += acc[i][j][r];
          else *p = acc[i][j][r];
        }
      }
    }
}

// ------------------------------------------------------- element-wise kernels

// h[t, :] = E[token[t], :] for the m tokens of the chunk; one workgroup per token
__global__ void k_pf_embed(const int *__restrict__ tokens, const void *tok_emb, int d, float *h) {
  const int t = blockIdx.x;
  const size_t src = (size_t)tokens[t] * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)t * d + i] = Store<1>::ld(tok_emb, src + i);
}

// x16[t, :] = fp16(h[t, :] * rsqrt(mean(h[t, :]^2) + eps) * gain); one workgroup (256) per token
__global__ __launch_bounds__(256) void k_pf_rmsnorm(const float *__restrict__ h, const void *gain, int d, float eps,
                                                    _Float16 *x16) {
  __shared__ float red[16];
  const int t = blockIdx.x;
  const float *row = h + (size_t)t * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += blockDim.x) ss += row[i] * row[i];
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += blockDim.x)
    x16[(size_t)t * d + i] = (_Float16)(row[i] * r * Store<1>::ld(gain, i));
}

// RoPE on q and k at position pos0 + t; q scaled by log2(e) / sqrt(hd) and stored as fp16 for
// the attention kernel; k (rotated) and v rounded to the cache dtype and written to slot
// (l, pos0 + t) of the shared cache.  qkv: fp32 [m, qd + 2 kvd] as the QKV GEMM left it.
// One workgroup per token; thread i handles rotation pair (i, i + hd/2) of one head.
__global__ void k_pf_rope_store(const float *__restrict__ qkv, const float2 *__restrict__ rope, int nq, int nkv,
                                int hd, int pos0, int l, int max_seq, void *kcache, void *vcache, int kv_f16,
                                _Float16 *q16) {
  const int t = blockIdx.x, p = pos0 + t, half = hd >> 1;
  const int qd = nq * hd, kvd = nkv * hd, ld = qd + 2 * kvd;
  const float *row = qkv + (size_t)t * ld;
  const float qs = 1.4426950408889634f / sqrtf((float)hd);
  for (int i = threadIdx.x; i < (nq + nkv) * half; i += blockDim.x) {
    const int head = i / half, e = i % half;
    const float2 cs = rope[(size_t)p * half + e];
    const float *src = row + head * hd;            // q heads, then k heads: contiguous in qkv
    const float a = src[e], b = src[e + half];
    const float lo = a * cs.x - b * cs.y, hi = a * cs.y + b * cs.x;
    if (head < nq) {
      q16[(size_t)t * qd + head * hd + e] = (_Float16)(lo * qs);
      q16[(size_t)t * qd + head * hd + e + half] = (_Float16)(hi * qs);
    } else {
      const size_t o = ((size_t)l * max_seq + p) * kvd + (size_t)(head - nq) * hd;
      cache_store(kcache, o + e, lo, kv_f16);
      cache_store(kcache, o + e + half, hi, kv_f16);
    }
  }
  for (int i = threadIdx.x; i < kvd; i += blockDim.x)
    cache_store(vcache, ((size_t)l * max_seq + p) * kvd + i, row[qd + kvd + i], kv_f16);
}

// a16[t, i] = fp16(silu(G[t, i]) * U[t, i]); gu: fp32 [m, 2 ffn], gate columns first
__global__ void k_pf_swiglu(const float *__restrict__ gu, int ffn, _Float16 *a16) {
  const int t = blockIdx.x;
  const float *row = gu + (size_t)t * 2 * ffn;
  for (int i = threadIdx.x; i < ffn; i += blockDim.x) {
    const float g = row[i], u = row[ffn + i];
    a16[(size_t)t * ffn + i] = (_Float16)(g / (1.0f + expf(-g)) * u);
  }
}

// dst[0 .. d) = src[0 .. d)   (the last prompt position's hidden state, kept for the head and
// for the debug view of h(0..L))
__global__ void k_pf_copy_row(const float *__restrict__ src, float *dst, int d) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < d; i += gridDim.x * blockDim.x) dst[i] = src[i];
}

// ------------------------------------------------------------- attention
//
// Causal attention of the chunk's queries (positions pos0 .. pos0 + m - 1) over cache
// positions 0 .. their own.  One workgroup of four wavefronts per (query head, 128 queries),
// 32 queries per wavefront.  Keys in tiles of 64 through LDS.  Transposed products, so that
// the softmax over keys runs along a lane's registers and the probabilities feed the second
// product from the registers they are in:
//   S^T[key, q] = K[key, :] . Q[q, :]        A = K tile rows (LDS), B = Q (registers, whole loop)
//   O^T[d, q]  += V^T[d, key] P^T[key, q]    A = V tile stored transposed (LDS), B = P^T (registers)
// In S^T's register layout lane l holds, for query l % 32, keys (r/4)*8 + (l/32)*4 + r%4: the
// eight keys of registers 0..7 (8..15) are the K slots of that lane group in the first
// (second) MFMA of a 32-key block, and V^T is read from LDS with the same assignment.
// The scores carry log2(e)/sqrt(hd) (folded into q16): base-2 online softmax.
template <int HD>
__global__ __launch_bounds__(256, 2) void k_pf_attn(const _Float16 *__restrict__ q16, const void *kcache,
                                                 const void *vcache, int kv_f16, int nq, int nkv, int l, int max_seq,
                                                 int pos0, int m, _Float16 *o16) {
  constexpr int LDH = HD + 8;                 // K tile row stride (halfs)
  constexpr int LDV = 64 + 8;                 // V^T tile row stride (halfs)
  __shared__ __attribute__((aligned(16))) _Float16 Ks[64 * LDH];
  __shared__ __attribute__((aligned(16))) _Float16 Vt[HD * LDV];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int h = blockIdx.x, kvh = h / (nq / nkv);
  const int q0 = blockIdx.y * 128 + wv * 32;               // first query (chunk-relative) of this wavefront
  const int r32 = lane & 31, g = lane >> 5;
  const int qd = nq * HD, kvd = nkv * HD;
  const int tq = min(q0 + r32, m - 1);                      // this lane's query row (clamped: rows >= m are don't-care)
  const int my_pos = pos0 + q0 + r32;                       // its position (unclamped: masks keys beyond it)

  // Q of this wavefront as the B operand of S^T: for K step ks lane group g holds
  // d = ks*16 + g*8 .. +7 of query l % 32
  half8 qb[HD / 16];
#pragma unroll
  for (int ks = 0; ks < HD / 16; ++ks)
    qb[ks] = *(const half8 *)(q16 + (size_t)tq * qd + h * HD + ks * 16 + g * 8);

  f32x16 oacc[HD / 32];
#pragma unroll
  for (int b = 0; b < HD / 32; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[b][r] = 0.f;
  float mrun = -1.0e30f, lrun = 0.f;

  const int last_pos = min(pos0 + (int)blockIdx.y * 128 + 127, pos0 + m - 1);   // last key any query here attends
  const size_t cbase = (size_t)l * max_seq * kvd + (size_t)kvh * HD;
  for (int kt = 0; kt <= last_pos; kt += 64) {
    __syncthreads();                                        // previous tile consumed
    // stage the K tile [64 keys][HD] (16-byte runs along d, consecutive lanes along d) and the V
    // tile transposed [HD][64 keys] (consecutive lanes along the keys, so that the 2-byte
    // transposed stores of a wavefront fall into one row)
    for (int seg = tid; seg < 64 * (HD / 8); seg += 256) {
      const int key = seg / (HD / 8), ds = seg % (HD / 8);
      const int p = min(kt + key, last_pos);
      const uint4 kw = *(const uint4 *)((const char *)kcache + (cbase + (size_t)p * kvd + ds * 8) * 2);
      *(half8 *)(Ks + key * LDH + ds * 8) = cache_half8(kw, kv_f16);
    }
    for (int seg = tid; seg < 64 * (HD / 8); seg += 256) {
      const int key = seg & 63, ds = seg >> 6;
      const int p = min(kt + key, last_pos);
      const uint4 vw = *(const uint4 *)((const char *)vcache + (cbase + (size_t)p * kvd + ds * 8) * 2);
      const half8 vh = cache_half8(vw, kv_f16);
#pragma unroll
      for (int e = 0; e < 8; ++e) Vt[(ds * 8 + e) * LDV + key] = vh[e];
    }
    __syncthreads();
    // wavefronts whose queries all lie before this tile have nothing to add (uniform per wavefront)
    if (kt > pos0 + q0 + 31) continue;

    // S^T for the two 32-key blocks of the tile
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < HD / 16; ++ks) {
        const half8 ka = *(const half8 *)(Ks + (kb * 32 + r32) * LDH + ks * 16 + g * 8);
        s[kb] = mfma16(ka, qb[ks], s[kb]);
      }
    }
    // mask keys beyond the query's position, running maximum over the lane's 32 keys and the
    // other lane group's 32
    float mx = mrun;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kt + kb * 32 + c_row(r, lane);
        if (key > my_pos) s[kb][r] = -1.0e30f;
        mx = fmaxf(mx, s[kb][r]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float corr = __builtin_amdgcn_exp2f(mrun - mx);
    mrun = mx;
    float psum = 0.f;
    half8 pb[2][2];                                          // [key block][MFMA of the block]: B operands
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = s[kb][r] > -0.5e30f ? __builtin_amdgcn_exp2f(s[kb][r] - mx) : 0.f;
        const _Float16 ph = (_Float16)p;
        psum += (float)ph;                                   // the sum of what is actually multiplied
        pb[kb][r >> 3][r & 7] = ph;
      }
    psum += __shfl_xor(psum, 32);
    lrun = lrun * corr + psum;
#pragma unroll
    for (int b = 0; b < HD / 32; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[b][r] *= corr;
    // O^T += V^T P^T: per 32-key block two MFMAs; K slots of lane group g in MFMA j are keys
    // kb*32 + j*16 + {g*4 .. g*4+3, 8 + g*4 .. 8 + g*4+3} (registers 8j .. 8j+7 of S^T)
#pragma unroll
    for (int b = 0; b < HD / 32; ++b)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const _Float16 *vp = Vt + (b * 32 + r32) * LDV + kb * 32 + j * 16 + g * 4;
          const half4 v0 = *(const half4 *)vp, v1 = *(const half4 *)(vp + 8);
          half8 va;
          va[0] = v0[0]; va[1] = v0[1]; va[2] = v0[2]; va[3] = v0[3];
          va[4] = v1[0]; va[5] = v1[1]; va[6] = v1[2]; va[7] = v1[3];
          oacc[b] = mfma16(va, pb[kb][j], oacc[b]);
        }
  }
  // O^T[d, q] / l -> o16[q, h*HD + d]; registers 4i .. 4i+3 are four consecutive d
  if (q0 + r32 < m) {
    const float inv = 1.0f / lrun;
#pragma unroll
    for (int b = 0; b < HD / 32; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        half4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (_Float16)(oacc[b][4 * i + e] * inv);
        *(half4 *)(o16 + (size_t)(q0 + r32) * qd + h * HD + b * 32 + c_row(4 * i, lane)) = o;
      }
  }
}

}  // namespace pf

// =====================================================================================
// Batched decode step (several sequences, each at its own position and exit depth)
// =====================================================================================
//
// One decode step for n sequences, six launches per block: QKV GEMM, attention (with RoPE and
// the KV write), O-proj GEMM, gate/up GEMM (the norm in front of it rides on these two, see BdNorm;
// SwiGLU in its epilogue), down GEMM, block end (similarity, exit decision, next norm).  Every GEMM runs the bf16 backbone matrices for the
// rows (sequences) still in the backbone and the 4-bit river twins for the rows that have left
// it, over the same activation tile, each side touching only its own rows and not read at all
// when it has none (so a block whose rows all sit on one side reads one weight set).  With
// depths drawn independently per sequence most blocks read both sets: the reason Eq. 1 takes the
// minimum over the batch.  Which side a row is on is decided on the device after every backbone
// block (k_bd_block_end per sequence, k_bd_decide for Eq. 1's batch rule); the host never waits
// inside a step.
namespace bd {

using namespace pf;

constexpr int kRows = 32;             // most sequences per step (rows of the activation tile)
constexpr int kRecordsB = 1024;       // ring of per-step records of a batched context

struct SeqState {                     // device-side state of the sequences, [max_batch] each
  int *pos;                           // positions in the cache = position the next token is written to
  int *token;                         // token to consume next (produced by the last step / prefill)
  int *river;                         // 1: the sequence has left the backbone in the current step
  int *exit_pos;                      // exit position of the current step
  int *forced;                        // forced exit position of the current step (< 0: Eq. 1 decides)
};

// v_mfma_f32_16x16x32_f16: D[16x16] += A[16x32] B[32x16].  Lane l supplies row l % 16 of A and
// column l % 16 of B, the eight K values of lane group l / 16 each; D: register r of lane l is
// row (l / 16) * 4 + r, column l % 16.
typedef float f32x4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4v mfma16x16(half8 a, half8 b, f32x4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Eight 4-bit codes of one 32-bit word of the stream-order copy (see BdB: nibble j holds column 2j,
// nibble 4 + j column 2j + 1) -> the eight fp16 values 16 + code in column order: a nibble placed
// in bits 6..9 of the mantissa of 16.0 adds exactly its value, and pair j of the word needs one
// shift and one and-or.  Scale and zero point are applied to the products of a whole quantisation
// group (see bd_gemm_pass), not to the weights, so nothing is rounded here.
__device__ __forceinline__ half8 raw8(uint32_t w) {
  half8 out;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t sh = j < 2 ? w << (6 - 4 * j) : w >> (4 * j - 6);
    const half2v q = __builtin_bit_cast(half2v, (sh & 0x03c003c0u) | 0x4c004c00u);
    out[2 * j] = q[0];
    out[2 * j + 1] = q[1];
  }
  return out;
}

// The activations of a batched step (up to 32 sequence rows x K) are kept in the order the
// matrix-core operands are fetched in, so that a wavefront's A fragment of one MFMA step is one
// contiguous 1 KiB load: [step of 32 columns][row block of 16][lane group g][row % 16][8 columns
// 32 step + 8 g .. + 7]; 32 x K halfs (K % 32 == 0).
__host__ __device__ inline size_t frag_index(int m, int k) {
  return ((((size_t)(k >> 5)) * 2 + (m >> 4)) * 64 + ((k >> 3) & 3) * 16 + (m & 15)) * 8 + (k & 7);
}
__device__ __forceinline__ void frag_store(_Float16 *xf, int m, int k, _Float16 v) { xf[frag_index(m, k)] = v; }
// eight consecutive elements (m, k .. k+7), k % 8 == 0: one 16-byte store
__device__ __forceinline__ void frag_store8(_Float16 *xf, int m, int k, half8 v) { *(half8 *)(xf + frag_index(m, k)) = v; }

// The weights of a batched GEMM are kept a second time in **stream order**: the rows of the GEMM
// (matrices stacked along N, or the gate/up pair interleaved row by row) in units of 8 rows, and per
// unit and K tile the 16-byte pieces in the order the lanes of a wavefront fetch them ([lane group
// g][row % 8]).  A load instruction of a wavefront then reads two runs of 512 contiguous bytes (the
// two 8-row halves of its MFMA block) instead of 64 bytes from each of 16 rows, and the K tiles of
// a unit follow each other in memory.
//   bf16:   [unit][K tile of 64][step s][g][row % 8][columns k0 + 32 s + 8 g .. + 7]
//   codes:  [unit][K tile of 128][g][row % 8][4 words: word s = columns k0 + 32 s + 8 g .. + 7, column
//           2j in nibble j and column 2j + 1 in nibble 4 + j] -- a word is the B operand of one MFMA step
//   pairs:  [unit][K tile of 128][row % 8][64-column half] -- (scale, zero) as one packed word
// Rows beyond N and columns beyond K are zero (pairs: the row's last group).
struct BdB { const void *w, *sz; };
__host__ __device__ inline size_t bd_units(int N) { return (size_t)(N + 7) / 8; }
__host__ __device__ inline size_t bd_dense_bytes(int N, int K) { return bd_units(N) * (size_t)((K + 63) / 64) * 1024; }
__host__ __device__ inline size_t bd_codes_bytes(int N, int K) { return bd_units(N) * (size_t)((K + 127) / 128) * 512; }
__host__ __device__ inline size_t bd_pairs_bytes(int N, int K) { return bd_units(N) * (size_t)((K + 127) / 128) * 64; }

// row n of the GEMM -> (matrix, row) of the row-major source
__device__ __forceinline__ void bd_src_row(const GemmB &B, int interleaved, int n, int N, int &mat, int &row) {
  if (interleaved) { mat = n & 1; row = n >> 1; }
  else gemm_b_row(B, n, N, mat, row);
}
// one thread per 16-byte piece; K % 64 == 0, rows 16-byte aligned
__global__ void k_bd_pack_dense(GemmB B, int interleaved, int N, int K, uint4 *out) {
  const int nkt = (K + 63) / 64;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= bd_units(N) * nkt * 64) return;
  const int r8 = (int)(i & 7), g = (int)((i >> 3) & 3), st = (int)((i >> 5) & 1);
  const size_t t = i >> 6;
  const int kt = (int)(t % nkt), n = (int)(t / nkt) * 8 + r8, k = kt * 64 + st * 32 + g * 8;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (n < N && k + 8 <= K) {
    int mat, row;
    bd_src_row(B, interleaved, n, N, mat, row);
    v = *(const uint4 *)((const char *)B.w[mat] + ((size_t)row * K + k) * 2);
  }
  out[i] = v;
}
__global__ void k_bd_pack_codes(GemmB B, int interleaved, int N, int K, uint4 *out) {
  const int nkt = (K + 127) / 128;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= bd_units(N) * nkt * 32) return;
  const int r8 = (int)(i & 7), g = (int)((i >> 3) & 3);
  const size_t t = i >> 5;
  const int kt = (int)(t % nkt), n = (int)(t / nkt) * 8 + r8;
  uint32_t w[4] = {0u, 0u, 0u, 0u};
  if (n < N) {
    int mat, row;
    bd_src_row(B, interleaved, n, N, mat, row);
    const char *src = (const char *)B.w[mat] + (size_t)row * (K >> 1);
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      const int k = kt * 128 + st * 32 + g * 8;
      if (k + 8 > K) continue;
      // row-major: byte j = column k + 2j in the low nibble, k + 2j + 1 in the high nibble
      const uint32_t v = *(const uint32_t *)(src + (k >> 1));
#pragma unroll
      for (int j = 0; j < 4; ++j)
        w[st] |= (((v >> (8 * j)) & 0xfu) << (4 * j)) | (((v >> (8 * j + 4)) & 0xfu) << (16 + 4 * j));
    }
  }
  out[i] = make_uint4(w[0], w[1], w[2], w[3]);
}
// S.w[m] / S.sz[m]: the scales / zero points of matrix m, [rows][ceil(K / group)] bf16
__global__ void k_bd_pack_pairs(GemmB S, int interleaved, int N, int K, int group, uint32_t *out) {
  const int nkt = (K + 127) / 128, gpr = (K + group - 1) / group;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= bd_units(N) * nkt * 16) return;
  const int j = (int)(i & 1), r8 = (int)((i >> 1) & 7);
  const size_t t = i >> 4;
  const int kt = (int)(t % nkt), n = (int)(t / nkt) * 8 + r8, k = kt * 128 + j * 64;
  uint32_t v = 0;
  if (n < N) {
    int mat, row;
    bd_src_row(S, interleaved, n, N, mat, row);
    const size_t src = (size_t)row * gpr + min(k / group, gpr - 1);
    v = Store<1>::pack(Store<1>::ld(S.w[mat], src), Store<1>::ld(S.sz[mat], src));
  }
  out[i] = v;
}

// The row-wise kernels of a batched step (one workgroup of 256 per sequence row) read their row
// once: thread t owns columns 8 t + 2048 i .. + 7 and keeps up to kRowKeep such runs in registers
// between the reduction and the second use (rows longer than 2048 kRowKeep columns are read
// again).  n_part > 0: the partial sums [n_part][32][d] of the K-sliced GEMM that adds into h are
// added first, in order, and h is updated.
constexpr int kRowKeep = 4;
struct Run8 { float v[8]; };
__device__ __forceinline__ Run8 load_run8(float *row, const float *part, int n_part, int t, int d, int k) {
  float4 a = *(const float4 *)(row + k), b = *(const float4 *)(row + k + 4);
  if (n_part > 0) {
    for (int j = 0; j < n_part; ++j) {
      const float *p = part + ((size_t)j * kRows + t) * d + k;
      const float4 pa = *(const float4 *)p, pb = *(const float4 *)(p + 4);
      a.x += pa.x; a.y += pa.y; a.z += pa.z; a.w += pa.w;
      b.x += pb.x; b.y += pb.y; b.z += pb.z; b.w += pb.w;
    }
    *(float4 *)(row + k) = a;
    *(float4 *)(row + k + 4) = b;
  }
  return Run8{{a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w}};
}
__device__ __forceinline__ void norm_store_run8(const Run8 &x, float r, const void *gain, _Float16 *xf, int d, int t, int k) {
  half8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (_Float16)(x.v[j] * r * Store<1>::ld(gain, k + j));
  frag_store8(xf, t, k, o);
}

// xf[t, :] = fp16(h[t, :] * rsqrt(mean(h[t, :]^2) + eps) * gain) in fragment order; d % 8 == 0
__global__ __launch_bounds__(256) void k_bd_rmsnorm(float *__restrict__ h, const void *gain, int d, float eps,
                                                    _Float16 *xf, const float *__restrict__ part, int n_part) {
  __shared__ float red[16];
  const int t = blockIdx.x;
  float *row = h + (size_t)t * d;
  Run8 keep[kRowKeep];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < kRowKeep; ++i) {
    const int k = threadIdx.x * 8 + i * 2048;
    if (k < d) {
      keep[i] = load_run8(row, part, n_part, t, d, k);
#pragma unroll
      for (int j = 0; j < 8; ++j) ss = fmaf(keep[i].v[j], keep[i].v[j], ss);
    }
  }
  for (int k = threadIdx.x * 8 + kRowKeep * 2048; k < d; k += 2048) {
    const Run8 x = load_run8(row, part, n_part, t, d, k);
#pragma unroll
    for (int j = 0; j < 8; ++j) ss = fmaf(x.v[j], x.v[j], ss);
  }
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
  for (int i = 0; i < kRowKeep; ++i) {
    const int k = threadIdx.x * 8 + i * 2048;
    if (k < d) norm_store_run8(keep[i], r, gain, xf, d, t, k);
  }
  for (int k = threadIdx.x * 8 + kRowKeep * 2048; k < d; k += 2048)    // updated by this thread itself above
    norm_store_run8(load_run8(row, nullptr, 0, t, d, k), r, gain, xf, d, t, k);
}

// C[rows, N] (op)= A[rows, K] B^T for the rows r < n_rows with river[r] == want (want < 0: all
// rows); nothing is read if there is none.  MB = 1: up to 16 rows, MB = 2: up to 32.
//
// The weights are read once, so the kernel is a weight stream with the matrix cores doing the
// arithmetic.  Workgroup = eight wavefronts on `rows_per_wg` consecutive rows of B (a multiple
// of 8, chosen by the host so that the rows divide evenly over the CUs), taken in passes of
// RBW blocks of 16 rows; rows of a block beyond the workgroup's range are not loaded.  The
// wavefronts split K: wavefront w takes every eighth K tile (64 columns dense, 128 columns of
// 4-bit codes).  A lane loads its MFMA operands directly in the layout the instruction wants --
// no LDS on the way: for B, lane (n = lane % 16, g = lane / 16) fetches 16 bytes of row n (dense:
// columns k0 + 32 s + 8 g .. + 7 for the tile's two steps s; codes: the 32 columns
// k0 + 32 g .. + 31, one step per code word, which lie in one quantisation group) from the
// stream-order copy of the weights (see BdB), where they are the lane's piece of a contiguous run, for A the
// same columns of sequence row n (fp16, kept in fragment order: one contiguous 1 KiB per
// wavefront and step, from the L2; every workgroup reads the whole tile once, shared by its RBW
// row blocks).  P tiles are in flight per wavefront in registers.  The partial tiles of the
// wavefronts are summed in wavefront order through LDS.
// op (epi): store fp32, add into fp32, or -- with B's rows interleaved as (gate i, up i) --
// silu(gate) * up stored as fp16 in fragment order (the activation of the down projection; ldc is
// then its column count).
enum { EPI_STORE = 0, EPI_ADD = 1, EPI_SWIGLU = 2, EPI_ADD_NORM = 3 };
// The RMSNorm between a GEMM that completes h and the GEMM that consumes norm(h) costs no pass of
// its own: the producer (EPI_ADD_NORM: h += A B^T) also stores fp16(h * gain) in fragment order
// and, per workgroup and sequence row, the sum of squares of the h values it completed
// (ssq_out[workgroup][32]); the consumer adds those partial sums in workgroup order and applies
// the row's rsqrt(mean(h^2) + eps) to its product tile, which is the same product up to rounding.
constexpr int kSsqLoads = 16;                               // partial sums per lane: producers of up to 256 workgroups
struct BdRowScale {                                         // consumer side, per thread (see k_bd_gemm)
  float *rscale;                                            // LDS [32], or null: no fused norm
  float part[kSsqLoads];
  int d;
  float eps;
  __device__ __forceinline__ void finish() const {          // by every thread of the workgroup, before a workgroup barrier
    float v = 0.f;
#pragma unroll
    for (int u = 0; u < kSsqLoads; ++u) v += part[u];
    v = row16_sum(v);
    if ((threadIdx.x & 15) == 0 && (threadIdx.x >> 4) < kRows) rscale[threadIdx.x >> 4] = 1.0f / sqrtf(v / (float)d + eps);
  }
};
struct BdNorm {
  const void *gain;          // producer: gain of the norm in front of the consumer
  _Float16 *xnext;           // producer: fp16(h * gain), fragment order
  float *ssq_out;            // producer: [gridDim.x][32]
  const float *ssq_in;       // consumer: the producer's partial sums, or null
  int ssq_wgs;               // consumer: workgroups of the producer
  int d;                     // consumer: length of a row of h
  float eps;
};
constexpr int kBdWaves = 8;
constexpr int kBdKSplit = 4;                                // K slices of the narrow GEMMs (see k_bd_gemm)
template <int RBW, int MB> struct BdDepth {                 // K tiles in flight per wavefront (register budget)
  static constexpr int dense = MB == 1 ? (RBW == 1 ? 8 : RBW == 2 ? 5 : RBW == 4 ? 3 : 2) : (RBW == 1 ? 4 : RBW == 2 ? 3 : 2);
  static constexpr int w4 = MB == 1 ? (RBW == 1 ? 6 : RBW == 2 ? 4 : RBW == 4 ? 3 : 2) : (RBW <= 2 ? 3 : 2);
};
__host__ __device__ inline size_t bd_gemm_lds_bytes(int rbw, int mb) { return (size_t)kBdWaves * rbw * mb * 256 * 4; }

template <bool W4, int MB, int RBW>
__device__ __forceinline__ void bd_gemm_pass(const _Float16 *__restrict__ Af, const BdB &B, int N,
                                             int K, void *C, int ldc, int epi,
                                             const int *__restrict__ river, int want, int n_rows, int rows_per_wg,
                                             int k_split, int w0, int nw,
                                             float *red /* [kBdWaves][RBW][MB][256] */, const BdNorm &nrm,
                                             const BdRowScale &rsc) {
  const float *rscale = rsc.rscale;
  constexpr int P = W4 ? BdDepth<RBW, MB>::w4 : BdDepth<RBW, MB>::dense;
  constexpr int TILE = W4 ? 128 : 64;                         // columns per K tile
  constexpr int NA = W4 ? 4 : 2;                              // MFMA steps (16-byte A fragments) per tile
  // the pass is run by wavefronts w0 .. w0 + nw - 1 of the workgroup (all eight, or four when the
  // other four run the other weight format beside it); every wavefront of the workgroup executes the
  // same number of workgroup barriers in either case
  const int tid = threadIdx.x - w0 * 64, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);   // (a scalar: K tiles are addressed by scalar offsets)
  const int r16 = lane & 15, kg = lane >> 4;
  red += (size_t)w0 * RBW * MB * 256;
  // workgroup -> (group of rows, slice of K): with k_split > 1 the output is a partial sum, stored
  // as rows 32 ks .. of C for the consumer to add up (see load_run8)
  const int ks = blockIdx.x % k_split;
  const int wg_r0 = (blockIdx.x / k_split) * rows_per_wg, wg_r1 = min(N, wg_r0 + rows_per_wg);
  const int nkt_all = (K + TILE - 1) / TILE;
  const int kt0 = (int)((long long)nkt_all * ks / k_split), nkt = (int)((long long)nkt_all * (ks + 1) / k_split);
  struct Stage { uint4 a[MB * NA], b[RBW * (W4 ? 1 : 2)]; uint2 sz[W4 ? RBW : 1]; };
  float ssq[MB];                                              // EPI_ADD_NORM: this thread's sum of h^2, row i * 16 + (tid % 256) / 16
#pragma unroll
  for (int i = 0; i < MB; ++i) ssq[i] = 0.f;
  for (int p0 = wg_r0; p0 < wg_r1; p0 += RBW * 16) {
    // Stream order (see BdB): this lane's 16-byte piece of K tile 0 of row block 0 lies in unit p0 / 8
    // or the next one, at [g][row % 8]; a row block further is 2 units, a K tile further one tile.
    // Buffer loads: the pass's base in a descriptor, the lane's part of the address in one 32-bit
    // register, everything that is the same for all lanes in the scalar offset.
    constexpr unsigned UB = W4 ? 512u : 1024u;                // bytes of one unit's K tile
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((const char *)B.w + (size_t)(p0 >> 3) * nkt_all * UB), 0, 0x7ffffff0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((const char *)(W4 ? B.sz : B.w) + (W4 ? (size_t)(p0 >> 3) * nkt_all * 64 : 0)), 0, 0x7ffffff0, 0x00020000);
    const unsigned vw = (unsigned)(r16 >> 3) * nkt_all * UB + (kg * 8 + (r16 & 7)) * 16;
    const unsigned vz = (unsigned)(r16 >> 3) * nkt_all * 64u + (r16 & 7) * 8;      // both halves' pairs
    const unsigned bstride = (unsigned)nkt_all * 2u * UB, sstride = (unsigned)nkt_all * 128u;
    // Rows beyond the workgroup's range, columns beyond K (and K tiles beyond the slice, where such
    // a load is issued at all) get an offset beyond the descriptor's range: a buffer load then
    // returns zero without touching memory, and no load sits behind a branch.
    constexpr unsigned kOut = 0x80000000u;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc((void *)Af, 0, 0x7ffffff0, 0x00020000);
    auto row_ok = [&](int rb) { return p0 + rb * 16 + r16 < wg_r1; };
    auto ld16 = [&](const __amdgpu_buffer_rsrc_t &r, unsigned voff, unsigned soff, auto stream) {
      constexpr int aux = decltype(stream)::value ? 2 : 0;    // 2: streaming (read once)
      const u32x4 v = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, aux));
      return make_uint4(v.x, v.y, v.z, v.w);
    };
    auto load = [&](int kt, Stage &t) {
      const bool tile = kt < nkt;                             // (the same for all lanes)
      // step kt * NA + s of the activations; K % 64 == 0, so a 128-column tile may end after two steps
      // (columns of A beyond K are not defined; B's are zero)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int s = 0; s < NA; ++s)
          t.a[i * NA + s] = ld16(ra, tile && (kt * NA + s) * 32 < K ? lane * 16u : kOut,
                                 (unsigned)((kt * NA + s) * 2 + i) * 1024u, IC<0>{});
#pragma unroll
      for (int rb = 0; rb < RBW; ++rb) {
        const unsigned vo = tile && row_ok(rb) ? vw : kOut;
        if constexpr (W4) {
          t.b[rb] = ld16(rw, vo, rb * bstride + (unsigned)kt * UB, IC<1>{});
          const u32x2 q = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(
                                                        rz, tile && row_ok(rb) ? vz : kOut,
                                                        rb * sstride + (unsigned)kt * 64u, 0));
          t.sz[rb] = make_uint2(q.x, q.y);
        } else {
#pragma unroll
          for (int s = 0; s < 2; ++s) t.b[rb * 2 + s] = ld16(rw, vo, rb * bstride + (unsigned)kt * UB + s * 512u, IC<1>{});
        }
      }
    };
    f32x4v acc[RBW][MB];
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int i = 0; i < MB; ++i) acc[rb][i] = f32x4v{0.f, 0.f, 0.f, 0.f};
    auto compute = [&](const Stage &t) {
      if constexpr (W4) {
        // The codes go into the matrix cores as they are (16 + code, see raw8).  Per 64-column half of
        // the tile, which lies in one quantisation group: (W x)[m][n] = scale_n * sum_k a_mk (16 +
        // code_nk) - scale_n * (16 + zero_n) * sum_k a_mk; the last sum (rs) comes in the layout of
        // the product tile from a product with a matrix of ones, shared by the row blocks.
        const half8 ones = {(_Float16)1.f, (_Float16)1.f, (_Float16)1.f, (_Float16)1.f,
                            (_Float16)1.f, (_Float16)1.f, (_Float16)1.f, (_Float16)1.f};
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          f32x4v rs[MB];
#pragma unroll
          for (int i = 0; i < MB; ++i) {
            rs[i] = mfma16x16(__builtin_bit_cast(half8, t.a[i * NA + 2 * hf]), ones, f32x4v{0.f, 0.f, 0.f, 0.f});
            rs[i] = mfma16x16(__builtin_bit_cast(half8, t.a[i * NA + 2 * hf + 1]), ones, rs[i]);
          }
#pragma unroll
          for (int rb = 0; rb < RBW; ++rb) {
            const uint32_t w0 = hf ? t.b[rb].z : t.b[rb].x, w1 = hf ? t.b[rb].w : t.b[rb].y;
            const uint32_t pr = hf ? t.sz[rb].y : t.sz[rb].x;
            const half8 b0 = raw8(w0), b1 = raw8(w1);
            const float sc = bf16_lo(pr), nz = -sc * (16.0f + bf16_hi(pr));
#pragma unroll
            for (int i = 0; i < MB; ++i) {
              f32x4v tmp = mfma16x16(__builtin_bit_cast(half8, t.a[i * NA + 2 * hf]), b0, f32x4v{0.f, 0.f, 0.f, 0.f});
              tmp = mfma16x16(__builtin_bit_cast(half8, t.a[i * NA + 2 * hf + 1]), b1, tmp);
#pragma unroll
              for (int r = 0; r < 4; ++r) acc[rb][i][r] += sc * tmp[r] + nz * rs[i][r];
            }
          }
        }
      } else {
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
          for (int s = 0; s < 2; ++s) {
            const half8 b = bf16x8_to_half8(t.b[rb * 2 + s]);
#pragma unroll
            for (int i = 0; i < MB; ++i)
              acc[rb][i] = mfma16x16(__builtin_bit_cast(half8, t.a[i * NA + s]), b, acc[rb][i]);
          }
      }
    };
    // P stages in flight per wavefront; a round consumes each stage and refills it with the tile P
    // rounds of wavefronts further.  Refills beyond the slice are skipped -- except in the widest
    // 4-bit pass, which issues them all the same (beyond the range: no memory access), because the
    // compiler then needs fewer registers and that pass has none to spare.
    constexpr bool kAlways = W4 && RBW >= 8;
    Stage st[P];
#pragma unroll
    for (int u = 0; u < P; ++u)
      if (kAlways || kt0 + wv + nw * u < nkt) load(kt0 + wv + nw * u, st[u]);
    for (int kt = kt0 + wv; kt < nkt; kt += nw * P) {
#pragma unroll
      for (int u = 0; u < P; ++u) {
        const int k = kt + nw * u;
        if (k < nkt) compute(st[u]);
        if (kAlways || k + nw * P < nkt) load(k + nw * P, st[u]);
      }
    }
    // the partial tiles of the nw wavefronts -> one, in wavefront order; D: register r of lane l is sequence row
    // (l / 16) * 4 + r, B row l % 16
    if (rscale && p0 == wg_r0) rsc.finish();                  // (visible after the barriers below)
    __syncthreads();                                          // the previous pass has been read
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          red[((wv * RBW + rb) * MB + i) * 256 + (kg * 4 + r) * 16 + r16] = acc[rb][i][r];
    __syncthreads();
    constexpr int TILE_F = RBW * MB * 256;
    for (int e = tid; e < TILE_F; e += nw * 64) {
      const int rb = e / (MB * 256), i = (e / 256) % MB, row = i * 16 + ((e & 255) >> 4), n = p0 + rb * 16 + (e & 15);
      if (row >= n_rows || n >= wg_r1 || !(want < 0 || river[row] == want)) continue;
      const float rs_row = rscale ? rscale[row] : 1.0f;
      auto total = [&](int idx) {
        float v = red[idx];
#pragma unroll
        for (int w = 1; w < nw; ++w) v += red[w * TILE_F + idx];
        return v * rs_row;
      };
      if (epi == EPI_SWIGLU) {
        if (n & 1) continue;
        const float g = total(e), u = total(e + 1);
        frag_store((_Float16 *)C, row, n >> 1, (_Float16)(g / (1.0f + expf(-g)) * u));
      } else {
        float *p = (float *)C + (size_t)(k_split > 1 ? ks * kRows + row : row) * ldc + n;
        const float v = total(e);
        if (epi == EPI_ADD_NORM) {
          const float hv = *p + v;
          *p = hv;
          frag_store(nrm.xnext, row, n, (_Float16)(hv * Store<1>::ld(nrm.gain, n)));
#pragma unroll
          for (int i2 = 0; i2 < MB; ++i2)
            if (i2 == i) ssq[i2] = fmaf(hv, hv, ssq[i2]);
        } else if (epi == EPI_ADD) *p += v;
        else *p = v;
      }
    }
  }
  if (epi == EPI_ADD_NORM) {
    // this workgroup's sums of squares per sequence row: the 16 lanes of a row, then the thread
    // groups 256 apart (the same rows), in a fixed order
    __syncthreads();                                          // the last pass has been read
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const float sr = row16_sum(ssq[i]);
      if ((tid & 15) == 0) red[(tid >> 8) * kRows + i * 16 + ((tid & 255) >> 4)] = sr;
    }
    __syncthreads();
    if (tid < MB * 16 && tid < n_rows && (want < 0 || river[tid] == want)) {
      float v = red[tid];
      if (nw * 64 > 256) v += red[kRows + tid];
      nrm.ssq_out[(size_t)blockIdx.x * kRows + tid] = v;
    }
  }
}

// One launch per GEMM of a step: the bf16 matrices for the rows still in the backbone, then the
// 4-bit twins for the rows that have left it (by_flag; otherwise the bf16 matrices for all
// rows, as the LM head needs).  A side without rows is not read.  Af: the activations in fragment
// order (see frag_index).  k_split > 1: narrow matrices (16 rows per CU would leave every
// workgroup reading all of A for one row block) are dealt out as k_split K slices of four times
// the rows; C is then the partial-sum buffer [k_split][32][ldc].
template <int MB, int RBW>
__global__ __launch_bounds__(512) void k_bd_gemm(const _Float16 *__restrict__ Af, BdB Bd, BdB Bq,
                                                 int N, int K, void *C, int ldc, int epi,
                                                 const int *__restrict__ river, int by_flag, int n_rows,
                                                 int rows_per_wg, int k_split, BdNorm nrm) {
  extern __shared__ float red[];
  __shared__ int any[2];
  __shared__ float rscale[kRows];
  if (threadIdx.x < 2) any[threadIdx.x] = 0;
  __syncthreads();
  if ((int)threadIdx.x < n_rows) any[by_flag && river[threadIdx.x] != 0] = 1;
  // consumer of a fused norm: the producer's partial sums of squares of row threadIdx.x / 16 are
  // fetched here (16 lanes per row, up to kSsqLoads each) and added up, in a fixed order, where the
  // first product tile is complete (BdRowScale::finish) -- their latency is the K loop's
  BdRowScale rsc{nrm.ssq_in ? rscale : nullptr, {}, nrm.d, nrm.eps};
  if (nrm.ssq_in) {
    const int row = threadIdx.x >> 4, j0 = threadIdx.x & 15;
#pragma unroll
    for (int u = 0; u < kSsqLoads; ++u) {
      const int j = j0 + 16 * u;
      rsc.part[u] = row < n_rows && j < nrm.ssq_wgs ? nrm.ssq_in[(size_t)j * kRows + row] : 0.f;
    }
  }
  __syncthreads();
  const bool dense = any[0] != 0, twin = any[1] != 0;
  // Both sides: four wavefronts each, side by side -- the 4-bit side's dequantisation runs in the
  // shadow of the bf16 side's memory waits, and there is one ramp-up and one tail instead of two.
  constexpr int ND = kBdWaves / 2;                              // wavefronts of the bf16 side when both run (3 .. 4 measured best)
  const bool second = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) >= ND;   // (a scalar branch)
  if (dense && (!twin || !second))
    bd_gemm_pass<false, MB, RBW>(Af, Bd, N, K, C, ldc, epi, river, by_flag ? 0 : -1, n_rows,
                                 rows_per_wg, k_split, 0, twin ? ND : kBdWaves, red, nrm, rsc);
  if (twin && (!dense || second))
    bd_gemm_pass<true, MB, RBW>(Af, Bq, N, K, C, ldc, epi, river, 1, n_rows,
                                rows_per_wg, k_split, dense ? ND : 0, dense ? kBdWaves - ND : kBdWaves, red, nrm, rsc);
}

// h[b, :] = E[token[b], :] (also h_prev and the debug view of h(0)); start-of-step state of
// sequence b (forced exit position 0 puts it into the river from the first block on)
__global__ void k_bd_embed(SeqState st, const void *tok_emb, int d, int vocab, int L, float *h, float *h_prev,
                           float *hist) {
  const int b = blockIdx.x;
  const int tok = min(max(st.token[b], 0), vocab - 1);
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    const float v = Store<1>::ld(tok_emb, (size_t)tok * d + i);
    h[(size_t)b * d + i] = v;
    h_prev[(size_t)b * d + i] = v;
    hist[(size_t)b * d + i] = v;
  }
  if (threadIdx.x == 0) {
    const bool r0 = st.forced[b] == 0;
    st.river[b] = r0 ? 1 : 0;
    st.exit_pos[b] = r0 ? 0 : L;
  }
}

__global__ void k_bd_copy(const float *__restrict__ src, float *dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// Single-query attention of a batched step with RoPE and the KV write in front of it.  One
// workgroup per (sequence b, kv head, group of REP query heads of that kv head, split of the
// positions 0 .. pos[b]): the K/V rows of the kv head are read once for the REP heads.
//
// Prologue (from the raw QKV rows the GEMM left): the REP query vectors rotated at position
// pos[b] and scaled by log2(e)/sqrt(hd), this token's k (rotated) and v rounded to the cache
// dtype, all into LDS; the workgroup whose split holds position pos[b] (the first head group)
// also writes them to slot (b, l, pos[b]) of the shared cache -- the same slot for backbone and
// river rows -- and nobody reads that slot from the cache in this launch.
// Sixteen lanes share a cached row (HD/16 elements each, one 16- or 8-byte load), the 16 lane
// groups stride over the split's positions in batches of four K rows and their V rows, the next
// batch in flight while one is consumed.  Every lane group keeps a running softmax per head
// (base 2, rescaled once per batch; DPP row sums for the scores); lane groups, wavefronts and --
// with several splits -- workgroups are merged in a fixed order: every workgroup publishes (max,
// sum, unnormalised output) per head and the last one to arrive of the group merges them in
// split order (device-coherent stores and loads, no fences).  The result goes to o16 in fragment
// order (frag_store), the output projection's input.
constexpr int kBdAttnMaxSplits = 8;
__host__ __device__ inline size_t bd_attn_lds_bytes(int rep, int hd) {
  return ((size_t)rep * hd + 2 * hd + 64 + 4 * rep * hd) * 4;
}
template <int HD, bool KV_F16, int REP>
__global__ __launch_bounds__(256) void k_bd_attn(const float *__restrict__ qkv, const float2 *__restrict__ rope,
                                                 void *kcache, void *vcache, int nq, int nkv, int n_seq, int l,
                                                 int max_seq, size_t seq_stride, const int *__restrict__ pos,
                                                 int n_splits, float *part_o, float *part_ml,
                                                 unsigned int *tickets, _Float16 *o16) {
  constexpr int EL = HD / 16, HALF = HD / 2;                   // EL: elements per lane of a cached row
  extern __shared__ float sm[];
  float *qs = sm;                                              // [REP][HD]
  float *kc = qs + REP * HD, *vc = kc + HD;                    // this token's k, v (cache-rounded values)
  float *red = vc + HD;                                        // [64]
  float *part = red + 64;                                      // [4 wavefronts][REP][HD]
  const int tid = threadIdx.x, grp = tid >> 4, dl = tid & 15, wv = tid >> 6;
  const int rep = nq / nkv, hgs = rep / REP;
  // Workgroup index -> (data group g = (sequence, kv head, split), head group hg) such that the head
  // groups that read the same K/V rows run on the same XCD (consecutive workgroup ids go round the
  // 8 XCDs) and meet in that XCD's L2.
  const int bi = blockIdx.x, g = (bi / (8 * hgs)) * 8 + (bi & 7), hg = (bi % (8 * hgs)) >> 3;
  if (g >= n_seq * nkv * n_splits) return;
  const int sp = g % n_splits, kvh = (g / n_splits) % nkv, b = g / (n_splits * nkv);
  const int h0 = kvh * rep + hg * REP;
  const int P = pos[b], T = P + 1, qd = nq * HD, kvd = nkv * HD, ld = qd + 2 * kvd;
  const int chunk = (T + n_splits - 1) / n_splits, p0 = sp * chunk, p1 = min(T, p0 + chunk);
  const bool owner = P >= p0 && P < p1;                        // this split holds the current position
  const float *row_in = qkv + (size_t)b * ld;
  const size_t base = (size_t)b * seq_stride + (size_t)l * max_seq * kvd + (size_t)kvh * HD;
  // The cached rows p0 .. pc - 1 (the current position, the last one, is not read from the cache:
  // it seeds the first lane group's state from LDS).  Lane group grp takes rows p0 + grp + 16 t in
  // batches of RB, K and V rows together, the next batch in flight while one is consumed.
  const int pc = owner ? P : p1;
  constexpr int RB = 4;
  constexpr int NW = EL / 2;                                   // 32-bit words of a lane's row slice
  struct Batch { uint32_t k[RB][NW], v[RB][NW]; };
  auto load = [&](int j0, Batch &t) {
#pragma unroll
    for (int u = 0; u < RB; ++u) {
      const int j = min(j0 + 16 * u, pc - 1);                  // rows beyond the last read it again (masked below)
      const size_t off = (base + (size_t)j * kvd + dl * EL) * 2;
      if constexpr (NW == 4) {
        const uint4 a = *(const uint4 *)((const char *)kcache + off), c = *(const uint4 *)((const char *)vcache + off);
        t.k[u][0] = a.x; t.k[u][1] = a.y; t.k[u][2] = a.z; t.k[u][3] = a.w;
        t.v[u][0] = c.x; t.v[u][1] = c.y; t.v[u][2] = c.z; t.v[u][3] = c.w;
      } else {
        const uint2 a = *(const uint2 *)((const char *)kcache + off), c = *(const uint2 *)((const char *)vcache + off);
        t.k[u][0] = a.x; t.k[u][1] = a.y;
        t.v[u][0] = c.x; t.v[u][1] = c.y;
      }
    }
  };
  // the first batch does not depend on this step's q, k, v: it is in flight during the prologue
  Batch ba, bb;
  const int step = 16 * RB;
  int j0 = p0 + grp;
  if (j0 < pc) load(j0, ba);
  // ---- prologue: RoPE, rounding, KV write
  {
    const float qscale = 1.4426950408889634f / sqrtf((float)HD);
    for (int t = tid; t < REP * HALF; t += 256) {
      const int r = t / HALF, e = t % HALF;
      const float2 cs = rope[(size_t)P * HALF + e];
      const float *src = row_in + (h0 + r) * HD;
      const float a = src[e], c = src[e + HALF];
      qs[r * HD + e] = (a * cs.x - c * cs.y) * qscale;
      qs[r * HD + e + HALF] = (a * cs.y + c * cs.x) * qscale;
    }
    if (owner) {
      auto rnd = [](float v) { return KV_F16 ? (float)(_Float16)v : Store<1>::rnd(v); };
      const bool writer = hg == 0;
      const size_t slot = base + (size_t)P * kvd;
      if (tid < HALF) {
        const int e = tid;
        const float2 cs = rope[(size_t)P * HALF + e];
        const float *src = row_in + qd + kvh * HD;
        const float a = src[e], c = src[e + HALF];
        const float lo = a * cs.x - c * cs.y, hi = a * cs.y + c * cs.x;
        kc[e] = rnd(lo); kc[e + HALF] = rnd(hi);
        if (writer) { cache_store(kcache, slot + e, lo, KV_F16); cache_store(kcache, slot + e + HALF, hi, KV_F16); }
      } else if (tid >= 128 && tid < 128 + HD) {
        const int e = tid - 128;
        const float v = row_in[qd + kvd + kvh * HD + e];
        vc[e] = rnd(v);
        if (writer) cache_store(vcache, slot + e, v, KV_F16);
      }
    }
  }
  __syncthreads();
  float q[REP][EL];
#pragma unroll
  for (int r = 0; r < REP; ++r)
#pragma unroll
    for (int e = 0; e < EL; ++e) q[r][e] = qs[r * HD + dl * EL + e];
  // running softmax per head (base 2: the scores carry log2 e): maximum, sum, weighted values
  float m[REP], ls[REP], o[REP][EL];
#pragma unroll
  for (int r = 0; r < REP; ++r) {
    m[r] = -1.0e30f; ls[r] = 0.f;
#pragma unroll
    for (int e = 0; e < EL; ++e) o[r][e] = 0.f;
  }
  if (owner && grp == 0) {
#pragma unroll
    for (int r = 0; r < REP; ++r) {
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < EL; ++e) dot = fmaf(kc[dl * EL + e], q[r][e], dot);
      m[r] = row16_sum(dot);
      ls[r] = 1.f;
#pragma unroll
      for (int e = 0; e < EL; ++e) o[r][e] = vc[dl * EL + e];
    }
  }
  auto consume = [&](int j0, const Batch &t) {
    float sc[RB][REP];
#pragma unroll
    for (int u = 0; u < RB; ++u) {
      float kf[EL];
#pragma unroll
      for (int w = 0; w < NW; ++w) { kf[2 * w] = cache_lo(t.k[u][w], KV_F16); kf[2 * w + 1] = cache_hi(t.k[u][w], KV_F16); }
      const bool ok = j0 + 16 * u < pc;
#pragma unroll
      for (int r = 0; r < REP; ++r) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < EL; ++e) dot = fmaf(kf[e], q[r][e], dot);
        sc[u][r] = ok ? row16_sum(dot) : -1.0e30f;
      }
    }
#pragma unroll
    for (int r = 0; r < REP; ++r) {
      float mn = m[r];
#pragma unroll
      for (int u = 0; u < RB; ++u) mn = fmaxf(mn, sc[u][r]);
      const float cg = __builtin_amdgcn_exp2f(m[r] - mn);      // <= 1; 1 while nothing has been seen
      m[r] = mn;
      ls[r] *= cg;
#pragma unroll
      for (int e = 0; e < EL; ++e) o[r][e] *= cg;
#pragma unroll
      for (int u = 0; u < RB; ++u) sc[u][r] = sc[u][r] > -0.5e30f ? __builtin_amdgcn_exp2f(sc[u][r] - mn) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < RB; ++u) {
      float vf[EL];
#pragma unroll
      for (int w = 0; w < NW; ++w) { vf[2 * w] = cache_lo(t.v[u][w], KV_F16); vf[2 * w + 1] = cache_hi(t.v[u][w], KV_F16); }
#pragma unroll
      for (int r = 0; r < REP; ++r) {
        ls[r] += sc[u][r];
#pragma unroll
        for (int e = 0; e < EL; ++e) o[r][e] = fmaf(sc[u][r], vf[e], o[r][e]);
      }
    }
  };
  // (the loads of the loop are issued whether or not their rows exist -- beyond the last row they
  // fetch it again -- so that none sits behind a branch and a batch's wait leaves the next one alone)
  for (; j0 < pc; j0 += 2 * step) {
    load(j0 + step, bb);
    consume(j0, ba);
    load(j0 + 2 * step, ba);
    if (j0 + step < pc) consume(j0 + step, bb);
  }
  // merge: the four lane groups of a wavefront by lane exchange (lanes 16 and 32 apart hold the
  // same elements), then the four wavefronts through LDS, both in a fixed order
#pragma unroll
  for (int r = 0; r < REP; ++r) {
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float m2 = __shfl_xor(m[r], off), l2 = __shfl_xor(ls[r], off);
      const float mn = fmaxf(m[r], m2);
      const float c1 = __builtin_amdgcn_exp2f(m[r] - mn), c2 = __builtin_amdgcn_exp2f(m2 - mn);
      ls[r] = ls[r] * c1 + l2 * c2;
#pragma unroll
      for (int e = 0; e < EL; ++e) o[r][e] = o[r][e] * c1 + __shfl_xor(o[r][e], off) * c2;
      m[r] = mn;
    }
  }
  float *wml = red;                                            // [4 wavefronts][REP][2]
  if ((tid & 63) < 16) {
#pragma unroll
    for (int r = 0; r < REP; ++r) {
#pragma unroll
      for (int e = 0; e < EL; ++e) part[(wv * REP + r) * HD + dl * EL + e] = o[r][e];
      if (dl == 0) { wml[(wv * REP + r) * 2] = m[r]; wml[(wv * REP + r) * 2 + 1] = ls[r]; }
    }
  }
  __syncthreads();
  // element e of head r over the four wavefronts -> (M, L, O) of this split
  auto split_result = [&](int r, int e, float &M, float &Ls, float &O) {
    M = -1.0e30f; Ls = 0.f; O = 0.f;
    for (int w = 0; w < 4; ++w) M = fmaxf(M, wml[(w * REP + r) * 2]);
    for (int w = 0; w < 4; ++w) {
      const float cw = __builtin_amdgcn_exp2f(wml[(w * REP + r) * 2] - M);   // a wavefront that saw nothing has sum 0
      Ls = fmaf(wml[(w * REP + r) * 2 + 1], cw, Ls);
      O = fmaf(part[(w * REP + r) * HD + e], cw, O);
    }
  };
  if (n_splits == 1) {
    for (int t = tid; t < REP * HD; t += 256) {
      float M, Ls, O;
      split_result(t / HD, t % HD, M, Ls, O);
      frag_store(o16, b, (h0 + t / HD) * HD + t % HD, (_Float16)(O / Ls));
    }
    return;
  }
  // ---- several splits: publish the partial result, the last workgroup of the group merges
  for (int t = tid; t < REP * HD; t += 256) {
    const int r = t / HD, e = t % HD;
    float M, Ls, O;
    split_result(r, e, M, Ls, O);
    const size_t pi = ((size_t)b * nq + h0 + r) * kBdAttnMaxSplits + sp;
    pub(part_o + pi * HD + e, O);
    if (e == 0) { pub(part_ml + pi * 2, M); pub(part_ml + pi * 2 + 1, Ls); }
  }
  if (!last_arriver(tickets + ((size_t)b * nkv + kvh) * hgs + hg, (unsigned)n_splits, (int *)(red + 60))) return;
  for (int t = tid; t < REP * HD; t += 256) {
    const int r = t / HD, e = t % HD;
    const size_t pb = ((size_t)b * nq + h0 + r) * kBdAttnMaxSplits;
    float Mg = -1.0e30f;
    for (int j = 0; j < n_splits; ++j) Mg = fmaxf(Mg, sub(part_ml + (pb + j) * 2));
    float Lg = 0.f, Og = 0.f;
    for (int j = 0; j < n_splits; ++j) {
      const float cj = __builtin_amdgcn_exp2f(sub(part_ml + (pb + j) * 2) - Mg);   // an empty split has sum 0
      Lg = fmaf(sub(part_ml + (pb + j) * 2 + 1), cj, Lg);
      Og = fmaf(sub(part_o + (pb + j) * HD + e), cj, Og);
    }
    frag_store(o16, b, (h0 + r) * HD + e, (_Float16)(Og / Lg));
  }
}

// After block l1 (1-based), one workgroup per sequence b: s_b = cos(h_prev[b], h[b]) if the row
// is still in the backbone (recorded, and kept in s_of for k_bd_decide); h(l1) of the row is
// kept (hist, the debug view) and becomes the next block's h_prev; with decide != 0 the row's own
// exit decision (forced position, else s_b > tau; first hit at or above L_s, never at L -- the
// caller passes decide = 0 outside that range and when Eq. 1's batch rule decides); then the
// RMSNorm in front of the next GEMM (the next block's attention norm, or the final norm) into
// xf in fragment order -- its sum of squares is the similarity's <h, h>.
__global__ __launch_bounds__(256) void k_bd_block_end(float *h_prev, float *__restrict__ h, int d, int l1, int L,
                                                      SeqState st, float *s_of, float *sims /* [n][L] of this step */,
                                                      float *hist /* [n][d] */, int decide, float tau,
                                                      const void *next_gain, float eps, _Float16 *xf,
                                                      const float *__restrict__ part, int n_part) {
  __shared__ float red[32];
  const int b = blockIdx.x;
  const bool live = st.river[b] == 0;
  float *row = h + (size_t)b * d;
  float p3[3] = {0.f, 0.f, 0.f};
  // one run: the sums of Eq. 1's similarity, h(l1) into h_prev and the debug view
  auto take = [&](int k) {
    const float4 a0 = *(const float4 *)(h_prev + (size_t)b * d + k), a1 = *(const float4 *)(h_prev + (size_t)b * d + k + 4);
    const Run8 c = load_run8(row, part, n_part, b, d, k);      // (adds the down projection's partial sums)
    const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      p3[0] = fmaf(a[j], c.v[j], p3[0]); p3[1] = fmaf(a[j], a[j], p3[1]); p3[2] = fmaf(c.v[j], c.v[j], p3[2]);
    }
    const float4 c0 = make_float4(c.v[0], c.v[1], c.v[2], c.v[3]), c1 = make_float4(c.v[4], c.v[5], c.v[6], c.v[7]);
    *(float4 *)(h_prev + (size_t)b * d + k) = c0; *(float4 *)(h_prev + (size_t)b * d + k + 4) = c1;
    *(float4 *)(hist + (size_t)b * d + k) = c0; *(float4 *)(hist + (size_t)b * d + k + 4) = c1;
    return c;
  };
  Run8 keep[kRowKeep];
#pragma unroll
  for (int i = 0; i < kRowKeep; ++i) {
    const int k = threadIdx.x * 8 + i * 2048;
    if (k < d) keep[i] = take(k);
  }
  for (int k = threadIdx.x * 8 + kRowKeep * 2048; k < d; k += 2048) (void)take(k);
  block_sum_k<3>(p3, red);
  if (live && threadIdx.x == 0) {
    float s = 0.f;
    if (p3[1] > 0.f && p3[2] > 0.f) s = fminf(1.0f, fmaxf(-1.0f, p3[0] / (sqrtf(p3[1]) * sqrtf(p3[2]))));
    s_of[b] = s;
    sims[(size_t)b * L + (l1 - 1)] = s;
    if (decide) {
      const int f = st.forced[b];
      if (f >= 0 ? f == l1 : s > tau) { st.river[b] = 1; st.exit_pos[b] = l1; }
    }
  }
  const float r = 1.0f / sqrtf(p3[2] / (float)d + eps);
#pragma unroll
  for (int i = 0; i < kRowKeep; ++i) {
    const int k = threadIdx.x * 8 + i * 2048;
    if (k < d) norm_store_run8(keep[i], r, next_gain, xf, d, b, k);
  }
  for (int k = threadIdx.x * 8 + kRowKeep * 2048; k < d; k += 2048)    // updated by this thread itself above
    norm_store_run8(load_run8(row, nullptr, 0, b, d, k), r, next_gain, xf, d, b, k);
}

// The exit decision after backbone block l1 from the similarities k_bd_block_end left (launched
// when Eq. 1's batch rule is in force).  rule 0: every
// sequence for itself (s_b > tau); rule 1: Eq. 1 as printed, the whole batch leaves together
// once min_b s_b > tau.  A forced exit position overrides the threshold for its sequence.
// First hit at or above L_s, never at L, strict '>'.  One wavefront.
__global__ void k_bd_decide(int n, int l1, int L, int min_exit, float tau, int rule, SeqState st,
                            const float *__restrict__ s_of) {
  if (threadIdx.x != 0 || l1 < min_exit || l1 >= L) return;
  bool all_pass = true;                                       // Eq. 1's minimum over the batch
  for (int b = 0; b < n; ++b)
    if (!st.river[b] && !(s_of[b] > tau)) all_pass = false;
  for (int b = 0; b < n; ++b) {
    if (st.river[b]) continue;
    const int f = st.forced[b];
    const bool go = f >= 0 ? f == l1 : (rule == 1 ? all_pass : s_of[b] > tau);
    if (go) { st.river[b] = 1; st.exit_pos[b] = l1; }
  }
}

// Greedy token of every sequence (lowest index on ties), its record, and the step's end: the
// sequence advances by one position.  kBdArgmaxChunks workgroups per sequence scan a chunk of the
// row each and publish (value, index); the last one to arrive takes the best of them in chunk
// order (part: [n][chunks][2], tickets: [n], zero between launches).
constexpr int kBdArgmaxChunks = 16;
__global__ __launch_bounds__(256) void k_bd_argmax(const float *__restrict__ logits, int vocab, SeqState st,
                                                   int *rec_token, int *rec_exit, float *part, unsigned int *tickets) {
  __shared__ float red[64];
  __shared__ int flag;
  const int b = blockIdx.x / kBdArgmaxChunks, c = blockIdx.x % kBdArgmaxChunks;
  const int per = ((vocab + kBdArgmaxChunks - 1) / kBdArgmaxChunks + 3) / 4 * 4;
  const int i_begin = c * per, i_end = min(vocab, i_begin + per);
  float best = -INFINITY;
  int besti = 0x7fffffff;
  const float *row = logits + (size_t)b * vocab;
  // eight loads in flight per thread (the scan is a chain of load latencies otherwise)
  for (int i0 = i_begin + threadIdx.x; i0 < i_end; i0 += 8 * blockDim.x) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * blockDim.x;
      v[u] = i < i_end ? row[i] : -INFINITY;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u * (int)blockDim.x;
      argmax_take(best, besti, v[u], i < i_end ? i : 0x7fffffff);
    }
  }
  block_argmax(best, besti, red);
  float *mine = part + ((size_t)b * kBdArgmaxChunks + c) * 2;
  if (threadIdx.x == 0) { pub(mine, best); pub(mine + 1, __int_as_float(besti)); }
  if (!last_arriver(tickets + b, kBdArgmaxChunks, &flag)) return;
  if (threadIdx.x == 0) {
    best = -INFINITY;
    besti = 0x7fffffff;
    for (int j = 0; j < kBdArgmaxChunks; ++j) {
      const float *pj = part + ((size_t)b * kBdArgmaxChunks + j) * 2;
      argmax_take(best, besti, sub(pj), __float_as_int(sub(pj + 1)));
    }
    st.token[b] = besti;
    st.pos[b] += 1;
    if (rec_token) { rec_token[b] = besti; rec_exit[b] = st.exit_pos[b]; }
  }
}

// sims[b][l] = NaN for every block (blocks that run as river twins keep it)
__global__ void k_bd_fill_nan(float *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = __uint_as_float(0x7fc00000u);
}

// after a prefill of sequence `seq`: its next token and length
__global__ void k_bd_after_prefill(SeqState st, int seq, const int *cur_token, int len) {
  if (threadIdx.x == 0 && blockIdx.x == 0) { st.token[seq] = *cur_token; st.pos[seq] = len; }
}

}  // namespace bd
}  // namespace river
