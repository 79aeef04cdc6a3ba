// Host side of the C ABI declared in include/river.h: workspace layout, launches,
// bookkeeping.  All arithmetic of the decode step lives in river_device.h.
#include "river.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstddef>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "river_device.h"
#include "river_prefill.h"

using namespace river;

// ------------------------------------------------------------------ kernels
//
// All kernels take the device descriptor by pointer (it lives in the workspace and is read
// with scalar loads) and the per-step arguments by value.

// One-kernel-per-phase mode.  The exit state travels between the kernels of a token in
// DevState: the QKV kernel of block l derives it (every workgroup identically), workgroup 0
// stores it in slot l & 1, the other kernels of the block read that slot.
__device__ __forceinline__ Ctl load_ctl(DevRef D, int l) {
  Ctl c;
  c.river = D.st->slot_river[l & 1] != 0;
  c.exit_pos = D.st->slot_exit[l & 1];
  return c;
}

template <int DT>
__global__ __launch_bounds__(kBlock) void k_qkv(const Dev *Dp, StepArgs A, int l) {
  extern __shared__ float lds[];
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  Ctl ctl;
  if (l == 0) {
    ctl = ctl_init(D, A);
    record_init(D, A);
  } else {
    ctl = load_ctl(D, l - 1);
    exit_test(D, A, l, ctl, lds);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    D.st->slot_river[l & 1] = ctl.river;
    D.st->slot_exit[l & 1] = ctl.exit_pos;
  }
  Pre<DT> pre;
  prefetch_phase<DT>(D, l, PH_QKV, ctl.river, pre);
  phase_qkv<DT>(D, A, l, ctl.river, lds, pre, [] {});
}
// F16: the 16-bit KV cache of a bf16 model holds IEEE half values (a kernel of its own per
// cache type, so that no kernel carries both conversions)
template <int DT, bool F16>
__global__ __launch_bounds__(kBlock) void k_attn(const Dev *Dp, StepArgs A, int l) {
  extern __shared__ float lds[];
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  phase_attn<DT, F16>(D, A, l, load_ctl(D, l), lds, [] {}, [] {});
}
template <int DT>
__global__ __launch_bounds__(kBlock) void k_oproj(const Dev *Dp, StepArgs A, int l) {
  extern __shared__ float lds[];
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  const Ctl ctl = load_ctl(D, l);
  Pre<DT> pre;
  prefetch_phase<DT>(D, l, PH_O, ctl.river, pre);
  phase_oproj<DT>(D, A, l, ctl.river, lds, pre, [] {});
}
template <int DT>
__global__ __launch_bounds__(kBlock) void k_gateup(const Dev *Dp, StepArgs A, int l) {
  extern __shared__ float lds[];
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  const Ctl ctl = load_ctl(D, l);
  Pre<DT> pre;
  prefetch_phase<DT>(D, l, PH_GU, ctl.river, pre);
  phase_gateup<DT>(D, A, l, ctl.river, lds, pre, [] {});
}
template <int DT>
__global__ __launch_bounds__(kBlock) void k_down(const Dev *Dp, StepArgs A, int l) {
  extern __shared__ float lds[];
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  const Ctl ctl = load_ctl(D, l);
  Pre<DT> pre;
  prefetch_phase<DT>(D, l, PH_DOWN, ctl.river, pre);
  phase_down<DT>(D, A, l, ctl.river, lds, pre, [] {});
}
template <int DT>
__global__ __launch_bounds__(kBlock) void k_head(const Dev *Dp, StepArgs A) {
  extern __shared__ float lds[];
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  const Ctl ctl = load_ctl(D, D.L - 1);
  Pre<DT> pre;
  prefetch_head<DT>(D, pre);
  phase_head<DT>(D, A, ctl, lds, pre, [] {});
}

#ifdef RIVER_TRACE
// diagnostics build: every workgroup stamps the 100 MHz wall clock when it arrives at and
// when it is released from each device-wide barrier of the last launch
#define TRACE_ARRIVE() if (threadIdx.x == 0) D.trace[((k - A.bar_base - 1) * 2 + 0) * gridDim.x + blockIdx.x] = wall_clock64()
#define TRACE_RELEASE() if (threadIdx.x == 0) D.trace[((k - A.bar_base - 1) * 2 + 1) * gridDim.x + blockIdx.x] = wall_clock64()
#else
#define TRACE_ARRIVE()
#define TRACE_RELEASE()
#endif

// Persistent mode: one launch per token.  The phase functions are inlined into one loop body
// (as separate functions every call saved and restored ~100 registers per lane).  The
// device-wide barrier that PRECEDES a phase is executed inside that phase's function, and
// the phase's first weight loads are issued between arriving at and waiting on it, so they
// are in flight while the workgroups synchronise.  k is the index of that barrier (0: none,
// first phase of the launch).
#ifndef RIVER_PSTEP_INLINE
#define RIVER_PSTEP_INLINE __forceinline__
#endif
__device__ __forceinline__ int pack_ctl(const Ctl &c) { return (c.exit_pos << 1) | (c.river ? 1 : 0); }
__device__ __forceinline__ Ctl unpack_ctl(int v) { Ctl c; c.river = v & 1; c.exit_pos = v >> 1; return c; }

template <int DT>
__device__ RIVER_PSTEP_INLINE int pstep_qkv(const Dev *Dp, StepArgs A, int l, int ctl_packed,
                                      unsigned long long k, float *lds) {
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  Ctl ctl = unpack_ctl(ctl_packed);
  Pre<DT> pre;
  // block l (1-based) has just run: what will block l + 1 run as, as far as known now
  const bool guess = (l == 0) ? ctl.river : guess_river_after(A, ctl, l);
  if (l > 0) { barrier_arrive(D.bar, k); TRACE_ARRIVE(); }
  prefetch_phase<DT>(D, l, PH_QKV, guess, pre, l > 0 ? 0 : 2);
  bool late_part = false;                 // the late part of the prefetch is still to be issued
  if (l > 0) {
    barrier_wait(D.bar, k, D.spin_limit, D.bar_vector_poll); TRACE_RELEASE();
    exit_test(D, A, l, ctl, lds);
    if (ctl.river != guess) prefetch_phase<DT>(D, l, PH_QKV, ctl.river, pre);   // wrong guess: everything again
    else late_part = true;
  }
  const bool rv = ctl.river;
  phase_qkv<DT>(D, A, l, rv, lds, pre, [&] { if (late_part) prefetch_phase<DT>(D, l, PH_QKV, rv, pre, 1); });
  return pack_ctl(ctl);
}
template <int DT, bool F16>
__device__ RIVER_PSTEP_INLINE void pstep_attn(const Dev *Dp, StepArgs A, int l, int ctl_packed, unsigned long long k,
                                        float *lds) {
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  phase_attn<DT, F16>(D, A, l, unpack_ctl(ctl_packed), lds, [&] { barrier_arrive(D.bar, k); TRACE_ARRIVE(); },
                 [&] { barrier_wait(D.bar, k, D.spin_limit, D.bar_vector_poll); TRACE_RELEASE(); });
}
template <int DT, int PH>
__device__ RIVER_PSTEP_INLINE void pstep_gemv(const Dev *Dp, StepArgs A, int l, bool river, unsigned long long k,
                                        float *lds) {
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  Pre<DT> pre;
  barrier_arrive(D.bar, k); TRACE_ARRIVE();
  prefetch_phase<DT>(D, l, PH, river, pre, 0);
  barrier_wait(D.bar, k, D.spin_limit, D.bar_vector_poll); TRACE_RELEASE();
  // the late part of the prefetch goes out behind the first loads of the phase's input vector
  auto late = [&] { prefetch_phase<DT>(D, l, PH, river, pre, 1); };
  if (PH == PH_O) phase_oproj<DT>(D, A, l, river, lds, pre, late);
  else if (PH == PH_GU) phase_gateup<DT>(D, A, l, river, lds, pre, late);
  else phase_down<DT>(D, A, l, river, lds, pre, late);
}
template <int DT>
__device__ RIVER_PSTEP_INLINE void pstep_head(const Dev *Dp, StepArgs A, int ctl_packed, unsigned long long k,
                                        float *lds) {
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  const Ctl ctl = unpack_ctl(ctl_packed);
  Pre<DT> pre;
  barrier_arrive(D.bar, k); TRACE_ARRIVE();
  prefetch_head<DT>(D, pre, 0);
  barrier_wait(D.bar, k, D.spin_limit, D.bar_vector_poll); TRACE_RELEASE();
  phase_head<DT>(D, A, ctl, lds, pre, [&] { prefetch_head<DT>(D, pre, 1); });
}

// The number of barriers (5 L - 1, one more with the head) is the same for every workgroup
// whatever the exit state.
template <int DT, bool F16>
__global__ __launch_bounds__(kBlock) void k_step_persistent(const Dev *Dp, StepArgs A) {
  extern __shared__ float lds[];
  DevRef D = *RIVER_CONSTANT(Dev, Dp);
  unsigned long long k = A.bar_base;
  const int L = D.L;
  record_init(D, A);
  int ctl = pack_ctl(ctl_init(D, A));
  for (int l = 0; l < L; ++l) {
    ctl = pstep_qkv<DT>(Dp, A, l, ctl, l ? ++k : 0, lds);
    const bool river = ctl & 1;
    pstep_attn<DT, F16>(Dp, A, l, ctl, ++k, lds);
    pstep_gemv<DT, PH_O>(Dp, A, l, river, ++k, lds);
    pstep_gemv<DT, PH_GU>(Dp, A, l, river, ++k, lds);
    pstep_gemv<DT, PH_DOWN>(Dp, A, l, river, ++k, lds);
  }
  if (A.want_head) pstep_head<DT>(Dp, A, ctl, ++k, lds);
}

// Interleaves the river's scale and zero arrays into one (scale, zero) pair per group,
// so that a lane fetches both with one load.
template <int DT>
__global__ void k_pack_sz(const void *scale, const void *zero, void *out, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n)
    ((typename Store<DT>::SZ *)out)[i] = Store<DT>::pack(Store<DT>::ld(scale, i), Store<DT>::ld(zero, i));
}

// River construction: one thread per quantisation group.
template <int DT>
__global__ void k_quantize_w4(const void *w, long long rows, int cols, int group, uint8_t *codes,
                              void *scale, void *zero) {
  const int gpr = (cols + group - 1) / group;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * gpr) return;
  const long long r = idx / gpr;
  const int g = (int)(idx % gpr);
  const int c0 = g * group;
  const int glen = min(group, cols - c0);
  const size_t base = (size_t)r * cols + c0;
  float mn = Store<DT>::ld(w, base), mx = mn;
  for (int i = 1; i < glen; ++i) {
    const float v = Store<DT>::ld(w, base + i);
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  }
  float s = (mx > mn) ? (mx - mn) / 15.0f : 1.0f;
  Store<DT>::st(scale, idx, s);
  s = Store<DT>::ld(scale, idx);              // the stored (rounded) value defines the grid
  float z = -mn / s;
  Store<DT>::st(zero, idx, z);
  z = Store<DT>::ld(zero, idx);
  for (int i = 0; i < glen; i += 2) {
    int q[2];
    for (int k = 0; k < 2; ++k) {
      const float t = rintf(Store<DT>::ld(w, base + i + k) / s + z);
      q[k] = t < 0.f ? 0 : (t > 15.f ? 15 : (int)t);
    }
    codes[(base + i) >> 1] = (uint8_t)(q[0] | (q[1] << 4));
  }
}

__global__ void k_fill_bytes(uint4 *p, size_t n16, uint32_t word) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (size_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(word, word, word, word);
}

// ------------------------------------------------------------------ context

struct Layout {
  size_t kcache, vcache, rope, hidden, qbuf, obuf, kvcur, h1, abuf, logits, part_o, part_ml, cos_part,
      amax_val, amax_idx, state, rec_token, rec_exit, rec_sims, layers, dev, trace, qsz, total;
  size_t cache_bytes, qsz_bytes;
  size_t bd_partial;                     // [kBdKSplit][32][d_model] partial sums of the K-sliced GEMMs
  size_t bd_ssq;
  size_t bd_stream, bd_stream_bytes;     // batched contexts: the GEMM weights a second time, in stream order (bd::BdB)
  // activation buffers of the GEMM prefill (pf_rows rows each; 0 rows: that path is not offered)
  size_t pf_tok, pf_h, pf_x16, pf_q16, pf_a16, pf_big;
  int pf_rows;
  // batched contexts (max_batch > 1): per-sequence state, step buffers, records
  size_t bd_state, bd_hprev, bd_part_o, bd_part_ml, bd_tickets, bd_logits, bd_hist, bd_rec_token, bd_rec_exit,
      bd_rec_sims;
};


// Barrier blocks that are polled with scalar loads live in uncached device memory, which is
// allocated once per device and process and never freed (freeing uncached memory that a
// kernel has read is not safe on all systems); contexts take and return slots of it.
namespace {
constexpr int kBarSlots = 64, kBarDevices = 16;
std::mutex g_bar_mu;
char *g_bar_pool[kBarDevices];
unsigned long long g_bar_used[kBarDevices];
}
// Static scratch for river_create_static: the step-transient part of the workspace
// (activations, partial results, counters, records, descriptor tables) and the barrier
// block, for callers that must not allocate.  Each device holds its own copy of the array;
// host code uses the per-device address from hipGetSymbolAddress, never the array's name.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
namespace {
char *g_static_ptr[kBarDevices];          // device address of g_static_scratch, per device
bool g_static_live[kBarDevices];          // a live context uses the device's scratch
}
// Address of the current device's copy of the static scratch (looked up once per device).
static int static_scratch_ptr(int dev, char **ptr, std::string *why) {
  std::lock_guard<std::mutex> lk(g_bar_mu);
  if (dev < 0 || dev >= kBarDevices) { *why = "device index too large for the static scratch table"; return RIVER_EINVAL; }
  if (!g_static_ptr[dev]) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess || !p) {
      *why = std::string("hipGetSymbolAddress(static scratch): ") + hipGetErrorString(e);
      return RIVER_EHIP;
    }
    g_static_ptr[dev] = (char *)p;
  }
  *ptr = g_static_ptr[dev];
  return RIVER_OK;
}

static int bar_acquire(int dev, int *slot, char **ptr, std::string *why) {
  std::lock_guard<std::mutex> lk(g_bar_mu);
  if (dev < 0 || dev >= kBarDevices) { *why = "device index too large for the barrier pool"; return RIVER_EINVAL; }
  if (!g_bar_pool[dev]) {
    void *p = nullptr;
    const hipError_t e = hipExtMallocWithFlags(&p, (size_t)kBarSlots * kBarBytes, hipDeviceMallocUncached);
    if (e != hipSuccess) { *why = std::string("uncached barrier pool: ") + hipGetErrorString(e); return RIVER_EHIP; }
    g_bar_pool[dev] = (char *)p;
  }
  for (int i = 0; i < kBarSlots; ++i)
    if (!(g_bar_used[dev] >> i & 1ull)) {
      g_bar_used[dev] |= 1ull << i;
      *slot = i;
      *ptr = g_bar_pool[dev] + (size_t)i * kBarBytes;
      return RIVER_OK;
    }
  *why = "more than 64 live contexts on one device";
  return RIVER_ENOSPC;
}
static void bar_release(int dev, int slot) {
  std::lock_guard<std::mutex> lk(g_bar_mu);
  if (slot >= 0) g_bar_used[dev] &= ~(1ull << slot);
}

struct river_ctx {
  river_config cfg;
  Dev dev;              // host copy of the descriptor
  const Dev *dev_d;     // the same in the workspace
  Layout lay;
  char *ws;
  hipStream_t stream;
  int pos;              // positions in the cache
  bool have_token;      // DevState::cur_token is valid
  bool have_river;
  long long steps;      // decode steps recorded so far
  unsigned long long bar_total;
  int bar_slot = -1;    // slot of the process-wide barrier pool
  int bar_device = 0;
  bool is_static = false; // activations and barrier block live in the device's static scratch
  ~river_ctx() {
    bar_release(bar_device, bar_slot);
    if (is_static) {
      std::lock_guard<std::mutex> lk(g_bar_mu);
      g_static_live[bar_device] = false;
    }
  }
  int grid_persist, grid_gemv, block;
  size_t lds_bytes;
  bool broken;
  std::string err;
  std::vector<DevLayer> layers_h;   // host copy of the per-block pointer table (GEMM prefill launches)
  std::vector<bd::BdB> bd_dense_h, bd_twin_h;   // [L][4] stream-order weights of the QKV / O / gate-up / down GEMMs
  bd::BdB bd_head;                  // (batched contexts; a twin that was not given: null)
  std::vector<int> pos_b;           // batched contexts: positions in the cache, per sequence
  long long steps_b = 0;            // batched decode steps recorded so far
  int last_n = 0;                   // sequences of the last batched step
  bd::SeqState st_b{};
};

static thread_local std::string g_create_err;

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Shapes the GEMM prefill handles: bf16 storage, every contraction length a multiple of the
// 64-column K tile, quantisation groups made of whole K tiles.
static bool gemm_prefill_ok(const river_config *c) {
  return c->dtype == RIVER_BF16 && c->d_model % 64 == 0 && c->d_ffn % 64 == 0 &&
         (c->n_q_heads * c->head_dim) % 64 == 0 && c->river_group % 64 == 0 && c->prefill_gemm_min_tokens >= 0;
}

static bool valid_cfg(const river_config *c, std::string *why) {
  auto bad = [&](const char *m) { if (why) *why = m; return false; };
  if (!c) return bad("null config");
  if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 1 ||
      c->vocab < 1 || c->max_seq < 1)
    return bad("non-positive dimension");
  if (c->dtype != RIVER_F32 && c->dtype != RIVER_BF16) return bad("dtype must be RIVER_F32 or RIVER_BF16");
  if (c->max_batch < 1 || c->max_batch > bd::kRows) return bad("max_batch must be in [1, 32]");
  if (c->batch_exit_rule != 0 && c->batch_exit_rule != 1) return bad("batch_exit_rule must be 0 or 1");
  if (c->river_bits != 4) return bad("river_bits must be 4");
  if (c->river_group < 32 || c->river_group % 32) return bad("river_group must be a multiple of 32");
  if (c->n_q_heads % c->n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
  const int hd = c->head_dim;
  if (hd != 64 && hd != 128) return bad("head_dim must be 64 or 128");
  if (c->d_model % 16 || c->d_ffn % 16) return bad("d_model and d_ffn must be multiples of 16");
  if (c->vocab % 2) return bad("vocab must be even");
  if (c->min_exit_layer < 0 || c->min_exit_layer > c->n_layers) return bad("min_exit_layer out of range");
  if (c->exec_mode != RIVER_EXEC_KERNELS && c->exec_mode != RIVER_EXEC_PERSISTENT) return bad("bad exec_mode");
  if (c->exec_mode == RIVER_EXEC_PERSISTENT && c->dtype != RIVER_BF16)
    return bad("RIVER_EXEC_PERSISTENT is available for RIVER_BF16 only; use RIVER_EXEC_KERNELS for RIVER_F32");
  if (c->spin_limit < 0) return bad("negative spin_limit");
  if (c->kv_dtype != RIVER_KV_SAME && c->kv_dtype != RIVER_KV_F16) return bad("bad kv_dtype");
  if (c->kv_dtype == RIVER_KV_F16 && c->dtype != RIVER_BF16) return bad("RIVER_KV_F16 needs RIVER_BF16 weights");
  if (!(c->rope_base > 0.f) || !(c->rms_eps >= 0.f)) return bad("bad rope_base / rms_eps");
  if (c->max_batch > 1) {
    if (!gemm_prefill_ok(c))
      return bad("max_batch > 1 needs RIVER_BF16 with d_model, d_ffn and river_group multiples of 64 and the GEMM "
                 "prefill enabled");
  }
  return true;
}


static int x_capacity(const river_config *c) {
  int cap = c->d_model;
  cap = std::max(cap, c->n_q_heads * c->head_dim);
  cap = std::max(cap, c->d_ffn);
  cap = std::max(cap, attn_lds_floats(c->head_dim));
  // the staged vector is stored granule-wise (64 lanes x up to 32 columns): whole granules
  return (int)align_up(cap, 2048);
}

// [rows, cols] of block matrix m (wq wk wv wo w_gate w_up w_down)
static void matrix_shape(const river_config *c, int m, long long *rows, long long *cols) {
  const long long q = (long long)c->n_q_heads * c->head_dim, kv = (long long)c->n_kv_heads * c->head_dim;
  const long long d = c->d_model, f = c->d_ffn;
  const long long R[7] = {q, kv, kv, d, f, f, d}, C[7] = {d, d, d, q, d, d, f};
  *rows = R[m];
  *cols = C[m];
}
static size_t qsz_matrix_bytes(const river_config *c, int m) {
  long long rows, cols;
  matrix_shape(c, m, &rows, &cols);
  const long long gpr = (cols + c->river_group - 1) / c->river_group;
  return (size_t)(rows * gpr) * (c->dtype == RIVER_BF16 ? 4 : 8);
}

// The four GEMMs of a block in a batched step: matrices (stacked along N, or interleaved), N, K
struct BdGemmShape { int ms[3], nm, interleaved, N, K; };
static BdGemmShape bd_gemm_shape(const river_config *c, int g) {
  const int q = c->n_q_heads * c->head_dim, kv = c->n_kv_heads * c->head_dim, d = c->d_model, f = c->d_ffn;
  switch (g) {
    case 0: return {{M_WQ, M_WK, M_WV}, 3, 0, q + 2 * kv, d};
    case 1: return {{M_WO, M_WO, M_WO}, 1, 0, d, q};
    case 2: return {{M_GATE, M_UP, M_UP}, 2, 1, 2 * f, d};
    default: return {{M_DOWN, M_DOWN, M_DOWN}, 1, 0, d, f};
  }
}
static size_t bd_stream_bytes_of(const river_config *c) {
  size_t per_block = 0;
  for (int g = 0; g < 4; ++g) {
    const BdGemmShape sh = bd_gemm_shape(c, g);
    per_block += align_up(bd::bd_dense_bytes(sh.N, sh.K), 256) + align_up(bd::bd_codes_bytes(sh.N, sh.K), 256) +
                 align_up(bd::bd_pairs_bytes(sh.N, sh.K), 256);
  }
  return per_block * (size_t)c->n_layers + align_up(bd::bd_dense_bytes(c->vocab, c->d_model), 256);
}

static Layout make_layout(const river_config *c) {
  Layout y{};
  const size_t es = c->dtype == RIVER_BF16 ? 2 : 4;
  const size_t kvd = (size_t)c->n_kv_heads * c->head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  y.cache_bytes = (size_t)c->n_layers * c->max_seq * kvd * es;      // one sequence
  y.kcache = take(y.cache_bytes * c->max_batch);
  y.vcache = take(y.cache_bytes * c->max_batch);
  y.rope = take((size_t)c->max_seq * (c->head_dim / 2) * sizeof(float2));
  y.hidden = take((size_t)(c->n_layers + 1) * c->d_model * 4);
  y.qbuf = take((size_t)c->n_q_heads * c->head_dim * 4);
  y.obuf = take((size_t)c->n_q_heads * c->head_dim * 4);
  y.kvcur = take((size_t)2 * kvd * 4);
  y.h1 = take((size_t)c->d_model * 4);
  y.abuf = take((size_t)c->d_ffn * 4);
  y.logits = take((size_t)c->vocab * 4);
  y.part_o = take((size_t)c->n_q_heads * kMaxSplits * c->head_dim * 4);
  y.part_ml = take((size_t)c->n_q_heads * kMaxSplits * 4 * 4);
  y.cos_part = take((size_t)kMaxGrid * 4 * 4);
  y.amax_val = take((size_t)kMaxGrid * 4);
  y.amax_idx = take((size_t)kMaxGrid * 4);
  y.state = take(sizeof(DevState));
  y.rec_token = take((size_t)kRecords * 4);
  y.rec_exit = take((size_t)kRecords * 4);
  y.rec_sims = take((size_t)kRecords * c->n_layers * 4);
  y.layers = take((size_t)c->n_layers * sizeof(DevLayer));
  y.dev = take(sizeof(Dev));
  y.trace = take(((size_t)5 * c->n_layers * 2 * kMaxGrid + 64) * 8);
  // packed (scale, zero) pairs of every river matrix of every block
  y.qsz_bytes = 0;
  for (int m = 0; m < 7; ++m) y.qsz_bytes += align_up(qsz_matrix_bytes(c, m), 256);
  y.qsz_bytes *= (size_t)c->n_layers;
  y.qsz = take(y.qsz_bytes);
  y.pf_rows = 0;
  if (gemm_prefill_ok(c)) {
    const size_t rows = align_up((size_t)std::min(c->max_seq, pf::kChunk), 128);
    const size_t qd = (size_t)c->n_q_heads * c->head_dim;
    y.pf_rows = (int)rows;
    y.pf_tok = take(rows * 4);
    y.pf_h = take(rows * c->d_model * 4);
    y.pf_x16 = take(rows * std::max((size_t)c->d_model, qd) * 2);
    y.pf_q16 = take(rows * qd * 2);
    y.pf_a16 = take(rows * c->d_ffn * 2);
    y.pf_big = take(rows * std::max((size_t)2 * c->d_ffn, qd + 2 * kvd) * 4);
  }
  if (c->max_batch > 1) {
    const size_t B = c->max_batch, qd = (size_t)c->n_q_heads * c->head_dim;
    y.bd_state = take(6 * B * 4);
    y.bd_hprev = take((size_t)bd::kRows * c->d_model * 4);
    y.bd_part_o = take((size_t)bd::kRows * qd * bd::kBdAttnMaxSplits * 4);      // attention split partials
    y.bd_part_ml = take((size_t)bd::kRows * std::max(c->n_q_heads * bd::kBdAttnMaxSplits, bd::kBdArgmaxChunks) * 2 * 4);  // (also the argmax partials)
    y.bd_tickets = take((size_t)bd::kRows * c->n_q_heads * 4);
    y.bd_logits = take(B * c->vocab * 4);
    y.bd_hist = take((size_t)(c->n_layers + 1) * B * c->d_model * 4);
    y.bd_rec_token = take((size_t)bd::kRecordsB * B * 4);
    y.bd_rec_exit = take((size_t)bd::kRecordsB * B * 4);
    y.bd_rec_sims = take((size_t)bd::kRecordsB * B * c->n_layers * 4);
    y.bd_partial = take((size_t)bd::kBdKSplit * bd::kRows * c->d_model * 4);
    y.bd_ssq = take((size_t)kMaxGrid * bd::kRows * 4);                          // sums of squares per GEMM workgroup and row
    y.bd_stream_bytes = bd_stream_bytes_of(c);
    y.bd_stream = take(y.bd_stream_bytes);
  }
  y.total = off;
  return y;
}

#define HIP_TRY(ctx, expr)                                                              \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) {                                                             \
      (ctx)->err = std::string(#expr) + ": " + hipGetErrorString(e_);                   \
      (ctx)->broken = true;                                                             \
      return RIVER_EHIP;                                                                \
    }                                                                                   \
  } while (0)

extern "C" size_t river_workspace_bytes(const river_config *cfg) {
  if (!valid_cfg(cfg, nullptr)) return 0;
  return make_layout(cfg).total;
}

extern "C" int river_quantize_w4(const void *w, int64_t rows, int64_t cols, int32_t group,
                                 int32_t dtype, void *codes, void *scale, void *zero,
                                 void *hip_stream) {
  if (!w || !codes || !scale || !zero || rows < 1 || cols < 16 || cols % 16 || group < 32 ||
      group % 32 || cols > (1 << 30) || (dtype != RIVER_F32 && dtype != RIVER_BF16))
    return RIVER_EINVAL;
  const long long gpr = (cols + group - 1) / group;
  const long long n = rows * gpr;
  const int bs = 256;
  const long long nb = (n + bs - 1) / bs;
  if (nb > 0x7fffffffLL) return RIVER_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  if (dtype == RIVER_BF16)
    k_quantize_w4<1><<<dim3((unsigned)nb), dim3(bs), 0, st>>>(w, rows, (int)cols, group,
                                                               (uint8_t *)codes, scale, zero);
  else
    k_quantize_w4<0><<<dim3((unsigned)nb), dim3(bs), 0, st>>>(w, rows, (int)cols, group,
                                                               (uint8_t *)codes, scale, zero);
  return hipGetLastError() == hipSuccess ? RIVER_OK : RIVER_EHIP;
}

static int reset_state(river_ctx *x) {
  HIP_TRY(x, hipMemsetAsync(x->ws + x->lay.state, 0, sizeof(DevState), x->stream));
  HIP_TRY(x, hipMemsetAsync(x->dev.bar, 0, kBarBytes, x->stream));
  x->bar_total = 0;
  return RIVER_OK;
}

static int create_impl(const river_config *cfg, const river_weights *w, const river_qweights *q,
                       void *workspace, size_t workspace_bytes, void *hip_stream, river_ctx **out,
                       bool use_static) {
  std::string why;
  if (!out) { g_create_err = "null out"; return RIVER_EINVAL; }
  *out = nullptr;
  if (!valid_cfg(cfg, &why)) { g_create_err = why; return RIVER_EINVAL; }
  if (!w || !workspace) { g_create_err = "null weights or workspace"; return RIVER_EINVAL; }
  if (((uintptr_t)workspace) % 256) { g_create_err = "workspace must be 256-byte aligned"; return RIVER_EINVAL; }
  if (!w->tok_emb || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wq || !w->wk || !w->wv ||
      !w->wo || !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down) {
    g_create_err = "null weight table";
    return RIVER_EINVAL;
  }
  const int L = cfg->n_layers;
  const void *const *tabs[9] = {w->attn_norm, w->ffn_norm, w->wq, w->wk, w->wv, w->wo,
                                w->w_gate, w->w_up, w->w_down};
  for (int l = 0; l < L; ++l)
    for (int t = 0; t < 9; ++t)
      if (!tabs[t][l] || ((uintptr_t)tabs[t][l]) % 16) {
        g_create_err = "null or misaligned (16 B) layer weight";
        return RIVER_EINVAL;
      }
  Layout lay = make_layout(cfg);
  if (workspace_bytes < lay.total) { g_create_err = "workspace too small"; return RIVER_ENOSPC; }

  river_ctx *x = new river_ctx();
  x->cfg = *cfg;
  x->lay = lay;
  x->ws = (char *)workspace;
  x->stream = (hipStream_t)hip_stream;
  x->pos = 0;
  x->have_token = false;
  x->steps = 0;
  x->bar_total = 0;
  x->broken = false;
  x->block = kBlock;

  // river twins: a block's twin is usable only if all its 21 pointers are given
  std::vector<DevLayer> hl(L);
  std::vector<const void *> hqs((size_t)L * 7, nullptr), hqz((size_t)L * 7, nullptr);
  x->have_river = q != nullptr;
  for (int l = 0; l < L; ++l) {
    DevLayer &d = hl[l];
    d.attn_norm = w->attn_norm[l];
    d.ffn_norm = w->ffn_norm[l];
    d.w[0] = w->wq[l]; d.w[1] = w->wk[l]; d.w[2] = w->wv[l]; d.w[3] = w->wo[l];
    d.w[4] = w->w_gate[l]; d.w[5] = w->w_up[l]; d.w[6] = w->w_down[l];
    for (int m = 0; m < 7; ++m) {
      d.qc[m] = nullptr; d.qsz[m] = nullptr;
      if (q && q->codes[m] && q->scale[m] && q->zero[m]) {
        d.qc[m] = (const uint8_t *)q->codes[m][l];
        hqs[(size_t)l * 7 + m] = q->scale[m][l];
        hqz[(size_t)l * 7 + m] = q->zero[m][l];
        if (((uintptr_t)d.qc[m]) % 16) {
          g_create_err = "misaligned (16 B) river codes";
          delete x;
          return RIVER_EINVAL;
        }
      }
    }
  }
  // blocks above L_s must have a complete twin if a river is given at all
  if (q)
    for (int l = std::max(cfg->min_exit_layer, 0); l < L; ++l)
      for (int m = 0; m < 7; ++m)
        if (!hl[l].qc[m] || !hqs[(size_t)l * 7 + m] || !hqz[(size_t)l * 7 + m]) {
          g_create_err = "river twin missing for a block above min_exit_layer";
          delete x;
          return RIVER_EINVAL;
        }

  int dev_id = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev_id) != hipSuccess || hipGetDeviceProperties(&prop, dev_id) != hipSuccess) {
    g_create_err = "no HIP device";
    delete x;
    return RIVER_EHIP;
  }
  const int cus = prop.multiProcessorCount;
  // one workgroup per CU, a multiple of 8 (the device-wide barrier counts in 8 groups)
  x->grid_persist = std::max(8, std::min(cus, kMaxGrid) / 8 * 8);
  x->grid_gemv = x->grid_persist;

  // Where the step-transient part of the layout [hidden, qsz) lives: in the workspace, or in
  // the device's static scratch followed by the barrier block (`act + lay.X` addresses member
  // X of that part in both cases).
  char *act = x->ws;
  char *static_bar = nullptr;
  if (use_static) {
    const size_t need = (lay.qsz - lay.hidden) + kBarBytes;
    if (need > kStaticScratchBytes) {
      g_create_err = "configuration needs " + std::to_string(need) + " bytes of scratch; the static scratch of "
                     "river_create_static holds " + std::to_string(kStaticScratchBytes) + " (use river_create)";
      delete x;
      return RIVER_ENOSPC;
    }
    char *sp = nullptr;
    std::string why2;
    const int rc = static_scratch_ptr(dev_id, &sp, &why2);
    if (rc != RIVER_OK) { g_create_err = why2; delete x; return rc; }
    bool busy;
    {
      std::lock_guard<std::mutex> lk(g_bar_mu);
      busy = g_static_live[dev_id];
      if (!busy) g_static_live[dev_id] = true;
    }
    if (busy) {                 // (the context's destructor takes the same lock)
      g_create_err = "the static scratch of this device is in use by a live context";
      delete x;
      return RIVER_ESTATE;
    }
    x->is_static = true;
    x->bar_device = dev_id;
    act = sp - lay.hidden;
    static_bar = sp + (lay.qsz - lay.hidden);
  }

  Dev &D = x->dev;
  D.L = L; D.d = cfg->d_model; D.nq = cfg->n_q_heads; D.nkv = cfg->n_kv_heads; D.hd = cfg->head_dim;
  D.ffn = cfg->d_ffn; D.vocab = cfg->vocab; D.max_seq = cfg->max_seq; D.min_exit = cfg->min_exit_layer;
  D.group = cfg->river_group;
  D.kv_f16 = cfg->kv_dtype == RIVER_KV_F16 ? 1 : 0;
  D.spin_limit = cfg->spin_limit > 0 ? cfg->spin_limit : (1 << 22);
  D.xcap = x_capacity(cfg);
  D.eps = cfg->rms_eps; D.tau = cfg->tau;
  D.tok_emb = w->tok_emb; D.final_norm = w->final_norm; D.lm_head = w->lm_head;
  char *ws = x->ws;
  D.layers = (const DevLayer *)(act + lay.layers);
  D.kcache = ws + lay.kcache; D.vcache = ws + lay.vcache;
  D.rope = (const float2 *)(ws + lay.rope);
  D.hidden = (float *)(act + lay.hidden);
  D.qbuf = (float *)(act + lay.qbuf); D.obuf = (float *)(act + lay.obuf);
  D.kvcur = (float *)(act + lay.kvcur);
  D.h1 = (float *)(act + lay.h1); D.abuf = (float *)(act + lay.abuf);
  D.logits = (float *)(act + lay.logits);
  D.part_o = (float *)(act + lay.part_o); D.part_ml = (float *)(act + lay.part_ml);
  D.cos_part = (float *)(act + lay.cos_part);
  D.amax_val = (float *)(act + lay.amax_val); D.amax_idx = (int *)(act + lay.amax_idx);
  D.st = (DevState *)(act + lay.state);
  if (use_static) {
    // ordinary device memory: polled with device-coherent vector loads (see barrier_wait)
    D.bar = (unsigned long long *)static_bar;
    D.bar_vector_poll = 1;
  } else {
    char *bp = nullptr;
    std::string why2;
    x->bar_device = dev_id;
    const int rc = bar_acquire(dev_id, &x->bar_slot, &bp, &why2);
    if (rc != RIVER_OK) { g_create_err = why2; delete x; return rc; }
    D.bar = (unsigned long long *)bp;
    D.bar_vector_poll = 0;
  }
  D.rec_token = (int *)(act + lay.rec_token); D.rec_exit = (int *)(act + lay.rec_exit);
  D.rec_sims = (float *)(act + lay.rec_sims);
  D.trace = (unsigned long long *)(act + lay.trace);
  x->lds_bytes = ((size_t)D.xcap + lds_half_floats(D.xcap) + 64) * sizeof(float);

  // RoPE table in double precision: angle = pos * base^(-2i/hd)
  const int half = cfg->head_dim / 2;
  std::vector<float2> rope((size_t)cfg->max_seq * half);
  for (int i = 0; i < half; ++i) {
    const double th = std::pow((double)cfg->rope_base, -2.0 * i / cfg->head_dim);
    for (int p = 0; p < cfg->max_seq; ++p) {
      const double a = (double)p * th;
      rope[(size_t)p * half + i] = make_float2((float)std::cos(a), (float)std::sin(a));
    }
  }
  auto fail = [&](const char *what, hipError_t e) {
    g_create_err = std::string(what) + ": " + hipGetErrorString(e);
    delete x;
    return RIVER_EHIP;
  };
  hipError_t e;
  if ((e = hipMemcpyAsync(ws + lay.rope, rope.data(), rope.size() * sizeof(float2),
                          hipMemcpyHostToDevice, x->stream)) != hipSuccess)
    return fail("rope upload", e);
  x->dev_d = (const Dev *)(act + lay.dev);
  if ((e = hipMemcpyAsync(act + lay.dev, &x->dev, sizeof(Dev), hipMemcpyHostToDevice, x->stream)) != hipSuccess)
    return fail("descriptor upload", e);
  // pack (scale, zero) pairs of every river matrix that was given into the workspace
  {
    size_t off = lay.qsz;
    for (int l = 0; l < L; ++l)
      for (int m = 0; m < 7; ++m) {
        const size_t bytes = qsz_matrix_bytes(cfg, m);
        if (hl[l].qc[m] && hqs[(size_t)l * 7 + m] && hqz[(size_t)l * 7 + m]) {
          const long long n = (long long)(bytes / (cfg->dtype == RIVER_BF16 ? 4 : 8));
          const unsigned nb = (unsigned)((n + 255) / 256);
          if (cfg->dtype == RIVER_BF16)
            k_pack_sz<1><<<dim3(nb), dim3(256), 0, x->stream>>>(hqs[(size_t)l * 7 + m], hqz[(size_t)l * 7 + m], ws + off, n);
          else
            k_pack_sz<0><<<dim3(nb), dim3(256), 0, x->stream>>>(hqs[(size_t)l * 7 + m], hqz[(size_t)l * 7 + m], ws + off, n);
          hl[l].qsz[m] = ws + off;
        }
        off += align_up(bytes, 256);
      }
    if ((e = hipGetLastError()) != hipSuccess) return fail("river (scale, zero) packing", e);
  }
  // batched contexts: the GEMM weights a second time, in the order the batched GEMM streams them
  x->bd_dense_h.assign((size_t)L * 4, bd::BdB{nullptr, nullptr});
  x->bd_twin_h.assign((size_t)L * 4, bd::BdB{nullptr, nullptr});
  x->bd_head = bd::BdB{nullptr, nullptr};
  if (cfg->max_batch > 1) {
    size_t off = lay.bd_stream;
    auto blocks_of = [](size_t pieces) { return dim3((unsigned)((pieces + 255) / 256)); };
    for (int l = 0; l <= L; ++l)
      for (int g = 0; g < (l < L ? 4 : 1); ++g) {
        pf::GemmB Bw{}, Bc{}, Bs{};
        BdGemmShape sh = bd_gemm_shape(cfg, g);
        bool twin = l < L;
        if (l == L) {                                         // the LM head
          sh = BdGemmShape{{0, 0, 0}, 1, 0, cfg->vocab, cfg->d_model};
          Bw.w[0] = Bw.w[1] = Bw.w[2] = w->lm_head;
          Bw.rows[0] = cfg->vocab;
        } else {
          for (int i = 0; i < 3; ++i) {
            const int m = sh.ms[i < sh.nm ? i : 0];
            long long r, cc;
            matrix_shape(cfg, m, &r, &cc);
            Bw.w[i] = hl[l].w[m];
            Bc.w[i] = hl[l].qc[m];
            Bs.w[i] = hqs[(size_t)l * 7 + m];
            Bs.sz[i] = hqz[(size_t)l * 7 + m];
            Bw.rows[i] = Bc.rows[i] = Bs.rows[i] = i < sh.nm ? (int)r : 0;
            twin = twin && Bc.w[i] && Bs.w[i] && Bs.sz[i];
          }
        }
        const size_t units = bd::bd_units(sh.N);
        bd::k_bd_pack_dense<<<blocks_of(units * (sh.K / 64) * 64), dim3(256), 0, x->stream>>>(
            Bw, sh.interleaved, sh.N, sh.K, (uint4 *)(ws + off));
        bd::BdB dense{ws + off, nullptr};
        off += align_up(bd::bd_dense_bytes(sh.N, sh.K), 256);
        if (l == L) { x->bd_head = dense; break; }
        x->bd_dense_h[(size_t)l * 4 + g] = dense;
        const size_t cb = align_up(bd::bd_codes_bytes(sh.N, sh.K), 256), pb = align_up(bd::bd_pairs_bytes(sh.N, sh.K), 256);
        if (twin) {
          const size_t nkt = (size_t)(sh.K + 127) / 128;
          bd::k_bd_pack_codes<<<blocks_of(units * nkt * 32), dim3(256), 0, x->stream>>>(
              Bc, sh.interleaved, sh.N, sh.K, (uint4 *)(ws + off));
          bd::k_bd_pack_pairs<<<blocks_of(units * nkt * 16), dim3(256), 0, x->stream>>>(
              Bs, sh.interleaved, sh.N, sh.K, cfg->river_group, (uint32_t *)(ws + off + cb));
          x->bd_twin_h[(size_t)l * 4 + g] = bd::BdB{ws + off, ws + off + cb};
        }
        off += cb + pb;
      }
    if ((e = hipGetLastError()) != hipSuccess) return fail("stream-order weight packing", e);
  }
  x->layers_h = hl;
  x->pos_b.assign(cfg->max_batch, 0);
  if (cfg->max_batch > 1) {
    int *sp = (int *)(ws + lay.bd_state);
    const int B = cfg->max_batch;
    x->st_b.pos = sp; x->st_b.token = sp + B; x->st_b.river = sp + 2 * B; x->st_b.exit_pos = sp + 3 * B;
    x->st_b.forced = sp + 4 * B;
    if ((e = hipMemsetAsync(ws + lay.bd_state, 0, (size_t)6 * B * 4, x->stream)) != hipSuccess)
      return fail("sequence state clear", e);
    if ((e = hipMemsetAsync(ws + lay.bd_tickets, 0, (size_t)bd::kRows * cfg->n_q_heads * 4, x->stream)) != hipSuccess)
      return fail("attention ticket clear", e);
  }
  if ((e = hipMemcpyAsync(act + lay.layers, hl.data(), hl.size() * sizeof(DevLayer),
                          hipMemcpyHostToDevice, x->stream)) != hipSuccess)
    return fail("layer table upload", e);
  // everything after the caches starts at zero (state, counters, records, activations); the
  // static scratch keeps the previous context's contents, so this clear is what resets it
  if ((e = hipMemsetAsync(act + lay.hidden, 0, lay.layers - lay.hidden, x->stream)) != hipSuccess)
    return fail("workspace clear", e);
  if (use_static && (e = hipMemsetAsync(static_bar, 0, kBarBytes, x->stream)) != hipSuccess)
    return fail("barrier block clear", e);
  if ((e = hipMemsetAsync(ws + lay.kcache, 0, lay.vcache - lay.kcache + align_up(lay.cache_bytes * cfg->max_batch, 256),
                          x->stream)) != hipSuccess)
    return fail("cache clear", e);
  if ((e = hipStreamSynchronize(x->stream)) != hipSuccess) return fail("create sync", e);

  {
    const int lb = (int)x->lds_bytes;
    const void *fns[] = {
        (const void *)k_qkv<0>, (const void *)k_qkv<1>, (const void *)k_attn<0, false>,
        (const void *)k_attn<1, false>, (const void *)k_attn<1, true>,
        (const void *)k_oproj<0>, (const void *)k_oproj<1>, (const void *)k_gateup<0>,
        (const void *)k_gateup<1>, (const void *)k_down<0>, (const void *)k_down<1>,
        (const void *)k_head<0>, (const void *)k_head<1>, (const void *)k_step_persistent<1, false>,
        (const void *)k_step_persistent<1, true>};
    for (const void *f : fns)
      if ((e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lb)) != hipSuccess)
        return fail("hipFuncSetAttribute(max dynamic LDS)", e);
    if (gemm_prefill_ok(cfg)) {
      const void *pfg[] = {(const void *)pf::k_pf_gemm<false, false>, (const void *)pf::k_pf_gemm<false, true>,
                           (const void *)pf::k_pf_gemm<true, false>, (const void *)pf::k_pf_gemm<true, true>};
      for (const void *f : pfg)
        if ((e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, pf::kGemmLdsBytes)) != hipSuccess)
          return fail("hipFuncSetAttribute(prefill GEMM LDS)", e);
    }
    if (cfg->max_batch > 1) {
      // the widest batched GEMMs keep 64 KiB of partial tiles beside their static LDS
      if ((e = hipFuncSetAttribute((const void *)bd::k_bd_gemm<1, 8>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)bd::bd_gemm_lds_bytes(8, 1))) != hipSuccess ||
          (e = hipFuncSetAttribute((const void *)bd::k_bd_gemm<2, 4>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)bd::bd_gemm_lds_bytes(4, 2))) != hipSuccess)
        return fail("hipFuncSetAttribute(batched GEMM LDS)", e);
    }
  }
  *out = x;
  return RIVER_OK;
}

extern "C" int river_create(const river_config *cfg, const river_weights *w, const river_qweights *q,
                            void *workspace, size_t workspace_bytes, void *hip_stream,
                            river_ctx **out) {
  return create_impl(cfg, w, q, workspace, workspace_bytes, hip_stream, out, false);
}

extern "C" int river_create_static(const river_config *cfg, const river_weights *w, const river_qweights *q,
                                   void *workspace, size_t workspace_bytes, void *hip_stream,
                                   river_ctx **out) {
  return create_impl(cfg, w, q, workspace, workspace_bytes, hip_stream, out, true);
}

// Enqueue one token (prompt position or decode step).
template <int DT>
static int launch_step(river_ctx *x, const StepArgs &A0) {
  StepArgs A = A0;
  const Dev &D = x->dev;
  const Dev *Dp = x->dev_d;
  const dim3 blk(x->block);
  const size_t lds = x->lds_bytes;
  hipStream_t s = x->stream;
  if (x->cfg.exec_mode == RIVER_EXEC_PERSISTENT) {
    // bf16 only (river_create refuses the combination with fp32)
    if constexpr (DT == 1) {
      A.bar_base = x->bar_total;
      if (D.kv_f16) k_step_persistent<DT, true><<<dim3(x->grid_persist), blk, lds, s>>>(Dp, A);
      else k_step_persistent<DT, false><<<dim3(x->grid_persist), blk, lds, s>>>(Dp, A);
      x->bar_total += 5ull * D.L - 1 + (A.want_head ? 1 : 0);
    } else {
      x->err = "RIVER_EXEC_PERSISTENT is available for RIVER_BF16 only";
      return RIVER_EINVAL;
    }
  } else {
    const dim3 gg(x->grid_gemv);
    for (int l = 0; l < D.L; ++l) {
      k_qkv<DT><<<gg, blk, lds, s>>>(Dp, A, l);
      if (DT == 1 && D.kv_f16) k_attn<DT, DT == 1><<<gg, blk, lds, s>>>(Dp, A, l);
      else k_attn<DT, false><<<gg, blk, lds, s>>>(Dp, A, l);
      k_oproj<DT><<<gg, blk, lds, s>>>(Dp, A, l);
      k_gateup<DT><<<gg, blk, lds, s>>>(Dp, A, l);
      k_down<DT><<<gg, blk, lds, s>>>(Dp, A, l);
    }
    if (A.want_head) k_head<DT><<<gg, blk, lds, s>>>(Dp, A);
  }
  HIP_TRY(x, hipGetLastError());
  return RIVER_OK;
}

static int enqueue(river_ctx *x, int token, int forced_e, int want_head, int rec_slot) {
  StepArgs A{};
  A.pos = x->pos;
  A.token = token;
  A.forced_e = forced_e;
  A.want_head = want_head;
  A.rec_slot = rec_slot;
  const int T = x->pos + 1;
  // one workgroup per (query head, split); splits as far as there are workgroups for them
  const int max_splits = std::max(1, std::min(kMaxSplits, x->grid_persist / x->cfg.n_q_heads));
  // One split per kAttnPosPerSplit positions up to four splits; every further split costs each
  // consumer another read of all partial outputs, so beyond that a workgroup first takes
  // twice the positions (measured at contexts 768 .. 4096).
  int S = (T + kAttnPosPerSplit - 1) / kAttnPosPerSplit;
  if (S > 4) S = std::max(4, (T + 2 * kAttnPosPerSplit - 1) / (2 * kAttnPosPerSplit));
  A.n_splits = std::max(1, std::min(max_splits, S));
  A.bar_base = 0;
  const int rc = x->cfg.dtype == RIVER_BF16 ? launch_step<1>(x, A) : launch_step<0>(x, A);
  if (rc == RIVER_OK) x->pos += 1;
  return rc;
}

// After a synchronising call: did a bounded device wait give up?
static int check_device_error(river_ctx *x) {
  int err = 0;
  HIP_TRY(x, hipMemcpyAsync(&err, (char *)x->dev.bar + kBarErrorByte, sizeof(int),
                            hipMemcpyDeviceToHost, x->stream));
  HIP_TRY(x, hipStreamSynchronize(x->stream));
  if (err) {
    x->err = "a device-wide barrier wait exceeded spin_limit; results of the step are invalid";
    x->broken = true;
    return RIVER_EHIP;
  }
  return RIVER_OK;
}

#define CHECK_CTX(x)                                   \
  do {                                                 \
    if (!(x)) return RIVER_EINVAL;                     \
    if ((x)->broken) return RIVER_EHIP;                \
  } while (0)

// GEMM of the prefill: C[rows, N] (+)= A[rows, K] B^T over the stacked matrices ms[0..nm) of block l.
template <bool W4, bool ADD>
static void launch_gemm(river_ctx *x, int l, const int *ms, int nm, const _Float16 *A, int K, float *C, int rows) {
  pf::GemmB B{};
  int N = 0;
  for (int i = 0; i < nm; ++i) {
    long long r, c;
    matrix_shape(&x->cfg, ms[i], &r, &c);
    B.w[i] = W4 ? (const void *)x->layers_h[l].qc[ms[i]] : x->layers_h[l].w[ms[i]];
    B.sz[i] = x->layers_h[l].qsz[ms[i]];
    B.rows[i] = (int)r;
    N += (int)r;
  }
  for (int i = nm; i < 3; ++i) { B.w[i] = B.w[0]; B.sz[i] = B.sz[0]; B.rows[i] = 0; }
  const int n_tiles = (N + pf::TN - 1) / pf::TN, m_tiles = rows / pf::TM;
  const dim3 grid((n_tiles + 7) / 8 * 8 * m_tiles);            // (see the kernel's workgroup -> tile mapping)
  pf::k_pf_gemm<W4, ADD><<<grid, dim3(256), pf::kGemmLdsBytes, x->stream>>>(A, K, B, N, K, x->cfg.river_group, C, N,
                                                                            m_tiles);
}

// Prefill phase on the matrix cores: the prompt in chunks of up to pf_rows tokens, every block
// as MFMA GEMMs over the chunk (see river_prefill.h); blocks above ep run as river twins.
static int prefill_gemm(river_ctx *x, int seq, const int32_t *tokens, int n, int ep) {
  const river_config &c = x->cfg;
  const Dev &D = x->dev;
  const Layout &y = x->lay;
  hipStream_t s = x->stream;
  const int L = c.n_layers, d = c.d_model, qd = c.n_q_heads * c.head_dim, ffn = c.d_ffn;
  int *tok = (int *)(x->ws + y.pf_tok);
  float *h = (float *)(x->ws + y.pf_h), *big = (float *)(x->ws + y.pf_big);
  _Float16 *x16 = (_Float16 *)(x->ws + y.pf_x16), *q16 = (_Float16 *)(x->ws + y.pf_q16);
  _Float16 *a16 = (_Float16 *)(x->ws + y.pf_a16);
  char *kc = (char *)D.kcache + (size_t)seq * y.cache_bytes, *vc = (char *)D.vcache + (size_t)seq * y.cache_bytes;
  const int m_qkv[3] = {M_WQ, M_WK, M_WV}, m_o[1] = {M_WO}, m_gu[2] = {M_GATE, M_UP}, m_d[1] = {M_DOWN};
  for (int c0 = 0; c0 < n; c0 += y.pf_rows) {
    const int m = std::min(y.pf_rows, n - c0), rows = (m + 127) / 128 * 128;
    const bool last = c0 + m == n;
    HIP_TRY(x, hipMemcpyAsync(tok, tokens + c0, (size_t)m * 4, hipMemcpyHostToDevice, s));
    pf::k_pf_embed<<<dim3(m), dim3(256), 0, s>>>(tok, D.tok_emb, d, h);
    if (last) pf::k_pf_copy_row<<<dim3(4), dim3(256), 0, s>>>(h + (size_t)(m - 1) * d, D.hidden, d);
    for (int l = 0; l < L; ++l) {
      const bool river = l >= ep;
      const DevLayer &W = x->layers_h[l];
      pf::k_pf_rmsnorm<<<dim3(m), dim3(256), 0, s>>>(h, W.attn_norm, d, c.rms_eps, x16);
      if (river) launch_gemm<true, false>(x, l, m_qkv, 3, x16, d, big, rows);
      else launch_gemm<false, false>(x, l, m_qkv, 3, x16, d, big, rows);
      pf::k_pf_rope_store<<<dim3(m), dim3(256), 0, s>>>(big, D.rope, c.n_q_heads, c.n_kv_heads, c.head_dim, c0, l,
                                                        c.max_seq, kc, vc, D.kv_f16, q16);
      const dim3 ga(c.n_q_heads, (m + 127) / 128);
      if (c.head_dim == 128)
        pf::k_pf_attn<128><<<ga, dim3(256), 0, s>>>(q16, kc, vc, D.kv_f16, c.n_q_heads, c.n_kv_heads, l, c.max_seq,
                                                    c0, m, x16);
      else
        pf::k_pf_attn<64><<<ga, dim3(256), 0, s>>>(q16, kc, vc, D.kv_f16, c.n_q_heads, c.n_kv_heads, l, c.max_seq,
                                                   c0, m, x16);
      if (river) launch_gemm<true, true>(x, l, m_o, 1, x16, qd, h, rows);
      else launch_gemm<false, true>(x, l, m_o, 1, x16, qd, h, rows);
      pf::k_pf_rmsnorm<<<dim3(m), dim3(256), 0, s>>>(h, W.ffn_norm, d, c.rms_eps, x16);
      if (river) launch_gemm<true, false>(x, l, m_gu, 2, x16, d, big, rows);
      else launch_gemm<false, false>(x, l, m_gu, 2, x16, d, big, rows);
      pf::k_pf_swiglu<<<dim3(m), dim3(256), 0, s>>>(big, ffn, a16);
      if (river) launch_gemm<true, true>(x, l, m_d, 1, a16, ffn, h, rows);
      else launch_gemm<false, true>(x, l, m_d, 1, a16, ffn, h, rows);
      if (last)
        pf::k_pf_copy_row<<<dim3(4), dim3(256), 0, s>>>(h + (size_t)(m - 1) * d, D.hidden + (size_t)(l + 1) * d, d);
    }
    HIP_TRY(x, hipGetLastError());
  }
  // the original final norm + LM head + argmax on the last prompt position (the decode path's kernel)
  StepArgs A{};
  A.pos = n - 1; A.token = -1; A.forced_e = ep; A.want_head = 1; A.rec_slot = -1; A.n_splits = 1; A.bar_base = 0;
  k_head<1><<<dim3(x->grid_gemv), dim3(x->block), x->lds_bytes, s>>>(x->dev_d, A);
  if (c.max_batch > 1)
    bd::k_bd_after_prefill<<<dim3(1), dim3(64), 0, s>>>(x->st_b, seq, &D.st->cur_token, n);
  HIP_TRY(x, hipGetLastError());
  if (c.max_batch > 1) x->pos_b[seq] = n;
  else x->pos = n;
  return RIVER_OK;
}

extern "C" int river_prefill(river_ctx *x, int32_t seq, const int32_t *tokens, int32_t n_tokens,
                             int32_t prefill_exit_layer, int32_t *out_token, float *out_logits) {
  if (!x) return RIVER_EINVAL;
  if (seq < 0 || seq >= x->cfg.max_batch || !tokens || n_tokens < 1) {
    x->err = "bad prefill arguments";
    return RIVER_EINVAL;
  }
  if (n_tokens > x->cfg.max_seq) { x->err = "prompt longer than max_seq"; return RIVER_ENOSPC; }
  for (int i = 0; i < n_tokens; ++i)
    if (tokens[i] < 0 || tokens[i] >= x->cfg.vocab) { x->err = "token id out of range"; return RIVER_EINVAL; }
  const int L = x->cfg.n_layers;
  const int ep = prefill_exit_layer < 0 ? L : prefill_exit_layer;
  if (ep != L && (ep < x->cfg.min_exit_layer || ep > L)) {
    x->err = "prefill exit layer outside [L_s, L]";
    return RIVER_EINVAL;
  }
  if (ep < L && !x->have_river) { x->err = "prefill below full depth needs river weights"; return RIVER_ESTATE; }
  // a new sequence also clears a previous device-side time-out
  x->broken = false;
  int rc = reset_state(x);
  if (rc) return rc;
  x->pos = 0;
  x->have_token = false;
  const int min_gemm = x->cfg.prefill_gemm_min_tokens > 0 ? x->cfg.prefill_gemm_min_tokens : 32;
  if (x->lay.pf_rows > 0 && (n_tokens >= min_gemm || x->cfg.max_batch > 1)) {
    rc = prefill_gemm(x, seq, tokens, n_tokens, ep);
    if (rc) return rc;
  } else {
    // short prompts, fp32 models and shapes the GEMM path does not take: the decode kernels,
    // one prompt position after the other
    for (int i = 0; i < n_tokens; ++i) {
      rc = enqueue(x, tokens[i], ep, i == n_tokens - 1, -1);
      if (rc) return rc;
    }
  }
  if (out_logits)
    HIP_TRY(x, hipMemcpyAsync(out_logits, x->dev.logits, (size_t)x->cfg.vocab * 4, hipMemcpyDeviceToDevice,
                              x->stream));
  rc = check_device_error(x);
  if (rc) return rc;
  x->have_token = true;
  if (out_token) {
    HIP_TRY(x, hipMemcpyAsync(out_token, (char *)x->dev.st + offsetof(DevState, cur_token), sizeof(int),
                              hipMemcpyDeviceToHost, x->stream));
    HIP_TRY(x, hipStreamSynchronize(x->stream));
  }
  return RIVER_OK;
}

extern "C" int river_decode_step(river_ctx *x, const int32_t *in_token, const int32_t *forced_exit,
                                 int32_t *out_token, int32_t *out_exit_layer, float *out_sims) {
  CHECK_CTX(x);
  if (x->cfg.max_batch > 1) { x->err = "a batched context decodes with river_decode_batch"; return RIVER_ESTATE; }
  if (!x->have_token && !in_token) { x->err = "decode before prefill"; return RIVER_ESTATE; }
  if (x->pos < 1) { x->err = "decode before prefill"; return RIVER_ESTATE; }
  if (x->pos >= x->cfg.max_seq) { x->err = "KV cache full"; return RIVER_ENOSPC; }
  const int L = x->cfg.n_layers;
  int tok = -1, fe = -1;
  if (in_token) {
    tok = *in_token;
    if (tok < 0 || tok >= x->cfg.vocab) { x->err = "token id out of range"; return RIVER_EINVAL; }
  }
  if (forced_exit) {
    fe = *forced_exit;
    const bool ok = fe == L || (fe >= x->cfg.min_exit_layer && fe <= L && fe >= 0);
    if (!ok) { x->err = "forced exit position outside [L_s, L]"; return RIVER_EINVAL; }
  }
  if ((fe >= 0 && fe < L) || (fe < 0 && x->cfg.tau < 1.0f)) {
    if (!x->have_river) { x->err = "an exit is possible but no river weights were given"; return RIVER_ESTATE; }
  }
  if (!out_token && (out_exit_layer || out_sims)) {
    x->err = "out_token is NULL but other outputs are not";
    return RIVER_EINVAL;
  }
  const int slot = (int)(x->steps % kRecords);
  int rc = enqueue(x, tok, fe, 1, slot);
  if (rc) return rc;
  x->steps += 1;
  x->have_token = true;
  if (!out_token) return RIVER_OK;
  HIP_TRY(x, hipMemcpyAsync(out_token, x->dev.rec_token + slot, 4, hipMemcpyDeviceToHost, x->stream));
  if (out_exit_layer)
    HIP_TRY(x, hipMemcpyAsync(out_exit_layer, x->dev.rec_exit + slot, 4, hipMemcpyDeviceToHost, x->stream));
  if (out_sims)
    HIP_TRY(x, hipMemcpyAsync(out_sims, x->dev.rec_sims + (size_t)slot * L, (size_t)L * 4,
                              hipMemcpyDeviceToHost, x->stream));
  return check_device_error(x);
}

// GEMM g (QKV, O, gate/up, down) of block l of a batched decode step, or the LM head (Bq null,
// by_flag 0): bf16 matrices for the rows in the backbone, 4-bit twins for the others (see
// bd::k_bd_gemm).  The rows of B are dealt out to one workgroup per CU, eight at a time.
static int launch_bd_gemm_b(river_ctx *x, const bd::BdB &Bd, const bd::BdB &Bq, int N, const _Float16 *Af, int K,
                            void *C, int ldc, int epi, int by_flag, int n, bd::BdNorm nrm = bd::BdNorm{},
                            int *grid_out = nullptr) {
  // A matrix with at most 16 rows per CU (the down projection; the output projection, which also
  // prepares the next norm, stays whole) would have every workgroup
  // read the whole activation tile for a single row block; it is dealt out as K slices of four
  // times the rows instead, and the kernel that consumes the sum adds the partial sums up.
  int k_split = 1;
  if (epi == bd::EPI_ADD && N <= 16 * x->grid_persist && K >= 4096 && ldc == x->cfg.d_model) k_split = bd::kBdKSplit;
  // (the consumer of a fused norm adds up at most 16 * kSsqLoads partial sums per row)
  const int cus = epi == bd::EPI_ADD_NORM ? std::min(x->grid_persist, 16 * bd::kSsqLoads) : x->grid_persist;
  const int per_cu = (N * k_split + cus - 1) / cus;
  const int rows_per_wg = std::max(8, (per_cu + 7) / 8 * 8);
  const int blocks = (rows_per_wg + 15) / 16;
  const dim3 grid((N + rows_per_wg - 1) / rows_per_wg * k_split), blk(512);
  if (grid_out) *grid_out = (int)grid.x;
  hipStream_t s = x->stream;
  const int *rv = x->st_b.river;
  if (k_split > 1) { C = x->ws + x->lay.bd_partial; epi = bd::EPI_STORE; }
#define RIVER_BD_LAUNCH(MB, RBW)                                                                               \
  bd::k_bd_gemm<MB, RBW><<<grid, blk, bd::bd_gemm_lds_bytes(RBW, MB), s>>>(Af, Bd, Bq, N, K, C, ldc, epi, rv, \
                                                                          by_flag, n, rows_per_wg, k_split, nrm)
  if (n <= 16) {
    if (blocks <= 1) RIVER_BD_LAUNCH(1, 1);
    else if (blocks <= 2) RIVER_BD_LAUNCH(1, 2);
    else if (blocks <= 4) RIVER_BD_LAUNCH(1, 4);
    else RIVER_BD_LAUNCH(1, 8);
  } else {
    if (blocks <= 1) RIVER_BD_LAUNCH(2, 1);
    else if (blocks <= 2) RIVER_BD_LAUNCH(2, 2);
    else RIVER_BD_LAUNCH(2, 4);
  }
#undef RIVER_BD_LAUNCH
  return k_split > 1 ? k_split : 0;          // partial sums the consumer has to add
}
static int launch_bd_gemm(river_ctx *x, int l, int g, const _Float16 *Af, void *C, int ldc, int epi, int n,
                          bd::BdNorm nrm = bd::BdNorm{}, int *grid_out = nullptr) {
  const BdGemmShape sh = bd_gemm_shape(&x->cfg, g);
  return launch_bd_gemm_b(x, x->bd_dense_h[(size_t)l * 4 + g], x->bd_twin_h[(size_t)l * 4 + g], sh.N, Af, sh.K, C, ldc,
                          epi, 1, n, nrm, grid_out);
}

extern "C" int river_decode_batch(river_ctx *x, int32_t n_seq, const int32_t *in_tokens, const int32_t *forced_exit,
                                  int32_t *out_tokens, int32_t *out_exit_layers, float *out_sims) {
  CHECK_CTX(x);
  const river_config &c = x->cfg;
  if (c.max_batch < 2) { x->err = "river_decode_batch needs a context created with max_batch > 1"; return RIVER_ESTATE; }
  if (n_seq < 1 || n_seq > c.max_batch) { x->err = "n_seq outside [1, max_batch]"; return RIVER_EINVAL; }
  if (!out_tokens && (out_exit_layers || out_sims)) {
    x->err = "out_tokens is NULL but other outputs are not";
    return RIVER_EINVAL;
  }
  const int L = c.n_layers, n = n_seq;
  std::vector<int32_t> fe(n, -1);
  for (int b = 0; b < n; ++b) {
    if (x->pos_b[b] < 1) { x->err = "decode before prefill of every sequence"; return RIVER_ESTATE; }
    if (x->pos_b[b] >= c.max_seq) { x->err = "KV cache full"; return RIVER_ENOSPC; }
    if (in_tokens && (in_tokens[b] < 0 || in_tokens[b] >= c.vocab)) { x->err = "token id out of range"; return RIVER_EINVAL; }
    if (forced_exit) {
      fe[b] = forced_exit[b];
      const bool ok = fe[b] < 0 || fe[b] == L || (fe[b] >= c.min_exit_layer && fe[b] <= L);
      if (!ok) { x->err = "forced exit position outside [L_s, L]"; return RIVER_EINVAL; }
    }
    if (((fe[b] >= 0 && fe[b] < L) || (fe[b] < 0 && c.tau < 1.0f)) && !x->have_river) {
      x->err = "an exit is possible but no river weights were given";
      return RIVER_ESTATE;
    }
  }
  const Dev &D = x->dev;
  const Layout &y = x->lay;
  hipStream_t s = x->stream;
  const int d = c.d_model, qd = c.n_q_heads * c.head_dim, ffn = c.d_ffn;
  float *h = (float *)(x->ws + y.pf_h), *big = (float *)(x->ws + y.pf_big);
  float *hprev = (float *)(x->ws + y.bd_hprev);
  float *part_o = (float *)(x->ws + y.bd_part_o), *part_ml = (float *)(x->ws + y.bd_part_ml);
  unsigned int *tickets = (unsigned int *)(x->ws + y.bd_tickets);
  const float *partial = (const float *)(x->ws + y.bd_partial);
  float *logits = (float *)(x->ws + y.bd_logits), *hist = (float *)(x->ws + y.bd_hist);
  _Float16 *x16 = (_Float16 *)(x->ws + y.pf_x16), *o16 = (_Float16 *)(x->ws + y.pf_q16);
  _Float16 *a16 = (_Float16 *)(x->ws + y.pf_a16);
  const int slot = (int)(x->steps_b % bd::kRecordsB);
  const size_t B = c.max_batch;
  int *rec_token = (int *)(x->ws + y.bd_rec_token) + (size_t)slot * B;
  int *rec_exit = (int *)(x->ws + y.bd_rec_exit) + (size_t)slot * B;
  float *rec_sims = (float *)(x->ws + y.bd_rec_sims) + (size_t)slot * B * L;
  const bd::SeqState st = x->st_b;
  float *s_of = (float *)(st.forced + B);                    // [max_batch] similarities of the current block
  HIP_TRY(x, hipMemcpyAsync(st.forced, fe.data(), (size_t)n * 4, hipMemcpyHostToDevice, s));
  if (in_tokens) HIP_TRY(x, hipMemcpyAsync(st.token, in_tokens, (size_t)n * 4, hipMemcpyHostToDevice, s));
  bd::k_bd_fill_nan<<<dim3((n * L + 255) / 256), dim3(256), 0, s>>>(rec_sims, n * L);
  bd::k_bd_embed<<<dim3(n), dim3(256), 0, s>>>(st, D.tok_emb, d, c.vocab, L, h, hprev, hist);
  const size_t seq_stride = y.cache_bytes / 2;               // elements (bf16)
  // attention: one workgroup per (sequence, kv head, group of query heads, split of the positions);
  // splits so that every CU has two workgroups (measured best) of at least 128 positions
  const int rep = c.n_q_heads / c.n_kv_heads, arep = rep % 4 == 0 ? 4 : 1;
  int t_max = 1;
  for (int b = 0; b < n; ++b) t_max = std::max(t_max, x->pos_b[b] + 1);
  const int hgs = rep / arep, groups = n * c.n_kv_heads * hgs;
  int n_splits = (2 * x->grid_persist + groups - 1) / groups;
  n_splits = std::max(1, std::min({n_splits, bd::kBdAttnMaxSplits, (t_max + 127) / 128}));
  const size_t attn_lds = bd::bd_attn_lds_bytes(arep, c.head_dim);
  const int qkv_ld = qd + 2 * c.n_kv_heads * c.head_dim;
  for (int l = 0; l < L; ++l) {
    const DevLayer &W = x->layers_h[l];
    // the norm in front of the QKV GEMM: block 1's here, the others' by the previous block's last kernel
    if (l == 0) bd::k_bd_rmsnorm<<<dim3(n), dim3(256), 0, s>>>(h, W.attn_norm, d, c.rms_eps, x16, nullptr, 0);
    launch_bd_gemm(x, l, 0, x16, big, qkv_ld, bd::EPI_STORE, n);
    {
      const dim3 ga((n * c.n_kv_heads * n_splits + 7) / 8 * 8 * hgs);
      auto attn = c.head_dim == 128
                      ? (arep == 4 ? (D.kv_f16 ? bd::k_bd_attn<128, true, 4> : bd::k_bd_attn<128, false, 4>)
                                   : (D.kv_f16 ? bd::k_bd_attn<128, true, 1> : bd::k_bd_attn<128, false, 1>))
                      : (arep == 4 ? (D.kv_f16 ? bd::k_bd_attn<64, true, 4> : bd::k_bd_attn<64, false, 4>)
                                   : (D.kv_f16 ? bd::k_bd_attn<64, true, 1> : bd::k_bd_attn<64, false, 1>));
      attn<<<ga, dim3(256), attn_lds, s>>>(big, D.rope, D.kcache, D.vcache, c.n_q_heads, c.n_kv_heads, n, l, c.max_seq,
                                           seq_stride, st.pos, n_splits, part_o, part_ml, tickets, o16);
    }
    // The output projection completes h; the norm in front of gate/up rides on the two GEMMs:
    // fp16(h * gain) and the rows' partial sums of squares from the first, 1 / rms applied by the
    // second (see bd::BdNorm).
    float *ssq = (float *)(x->ws + y.bd_ssq);
    int o_grid = 0;
    launch_bd_gemm(x, l, 1, o16, h, d, bd::EPI_ADD_NORM, n, bd::BdNorm{W.ffn_norm, x16, ssq, nullptr, 0, 0, 0.f}, &o_grid);
    // gate and up rows interleaved, SwiGLU in the epilogue: the down projection's input as fp16
    launch_bd_gemm(x, l, 2, x16, a16, ffn, bd::EPI_SWIGLU, n, bd::BdNorm{nullptr, nullptr, nullptr, ssq, o_grid, d, c.rms_eps});
    const int pd = launch_bd_gemm(x, l, 3, a16, h, d, bd::EPI_ADD, n);
    // similarity, the sequences' own exit decisions, and the norm in front of the next GEMM
    const bool may_exit = l + 1 >= c.min_exit_layer && l + 1 < L;
    const bool batch_rule = c.batch_exit_rule == 1;
    bd::k_bd_block_end<<<dim3(n), dim3(256), 0, s>>>(hprev, h, d, l + 1, L, st, s_of, rec_sims,
                                                     hist + (size_t)(l + 1) * B * d, may_exit && !batch_rule, c.tau,
                                                     l + 1 < L ? x->layers_h[l + 1].attn_norm : D.final_norm,
                                                     c.rms_eps, x16, partial, pd);
    if (may_exit && batch_rule)
      bd::k_bd_decide<<<dim3(1), dim3(64), 0, s>>>(n, l + 1, L, c.min_exit_layer, c.tau, c.batch_exit_rule, st, s_of);
  }
  // the original LM head (its input is already normalised), greedy token per sequence
  launch_bd_gemm_b(x, x->bd_head, x->bd_head, c.vocab, x16, d, logits, c.vocab, bd::EPI_STORE, 0, n);
  // (the attention kernels are done with their partial-result area and tickets)
  bd::k_bd_argmax<<<dim3(n * bd::kBdArgmaxChunks), dim3(256), 0, s>>>(logits, c.vocab, st, rec_token, rec_exit, part_ml, tickets);
  HIP_TRY(x, hipGetLastError());
  for (int b = 0; b < n; ++b) x->pos_b[b] += 1;
  x->steps_b += 1;
  x->last_n = n;
  if (!out_tokens) return RIVER_OK;
  HIP_TRY(x, hipMemcpyAsync(out_tokens, rec_token, (size_t)n * 4, hipMemcpyDeviceToHost, s));
  if (out_exit_layers) HIP_TRY(x, hipMemcpyAsync(out_exit_layers, rec_exit, (size_t)n * 4, hipMemcpyDeviceToHost, s));
  if (out_sims) HIP_TRY(x, hipMemcpyAsync(out_sims, rec_sims, (size_t)n * L * 4, hipMemcpyDeviceToHost, s));
  HIP_TRY(x, hipStreamSynchronize(s));
  return RIVER_OK;
}

extern "C" int river_read_batch_records(river_ctx *x, int32_t n_steps, int32_t n_seq, int32_t *tokens,
                                        int32_t *exit_layers) {
  CHECK_CTX(x);
  if (x->cfg.max_batch < 2 || n_steps < 0 || n_steps > bd::kRecordsB || n_steps > x->steps_b || n_seq < 1 ||
      n_seq > x->cfg.max_batch || (n_steps > 0 && (!tokens || !exit_layers))) {
    x->err = "bad batch record request";
    return RIVER_EINVAL;
  }
  const size_t B = x->cfg.max_batch;
  for (int i = 0; i < n_steps; ++i) {
    const size_t slot = (size_t)((x->steps_b - n_steps + i) % bd::kRecordsB);
    HIP_TRY(x, hipMemcpyAsync(tokens + (size_t)i * n_seq, (int *)(x->ws + x->lay.bd_rec_token) + slot * B,
                              (size_t)n_seq * 4, hipMemcpyDeviceToHost, x->stream));
    HIP_TRY(x, hipMemcpyAsync(exit_layers + (size_t)i * n_seq, (int *)(x->ws + x->lay.bd_rec_exit) + slot * B,
                              (size_t)n_seq * 4, hipMemcpyDeviceToHost, x->stream));
  }
  HIP_TRY(x, hipStreamSynchronize(x->stream));
  return RIVER_OK;
}

extern "C" int river_read_records(river_ctx *x, int32_t n, int32_t *tokens, int32_t *exit_layers,
                                  float *sims) {
  CHECK_CTX(x);
  if (n < 0 || n > kRecords || n > x->steps || (n > 0 && (!tokens || !exit_layers))) {
    x->err = "bad record count";
    return RIVER_EINVAL;
  }
  const int L = x->cfg.n_layers;
  int rc = check_device_error(x);
  if (rc) return rc;
  for (int i = 0; i < n; ++i) {
    const int slot = (int)((x->steps - n + i) % kRecords);
    HIP_TRY(x, hipMemcpyAsync(tokens + i, x->dev.rec_token + slot, 4, hipMemcpyDeviceToHost, x->stream));
    HIP_TRY(x, hipMemcpyAsync(exit_layers + i, x->dev.rec_exit + slot, 4, hipMemcpyDeviceToHost, x->stream));
    if (sims)
      HIP_TRY(x, hipMemcpyAsync(sims + (size_t)i * L, x->dev.rec_sims + (size_t)slot * L, (size_t)L * 4,
                                hipMemcpyDeviceToHost, x->stream));
  }
  HIP_TRY(x, hipStreamSynchronize(x->stream));
  return RIVER_OK;
}

extern "C" int river_rewind(river_ctx *x, int32_t seq, int32_t new_len) {
  CHECK_CTX(x);
  if (x->cfg.max_batch > 1) {
    if (seq < 0 || seq >= x->cfg.max_batch || new_len < 0 || new_len > x->pos_b[seq]) {
      x->err = "bad rewind length";
      return RIVER_EINVAL;
    }
    x->pos_b[seq] = new_len;
    HIP_TRY(x, hipMemcpyAsync(x->st_b.pos + seq, &x->pos_b[seq], 4, hipMemcpyHostToDevice, x->stream));
    HIP_TRY(x, hipStreamSynchronize(x->stream));
    return RIVER_OK;
  }
  if (seq != 0 || new_len < 0 || new_len > x->pos) { x->err = "bad rewind length"; return RIVER_EINVAL; }
  x->pos = new_len;
  return RIVER_OK;
}

extern "C" int river_position(const river_ctx *x) { return x ? x->pos : RIVER_EINVAL; }
extern "C" int river_seq_position(const river_ctx *x, int32_t seq) {
  if (!x || seq < 0 || seq >= x->cfg.max_batch) return RIVER_EINVAL;
  return x->cfg.max_batch > 1 ? x->pos_b[seq] : x->pos;
}

extern "C" int river_get_debug(river_ctx *x, int32_t what, void *dst, size_t bytes) {
  if (!x || !dst) return RIVER_EINVAL;
  const char *src = nullptr;
  size_t n = 0;
  switch (what) {
    case RIVER_DBG_HIDDEN: src = (const char *)x->dev.hidden; n = (size_t)(x->cfg.n_layers + 1) * x->cfg.d_model * 4; break;
    case RIVER_DBG_LOGITS: src = (const char *)x->dev.logits; n = (size_t)x->cfg.vocab * 4; break;
    case RIVER_DBG_KCACHE: src = (const char *)x->dev.kcache; n = x->lay.cache_bytes * x->cfg.max_batch; break;
    case RIVER_DBG_VCACHE: src = (const char *)x->dev.vcache; n = x->lay.cache_bytes * x->cfg.max_batch; break;
    case RIVER_DBG_BATCH_HIDDEN:
      if (x->cfg.max_batch < 2) { x->err = "not a batched context"; return RIVER_EINVAL; }
      src = x->ws + x->lay.bd_hist;
      n = (size_t)(x->cfg.n_layers + 1) * x->cfg.max_batch * x->cfg.d_model * 4;
      break;
    case RIVER_DBG_BATCH_LOGITS:
      if (x->cfg.max_batch < 2) { x->err = "not a batched context"; return RIVER_EINVAL; }
      src = x->ws + x->lay.bd_logits;
      n = (size_t)x->cfg.max_batch * x->cfg.vocab * 4;
      break;
    case RIVER_DBG_TRACE: src = (const char *)x->dev.trace; n = ((size_t)5 * x->cfg.n_layers * 2 * x->grid_persist + 64) * 8; break;
    default: x->err = "unknown debug buffer"; return RIVER_EINVAL;
  }
  if (bytes != n) { x->err = "debug buffer size mismatch"; return RIVER_EINVAL; }
  HIP_TRY(x, hipMemcpyAsync(dst, src, n, hipMemcpyDeviceToHost, x->stream));
  HIP_TRY(x, hipStreamSynchronize(x->stream));
  return RIVER_OK;
}

extern "C" int river_fill_cache(river_ctx *x, int32_t value) {
  CHECK_CTX(x);
  const uint32_t b = (uint32_t)value & 0xffu;
  const uint32_t word = b | (b << 8) | (b << 16) | (b << 24);
  const size_t n16 = (x->lay.vcache - x->lay.kcache + align_up(x->lay.cache_bytes * x->cfg.max_batch, 256)) / 16;
  k_fill_bytes<<<dim3(1024), dim3(256), 0, x->stream>>>((uint4 *)x->dev.kcache, n16, word);
  HIP_TRY(x, hipGetLastError());
  return RIVER_OK;
}

extern "C" const char *river_last_error(const river_ctx *x) {
  return x ? x->err.c_str() : g_create_err.c_str();
}

extern "C" int river_destroy(river_ctx *x) {
  if (!x) return RIVER_OK;
  (void)hipStreamSynchronize(x->stream);
  delete x;
  return RIVER_OK;
}
