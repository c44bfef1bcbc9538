// MI355X (gfx950) pipelined online learner: HIP kernels and the C ABI around them.
//
// One stream tick of the method (Sec. III, Algorithm 1 of the PARTIME paper) for ALL stages is one
// grouped kernel launch.  A work-group owns a block of rows of one stage's weight matrix and makes a
// single pass over it: each wave pulls whole rows into registers, forms z = W x + b (Eq. 6), the local
// delta from the error the next stage published one tick earlier (Eq. 11), accumulates its share of
// W^T delta with the row as it was loaded (so with the not yet updated weights), applies the rank-1
// SGD update (Eq. 9 + Algorithm 1's update step) to the registers and writes the row back.  Every
// weight is read once and written once per learning tick, which is the algorithmic minimum.
//
// Nothing here includes or links the CPU oracle.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "partime.h"

namespace {

constexpr int kMaxIn = 4096;           // longest row a wave keeps in registers
constexpr int kMaxTileRows = 1024;     // rows of an ordinary tile
constexpr int kMaxHeadRows = 4096;     // rows of a single-tile softmax head
constexpr int kLossSlots = 1024;       // ticks per loss-partial block

// ------------------------------------------------------------------------------------------------
// device-side description of the pipeline
// ------------------------------------------------------------------------------------------------

struct StageDev {
  void *W;                 // [out_dim][ld] fp32 or bf16
  float *b;                // [out_dim]
  int in_dim, out_dim, ld; // ld: row pitch in elements, multiple of the per-lane vector width
  int act, nch, is_last;
  const float *in_act[2];  // what the previous stage published (NULL for the first stage)
  float *out_act[2];       // what this stage publishes (NULL for the last stage)
  const float *gin[2];     // error partials of the next stage: [n_gparts][gin_ld]
  int n_gparts, gin_ld;
  float *eout[2];          // this stage's error partials [n_parts][ld] (NULL for the first stage)
  int n_parts;
  float *mW, *vW, *mb, *vb;  // Adam moments, fp32: [out_dim][ld], [out_dim] (NULL under plain SGD)
  // skip connections (the paper's Sec. V-C): a skipped tensor crosses d stage boundaries in d ticks, like the main
  // path, so it waits in a ring of d + 1 slots of out_dim floats (slot = tick % (d + 1)); so does its gradient
  const float *skip_in;      // ring whose value of d ticks ago is added to this layer's output (NULL: none)
  int skip_in_n, skip_in_d;
  float *skip_out;           // ring this layer's output is also written to (it is the source of a skip)
  int skip_out_n;
  float *serr_out;           // ring the gradient at this layer's output is written to (it is the target of a skip)
  int serr_out_n;
  const float *serr_in;      // ring whose gradient of d ticks ago is added to the gradient at this layer's output
  int serr_in_n, serr_in_d;
};

// one stage as one tick sees it: ping-pong halves already chosen, no arrays, so it stays in registers
struct StageView {
  void *W;
  float *b;
  int in_dim, out_dim, ld, act, nch, is_last;
  const float *in_prev;
  float *out_cur;
  const float *gin_prev;
  int n_gparts, gin_ld;
  float *eout_cur;
  int n_parts;
  float *mW, *vW, *mb, *vb;
  const float *skip_in;      // already at the slot to read this tick
  float *skip_out;           // already at the slot to write this tick
  float *serr_out;
  const float *serr_in;
};

struct TileDev {
  int stage, row0, nrows, part;
};

// what a work-group reads first: its tile and, in the same record, a copy of the layer's record (with the layer records
// in an array of their own it would read the tile, then the layer, then its data: three cold round trips in a row)
struct TileRec {
  TileDev t;
  StageDev s;
};

struct NetDev {
  const TileRec *tiles;
  int depth, n_tiles, loss, out_dim, xs_len, red_len, max_rows;
  float lr;
  float beta1, beta2, eps;   // Adam
  // softmax head split over several tiles: where the tiles leave their outputs for each other, the counter of tiles
  // that have done so (monotonic over the ticks), how long a tile may wait for the others, the flag it raises if not
  float *head_o;
  unsigned int *head_ctr;
  int *err;
  long long spin_limit;
  int head_parts;            // tiles of the softmax head (1: it keeps its outputs to itself, nothing is exchanged)
};

struct TickArgs {
  const float *x;   // this tick's sample [in]
  const void *tgt;  // the target this tick is scored against
  float *out;       // [out] row of the caller's output array
  float *lossp;     // MSE: per-tile partial sums of this tick [n_parts of last stage]
  float *loss1;     // CE: the loss of this tick
  int cur;          // half written this tick
  int learn;        // 0 while the loss gradient is held at zero
  int rev;          // walk the rows of a tile backwards on this tick
  int tick;         // tick number modulo a common multiple of all ring lengths (ring slots of the skip connections)
  unsigned int head_target;   // value of the head counter once every tile of the softmax head has published its outputs
  float adam_c1;    // Adam, this tick's step n: lr / (1 - beta1^n)
  float adam_c2;    //                           1 / sqrt(1 - beta2^n)
};

// a block of ticks for the persistent kernel: per-tick pointers are derived on the device
struct BlockArgs {
  const float *x;             // [n_ticks][in]
  const unsigned char *tgt;   // caller's targets of this block
  const unsigned char *hist;  // the k targets that preceded the block, oldest first
  float *out;                 // [n_ticks][out]
  float *lossp;               // [n_ticks][pl]
  float *loss;                // [n_ticks] or NULL
  float *dummy;
  unsigned long long *bar;    // arrival counter of the grid barrier (monotonic)
  int *err;                   // set when a barrier wait ran out
  unsigned long long bar_base;
  unsigned int head_base, head_parts;   // head counter before the block; tiles of the softmax head
  long long t0, spin_limit;
  int n_ticks, fill, k, serp, has_loss, pl, tgt_bytes, in_stride, out_stride;
};

// ------------------------------------------------------------------------------------------------
// global-memory accessors
// ------------------------------------------------------------------------------------------------
// Pointers that a kernel reads out of a descriptor in memory are "generic" to the compiler, which then emits
// FLAT loads and stores; those cannot be waited for selectively, so every use waits for everything in flight.
// These helpers state that the address is global memory (address space 1).

typedef unsigned int pt_v4u __attribute__((ext_vector_type(4)));
typedef unsigned int pt_v2u __attribute__((ext_vector_type(2)));
typedef float pt_v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) pt_v4u g_v4u;
typedef __attribute__((address_space(1))) pt_v2u g_v2u;
typedef __attribute__((address_space(1))) pt_v4f g_v4f;
typedef __attribute__((address_space(1))) float g_f32;
typedef __attribute__((address_space(1))) int g_i32;
typedef __attribute__((address_space(1))) unsigned short g_u16;

__device__ __forceinline__ uint4 ldg16(const void *p) { const pt_v4u t = *(const g_v4u *)p; return make_uint4(t.x, t.y, t.z, t.w); }
__device__ __forceinline__ void stg16(void *p, const uint4 &v) { const pt_v4u t = {v.x, v.y, v.z, v.w}; *(g_v4u *)p = t; }
__device__ __forceinline__ uint2 ldg8(const void *p) { const pt_v2u t = *(const g_v2u *)p; return make_uint2(t.x, t.y); }
__device__ __forceinline__ void stg8(void *p, const uint2 &v) { const pt_v2u t = {v.x, v.y}; *(g_v2u *)p = t; }
__device__ __forceinline__ float4 ldg_f4(const void *p) { const pt_v4f t = *(const g_v4f *)p; return make_float4(t.x, t.y, t.z, t.w); }
__device__ __forceinline__ void stg_f4(void *p, const float4 &v) { const pt_v4f t = {v.x, v.y, v.z, v.w}; *(g_v4f *)p = t; }
__device__ __forceinline__ float ldg_f(const void *p) { return *(const g_f32 *)p; }
__device__ __forceinline__ void stg_f(void *p, float v) { *(g_f32 *)p = v; }
__device__ __forceinline__ int ldg_i(const void *p) { return *(const g_i32 *)p; }
__device__ __forceinline__ void stg_u16(void *p, unsigned int v) { *(g_u16 *)p = (unsigned short)v; }

// ------------------------------------------------------------------------------------------------
// storage types
// ------------------------------------------------------------------------------------------------

struct bf16_t {
  unsigned short v;
};

__device__ __forceinline__ unsigned int f32_bits(float f) { return __float_as_uint(f); }

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN
__device__ __forceinline__ unsigned int bf16_rne(float f) {
  unsigned int u = f32_bits(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// two fp32 -> two bf16 (round to nearest even) in one word; gfx950 has a packed conversion instruction
typedef __bf16 pt_bf16x2 __attribute__((ext_vector_type(2)));
typedef float pt_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned int pack_bf16_rne(float lo, float hi) {
  const pt_f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, pt_bf16x2));
}

template <typename WT>
struct WTraits;
template <>
struct WTraits<float> {
  static constexpr int EPL = 4;
  static __device__ __forceinline__ void load(const float *p, float (&w)[4]) {
    const float4 v = ldg_f4(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  }
  static __device__ __forceinline__ void store(float *p, const float (&w)[4]) {
    // plain cached accesses on purpose: streaming (non-temporal) hints keep the rows out of the memory-side
    // cache and lose the reuse that the alternating row order creates between consecutive ticks
    stg_f4(p, make_float4(w[0], w[1], w[2], w[3]));
  }
};
template <>
struct WTraits<bf16_t> {
  static constexpr int EPL = 8;
  static __device__ __forceinline__ void load(const bf16_t *p, float (&w)[8]) {
    const uint4 v = ldg16(p);
    const unsigned int u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[2 * i] = __uint_as_float(u[i] << 16);
      w[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16_t *p, const float (&w)[8]) {
    unsigned int u[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) u[i] = pack_bf16_rne(w[2 * i], w[2 * i + 1]);
    stg16(p, make_uint4(u[0], u[1], u[2], u[3]));
  }
};

// ------------------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------------------

// one data-parallel-primitive move of a 32-bit value between lanes; lanes whose row is masked off get `old`
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float old, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
// sum / max over the 64 lanes of a wave; the result is wave-uniform.  Six DPP steps: swap within pairs,
// swap pairs within quads, mirror within 8, mirror within 16, then carry lane 15 / lane 31 of a 16-lane
// row into the following rows; lane 63 ends up with the total.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<0xB1, 0xf>(0.f, v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E, 0xf>(0.f, v);   // quad_perm [2,3,0,1]
  v += dpp_move<0x141, 0xf>(0.f, v);  // row_half_mirror
  v += dpp_move<0x140, 0xf>(0.f, v);  // row_mirror
  v += dpp_move<0x142, 0xa>(0.f, v);  // row_bcast15 into rows 1 and 3
  v += dpp_move<0x143, 0xc>(0.f, v);  // row_bcast31 into rows 2 and 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1, 0xf>(v, v));
  v = fmaxf(v, dpp_move<0x4E, 0xf>(v, v));
  v = fmaxf(v, dpp_move<0x141, 0xf>(v, v));
  v = fmaxf(v, dpp_move<0x140, 0xf>(v, v));
  v = fmaxf(v, dpp_move<0x142, 0xa>(v, v));
  v = fmaxf(v, dpp_move<0x143, 0xc>(v, v));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// block-wide reductions through NW floats of LDS; every thread gets the result
template <int NW>
__device__ __forceinline__ float block_sum(float v, float *sm) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) t += sm[i];
  return t;
}
template <int NW>
__device__ __forceinline__ float block_max(float v, float *sm) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = sm[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) t = fmaxf(t, sm[i]);
  return t;
}

// Accesses to the vectors that one work-group writes and another reads one tick later.  Inside the
// persistent kernel (COH) no kernel boundary separates the two, and the L2 caches of different XCDs are
// not coherent with each other for ordinary accesses: device-scope atomic loads/stores go past them.
template <bool COH>
__device__ __forceinline__ float ld_x(const float *p) {
  if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return ldg_f(p);
}
template <bool COH>
__device__ __forceinline__ void st_x(float *p, float v) {
  if constexpr (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else stg_f(p, v);
}

__device__ __forceinline__ float act_fwd(int act, float z) {
  if (act == PT_RELU) return z > 0.f ? z : 0.f;
  if (act == PT_GELU) return 0.5f * z * (1.f + erff(z * 0.70710678118654752440f));
  return z;
}
__device__ __forceinline__ float act_der(int act, float z) {
  if (act == PT_RELU) return z > 0.f ? 1.f : 0.f;
  if (act == PT_GELU) {
    const float cdf = 0.5f * (1.f + erff(z * 0.70710678118654752440f));
    const float pdf = expf(-0.5f * z * z) * 0.3989422804014326779f;
    return cdf + z * pdf;
  }
  return 1.f;
}

// ------------------------------------------------------------------------------------------------
// one tile = a block of rows of one stage, processed by one work-group of NW waves
// ------------------------------------------------------------------------------------------------

template <typename WT, int NCH, int RB>
struct RowRegs {
  static constexpr int EPL = WTraits<WT>::EPL;
  float w[RB][NCH][EPL];
};

// load RB rows starting at `row` (rows >= row_end are left as zeros)
template <typename WT, int NCH, int RB>
__device__ __forceinline__ void load_rows(RowRegs<WT, NCH, RB> &R, const WT *W, int ld, int row, int row_end,
                                          int lane) {
  constexpr int EPL = WTraits<WT>::EPL;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (c * 64 + lane) * EPL;
      if (row + rb < row_end && col < ld) {
        WTraits<WT>::load(W + (size_t)(row + rb) * ld + col, R.w[rb][c]);
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) R.w[rb][c][e] = 0.f;
      }
    }
  }
}

template <int EPL>
__device__ __forceinline__ void load_x(const float *xs, int c, int lane, float (&xv)[EPL]) {
  const float4 *xp = reinterpret_cast<const float4 *>(xs + (c * 64 + lane) * EPL);
#pragma unroll
  for (int q = 0; q < EPL / 4; ++q) {
    const float4 t = xp[q];
    xv[4 * q] = t.x; xv[4 * q + 1] = t.y; xv[4 * q + 2] = t.z; xv[4 * q + 3] = t.w;
  }
}

template <typename WT, int NCH, int RB>
__device__ __forceinline__ void dot_rows(const RowRegs<WT, NCH, RB> &R, const float *xs, int lane, float (&acc)[RB]) {
  constexpr int EPL = WTraits<WT>::EPL;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) acc[rb] = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    float xv[EPL];
    load_x<EPL>(xs, c, lane, xv);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[rb] = fmaf(R.w[rb][c][e], xv[e], acc[rb]);
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) acc[rb] = wave_sum(acc[rb]);
}

// LDS carve-up of a tile (floats)
template <int NW>
struct TileLds {
  float *xs, *red, *gs, *bsh, *ov, *dl, *rs, *sm;
  __device__ __forceinline__ TileLds(float *lds, int xs_len, int red_len, int max_rows) {
    xs = lds;                              // [xs_len] stage input, zero padded
    red = xs + xs_len;                     // [red_len] cross-wave error reduction [NW/2][xs_len]; gather scratch
    gs = red + red_len;                    // [max_rows] g (or the MSE target) per row
    bsh = gs + max_rows;                   // [max_rows] bias
    ov = bsh + max_rows;                   // [max_rows] stage output
    dl = ov + max_rows;                    // [max_rows] delta
    rs = dl + max_rows;                    // [max_rows] skipped tensor added to the output (zeros if none)
    sm = rs + max_rows;                    // [2*NW] reduction scratch
  }
};

template <typename WT, int NCH, int RB, bool LEARN, int NW, int NBUF, bool COH, int OPT = 0>
__device__ __forceinline__ void run_tile(const NetDev &net, const StageView &st, const TileDev &tl, const TickArgs &a,
                                         float *lds) {
  constexpr int EPL = WTraits<WT>::EPL;
  constexpr int XLEN = NCH * 64 * EPL;
  constexpr int NT = NW * 64;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const TileLds<NW> L(lds, net.xs_len, net.red_len, net.max_rows);
  float *xs = L.xs, *red = L.red, *gs = L.gs, *bsh = L.bsh, *ov = L.ov, *dl = L.dl, *rs = L.rs, *sm = L.sm;

  const int cur = a.cur, prev = cur ^ 1;
  const WT *W = static_cast<const WT *>(st.W);
  WT *Wm = static_cast<WT *>(st.W);
  const int ld = st.ld, nrows = tl.nrows, row0 = tl.row0, row_end = tl.row0 + tl.nrows;
  const bool last = st.is_last != 0;
  const bool ce_head = LEARN && last && net.loss == PT_LOSS_CE;
  const bool mse_head = LEARN && last && net.loss == PT_LOSS_MSE;
  const bool has_eout = LEARN && st.eout_cur != nullptr;
  const int n_it = (nrows + NW * RB - 1) / (NW * RB);
  auto g0_of = [&](int it) { return wv * RB + (a.rev ? n_it - 1 - it : it) * NW * RB; };

  // the first rows are requested before anything else so that they travel while the tile sets up
  RowRegs<WT, NCH, RB> R[NBUF];
  if (!ce_head) {
#pragma unroll
    for (int b = 0; b < NBUF; ++b)
      if (b < n_it) load_rows<WT, NCH, RB>(R[b], W, ld, row0 + g0_of(b), row_end, lane);
  }

  // a0: the stage input (Algorithm 1, first step): x(t) or what stage h-1 wrote last tick
  if (st.in_prev) {
    const float *xin = st.in_prev;
    for (int i = tid; i < XLEN; i += NT) xs[i] = i < st.in_dim ? ld_x<COH>(xin + i) : 0.f;
  } else {
    for (int i = tid; i < XLEN; i += NT) xs[i] = i < st.in_dim ? ldg_f(a.x + i) : 0.f;
  }
  // a3: the error the next stage published one tick earlier (Eq. 11).  It arrives as one partial vector per
  // tile of that stage; all threads fetch a share (thread -> row i, every n_grp-th partial) so that the
  // loads are in flight together, then the shares are added in a fixed order.
  const bool sum_g = LEARN && !last;
  const int rpad = (nrows + 63) & ~63;               // rows rounded up to whole waves
  const int n_grp = sum_g ? max(1, min(NT / rpad, st.n_gparts)) : 1;
  if (sum_g) {
    for (int j = tid; j < rpad * n_grp; j += NT) {
      const int i = j % rpad, grp = j / rpad;
      float g = 0.f;
      if (i < nrows) {
        const float *gp = st.gin_prev + row0 + i;
#pragma unroll 8
        for (int p = grp; p < st.n_gparts; p += n_grp) g += ld_x<COH>(gp + (size_t)p * st.gin_ld);
      }
      red[j] = g;
    }
  }
  for (int i = tid; i < nrows; i += NT) {
    bsh[i] = ldg_f(st.b + row0 + i);
    rs[i] = st.skip_in ? ldg_f(st.skip_in + row0 + i) : 0.f;
    if (mse_head) gs[i] = ldg_f(static_cast<const float *>(a.tgt) + row0 + i);
  }
  __syncthreads();
  if (sum_g) {
    for (int i = tid; i < nrows; i += NT) {
      float g = 0.f;
      for (int grp = 0; grp < n_grp; ++grp) g += red[grp * rpad + i];
      // a skip that started at this layer's output brings its gradient back over its own delay line; a skip that
      // ends here passes the gradient at this output on unchanged (o = phi(z) + skipped tensor)
      if (st.serr_in) g += ldg_f(st.serr_in + row0 + i);
      if (st.serr_out) stg_f(st.serr_out + row0 + i, g);
      gs[i] = g;
    }
    __syncthreads();
  }

  if (ce_head) {
    // softmax needs every output of the stage before any delta exists: a forward-only pass over this tile's rows first
    // (the learning pass below then finds them in the cache); the tiles of the stage leave their outputs for each other
    // in memory and each one waits until all have done so.  The head's tiles are the first of the launch and a launch
    // is one round of work-groups, so they are all running; the wait is bounded all the same, and when it runs out the
    // error flag is raised and the tile leaves the weights alone.
    __shared__ int s_head_ok;
    const bool xchg = net.head_parts > 1;
    const int n_all = st.out_dim;
    float *oall = red;
    for (int g0 = wv * RB; g0 < nrows; g0 += NW * RB) {
      load_rows<WT, NCH, RB>(R[0], W, ld, row0 + g0, row_end, lane);
      float acc[RB];
      dot_rows<WT, NCH, RB>(R[0], xs, lane, acc);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        if (g0 + rb < nrows && lane == 0) {
          const float o = act_fwd(st.act, acc[rb] + bsh[g0 + rb]);
          if (xchg) st_x<true>(net.head_o + row0 + g0 + rb, o);
          else oall[g0 + rb] = o;
        }
    }
    // every wave waits until its own stores have been acknowledged, then the work-group announces itself
    if (xchg) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (xchg && tid == 0) {
      __hip_atomic_fetch_add(net.head_ctr, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
      long long spins = 0;
      int ok = 1;
      while ((int)(__hip_atomic_load(net.head_ctr, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) - a.head_target) < 0) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > net.spin_limit) {
          __hip_atomic_store(net.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ok = 0;
          break;
        }
      }
      s_head_ok = ok;
    }
    if (xchg) {
      __syncthreads();
      if (!s_head_ok) return;
    }
    // all outputs of the stage, the same in every tile and summed in the same order: the tiles agree bit for bit
    float m = -INFINITY;
    for (int i = tid; i < n_all; i += NT) {
      const float v = xchg ? ld_x<true>(net.head_o + i) : oall[i];
      if (xchg) oall[i] = v;
      m = fmaxf(m, v);
    }
    m = block_max<NW>(m, sm);
    float s = 0.f;
    for (int i = tid; i < n_all; i += NT) s += expf(oall[i] - m);
    s = block_sum<NW>(s, sm + NW);
    const int y = min(max(static_cast<const int *>(a.tgt)[0], 0), n_all - 1);  // class id, kept in range
    for (int i = tid; i < nrows; i += NT)
      gs[i] = a.learn ? expf(oall[row0 + i] - m) / s - (row0 + i == y ? 1.f : 0.f) : 0.f;
    if (tid == 0 && tl.part == 0) a.loss1[0] = a.learn ? -(oall[y] - m - logf(s)) : 0.f;
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NBUF; ++b)
      if (b < n_it) load_rows<WT, NCH, RB>(R[b], W, ld, row0 + g0_of(b), row_end, lane);
  }

  float e[NCH][EPL];
#pragma unroll
  for (int c = 0; c < NCH; ++c)
#pragma unroll
    for (int q = 0; q < EPL; ++q) e[c][q] = 0.f;
  float sq = 0.f;
  const float inv_n = 1.f / (float)net.out_dim;

  // Adam moments of the rows in flight: two batches of CB column chunks (about 32 registers)
  constexpr int CB = OPT == 1 ? (RB * EPL >= 8 ? 1 : (8 / (RB * EPL) < NCH ? 8 / (RB * EPL) : NCH)) : 1;
  float mq[OPT == 1 ? 2 : 1][CB][RB][EPL], vq[OPT == 1 ? 2 : 1][CB][RB][EPL];
  auto fetch_mv = [&](int slot, int c0, int g0) {
#pragma unroll
    for (int cc = 0; cc < CB; ++cc)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const int col = ((c0 + cc) * 64 + lane) * EPL;
        const bool ok = g0 + rb < nrows && col < ld;                  // clamped address, unconditional load
        const size_t off = ok ? (size_t)(row0 + g0 + rb) * ld + col : 0;
#pragma unroll
        for (int q4 = 0; q4 < EPL; q4 += 4) {
          const float4 m4 = ldg_f4(st.mW + off + q4), v4 = ldg_f4(st.vW + off + q4);
          mq[slot][cc][rb][q4] = m4.x; mq[slot][cc][rb][q4 + 1] = m4.y; mq[slot][cc][rb][q4 + 2] = m4.z; mq[slot][cc][rb][q4 + 3] = m4.w;
          vq[slot][cc][rb][q4] = v4.x; vq[slot][cc][rb][q4 + 1] = v4.y; vq[slot][cc][rb][q4 + 2] = v4.z; vq[slot][cc][rb][q4 + 3] = v4.w;
        }
      }
  };

  for (int it0 = 0; it0 < n_it; it0 += NBUF) {
#pragma unroll
    for (int b = 0; b < NBUF; ++b) {
      const int it = it0 + b;
      if (it >= n_it) break;
      const int g0 = g0_of(it);
      if constexpr (LEARN && OPT == 1) fetch_mv(0, 0, g0);
      float acc[RB];
      dot_rows<WT, NCH, RB>(R[b], xs, lane, acc);   // a1: z = W x + b (Eq. 6)
      float delta[RB];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        delta[rb] = 0.f;
        if (g0 + rb < nrows) {
          const float z = acc[rb] + bsh[g0 + rb];
          const float o = act_fwd(st.act, z) + rs[g0 + rb];
          if (LEARN) {
            float g = gs[g0 + rb];
            if (mse_head) {  // a2: g_D = dL/do at this tick's output
              const float d = o - g;
              sq = fmaf(d, d, sq);
              g = a.learn ? 2.f * d * inv_n : 0.f;
            }
            delta[rb] = g * act_der(st.act, z);   // a4: derivative at this tick's z (Eq. 9)
          }
          if (lane == 0) {
            ov[g0 + rb] = o;
            if (LEARN) dl[g0 + rb] = delta[rb];
          }
        }
      }
      if constexpr (LEARN && OPT == 1) {
        // a6 with Adam: the moments of the rows travel in batches of CB column chunks, one batch ahead of the
        // arithmetic (the first batch was requested before the dot products)
#pragma unroll
        for (int bi = 0; bi < NCH / CB; ++bi) {
          if (bi + 1 < NCH / CB) fetch_mv((bi + 1) & 1, (bi + 1) * CB, g0);
#pragma unroll
          for (int cc = 0; cc < CB; ++cc) {
            const int c = bi * CB + cc, col = (c * 64 + lane) * EPL;
            float xv[EPL];
            load_x<EPL>(xs, c, lane, xv);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
              float mo[EPL], vo[EPL];
#pragma unroll
              for (int q = 0; q < EPL; ++q) {
                const float wold = R[b].w[rb][c][q];
                e[c][q] = fmaf(delta[rb], wold, e[c][q]);             // a5 with the loaded (old) row
                const float gq = delta[rb] * xv[q];                   // Eq. 9
                mo[q] = fmaf(net.beta1, mq[bi & 1][cc][rb][q], (1.f - net.beta1) * gq);
                vo[q] = fmaf(net.beta2, vq[bi & 1][cc][rb][q], (1.f - net.beta2) * gq * gq);
                R[b].w[rb][c][q] = wold - a.adam_c1 * mo[q] / (sqrtf(vo[q]) * a.adam_c2 + net.eps);
              }
              if (g0 + rb < nrows && col < ld) {
                const size_t off = (size_t)(row0 + g0 + rb) * ld + col;
                WTraits<WT>::store(Wm + off, R[b].w[rb][c]);
#pragma unroll
                for (int q4 = 0; q4 < EPL; q4 += 4) {
                  stg_f4(st.mW + off + q4, make_float4(mo[q4], mo[q4 + 1], mo[q4 + 2], mo[q4 + 3]));
                  stg_f4(st.vW + off + q4, make_float4(vo[q4], vo[q4 + 1], vo[q4 + 2], vo[q4 + 3]));
                }
              }
            }
          }
        }
      } else if (LEARN) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          const int col = (c * 64 + lane) * EPL;
          float xv[EPL];
          load_x<EPL>(xs, c, lane, xv);
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
            const float s = -net.lr * delta[rb];
#pragma unroll
            for (int q = 0; q < EPL; ++q) {
              e[c][q] = fmaf(delta[rb], R[b].w[rb][c][q], e[c][q]);   // a5: W^T delta with the loaded (old) row
              R[b].w[rb][c][q] = fmaf(s, xv[q], R[b].w[rb][c][q]);    // a6: W <- W - eta delta x^T
            }
            if (g0 + rb < nrows && col < ld)
              WTraits<WT>::store(Wm + (size_t)(row0 + g0 + rb) * ld + col, R[b].w[rb][c]);
          }
        }
      }
      if (it + NBUF < n_it) load_rows<WT, NCH, RB>(R[b], W, ld, row0 + g0_of(it + NBUF), row_end, lane);
    }
  }

  if (mse_head) {
    if (lane == 0) sm[wv] = sq;
  }
  __syncthreads();   // ov, dl (and sm) complete
  if (mse_head && tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += sm[i];
    a.lossp[tl.part] = a.learn ? t * inv_n : 0.f;
  }
  for (int i = tid; i < nrows; i += NT) {
    const int r = row0 + i;
    if (last) stg_f(a.out + r, ov[i]);
    else st_x<COH>(st.out_cur + r, ov[i]);
    if (st.skip_out) stg_f(st.skip_out + r, ov[i]);
    if constexpr (LEARN && OPT == 1) {
      const float mo = fmaf(net.beta1, ldg_f(st.mb + r), (1.f - net.beta1) * dl[i]);
      const float vo = fmaf(net.beta2, ldg_f(st.vb + r), (1.f - net.beta2) * dl[i] * dl[i]);
      stg_f(st.mb + r, mo);
      stg_f(st.vb + r, vo);
      stg_f(st.b + r, bsh[i] - a.adam_c1 * mo / (sqrtf(vo) * a.adam_c2 + net.eps));
    } else if (LEARN) {
      stg_f(st.b + r, bsh[i] - net.lr * dl[i]);
    }
  }
  if (has_eout) {
    // sum the waves' shares of W^T delta (fixed order), then publish this tile's partial vector
#pragma unroll
    for (int half = NW / 2; half >= 1; half >>= 1) {
      if (wv >= half && wv < 2 * half) {
        float *dst = red + (size_t)(wv - half) * net.xs_len;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
          for (int q = 0; q < EPL; q += 4)
            *reinterpret_cast<float4 *>(dst + (c * 64 + lane) * EPL + q) =
                make_float4(e[c][q], e[c][q + 1], e[c][q + 2], e[c][q + 3]);
      }
      __syncthreads();
      if (wv < half) {
        const float *src = red + (size_t)wv * net.xs_len;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
          for (int q = 0; q < EPL; q += 4) {
            const float4 t = *reinterpret_cast<const float4 *>(src + (c * 64 + lane) * EPL + q);
            e[c][q] += t.x; e[c][q + 1] += t.y; e[c][q + 2] += t.z; e[c][q + 3] += t.w;
          }
      }
      __syncthreads();
    }
    if (wv == 0) {
      float *dst = st.eout_cur + (size_t)tl.part * ld;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int col = (c * 64 + lane) * EPL;
        if (col < ld) {
          if constexpr (COH) {
#pragma unroll
            for (int q = 0; q < EPL; ++q) st_x<true>(dst + col + q, e[c][q]);
          } else {
#pragma unroll
            for (int q = 0; q < EPL; q += 4)
              stg_f4(dst + col + q, make_float4(e[c][q], e[c][q + 1], e[c][q + 2], e[c][q + 3]));
          }
        }
      }
    }
  }
}

template <typename WT>
constexpr int rows_per_iter(int nch) {
  // registers per lane: one row takes nch * EPL; about 64 of them hold rows, which with the W^T delta
  // share (another nch * EPL) and the rest of the tile's state still lets two waves share a SIMD
  const int per_row = nch * WTraits<WT>::EPL;
  return std::max(1, std::min(8, 64 / per_row));
}

// rows a wave works on at once under Adam: a quarter of the plain number, the moments need registers too
template <typename WT>
constexpr int rows_per_iter_adam(int nch) { return rows_per_iter<WT>(nch) >= 4 ? rows_per_iter<WT>(nch) / 4 : 1; }

template <typename WT, bool LEARN, int NW, int NBUF, bool COH, int OPT = 0>
__device__ __forceinline__ void dispatch_tile(const NetDev &net, const TileRec *rec, const TickArgs &a, float *lds) {
  const TileDev tl = rec->t;
  const StageDev *sp = &rec->s;
  StageView st;
  st.W = sp->W; st.b = sp->b;
  st.in_dim = sp->in_dim; st.out_dim = sp->out_dim; st.ld = sp->ld;
  st.act = sp->act; st.nch = sp->nch; st.is_last = sp->is_last;
  st.in_prev = a.cur ? sp->in_act[0] : sp->in_act[1];
  st.out_cur = a.cur ? sp->out_act[1] : sp->out_act[0];
  st.gin_prev = a.cur ? sp->gin[0] : sp->gin[1];
  st.n_gparts = sp->n_gparts; st.gin_ld = sp->gin_ld;
  st.eout_cur = a.cur ? sp->eout[1] : sp->eout[0];
  st.n_parts = sp->n_parts;
  st.mW = sp->mW; st.vW = sp->vW; st.mb = sp->mb; st.vb = sp->vb;
  {
    // ring slots of this tick: written at tick % n, read what was written d ticks ago
    const int od = sp->out_dim, t = a.tick;
    st.skip_in = sp->skip_in ? sp->skip_in + (size_t)((t + sp->skip_in_n - sp->skip_in_d) % sp->skip_in_n) * od : nullptr;
    st.skip_out = sp->skip_out ? sp->skip_out + (size_t)(t % sp->skip_out_n) * od : nullptr;
    st.serr_out = sp->serr_out ? sp->serr_out + (size_t)(t % sp->serr_out_n) * od : nullptr;
    st.serr_in = sp->serr_in ? sp->serr_in + (size_t)((t + sp->serr_in_n - sp->serr_in_d) % sp->serr_in_n) * od : nullptr;
  }
  if constexpr (OPT == 1) {
    switch (st.nch) {
      case 1: run_tile<WT, 1, rows_per_iter_adam<WT>(1), LEARN, NW, NBUF, COH, 1>(net, st, tl, a, lds); break;
      case 2: run_tile<WT, 2, rows_per_iter_adam<WT>(2), LEARN, NW, NBUF, COH, 1>(net, st, tl, a, lds); break;
      case 4: run_tile<WT, 4, rows_per_iter_adam<WT>(4), LEARN, NW, NBUF, COH, 1>(net, st, tl, a, lds); break;
      case 8: run_tile<WT, 8, rows_per_iter_adam<WT>(8), LEARN, NW, NBUF, COH, 1>(net, st, tl, a, lds); break;
      case 16:
        if constexpr (WTraits<WT>::EPL == 4) run_tile<WT, 16, 1, LEARN, NW, NBUF, COH, 1>(net, st, tl, a, lds);
        break;
      default: break;
    }
    return;
  }
  switch (st.nch) {
    case 1: run_tile<WT, 1, rows_per_iter<WT>(1), LEARN, NW, NBUF, COH>(net, st, tl, a, lds); break;
    case 2: run_tile<WT, 2, rows_per_iter<WT>(2), LEARN, NW, NBUF, COH>(net, st, tl, a, lds); break;
    case 4: run_tile<WT, 4, rows_per_iter<WT>(4), LEARN, NW, NBUF, COH>(net, st, tl, a, lds); break;
    case 8: run_tile<WT, 8, rows_per_iter<WT>(8), LEARN, NW, NBUF, COH>(net, st, tl, a, lds); break;
    case 16:
      if constexpr (WTraits<WT>::EPL == 4) run_tile<WT, 16, 1, LEARN, NW, NBUF, COH>(net, st, tl, a, lds);
      break;
    default: break;
  }
}

// All work-groups of the (co-resident) grid meet here between two ticks (step a7).  Whatever one work-group
// hands to another goes through device-scope accesses (ld_x / st_x), so no cache-wide write-back or
// invalidate is needed: every wave waits until its own stores have been acknowledged, the work-group
// synchronises, one thread announces the arrival and waits for the others.  The wait is bounded: when it
// runs out the error flag is raised and every work-group leaves the kernel at its next check.
__device__ __forceinline__ bool grid_barrier(const BlockArgs &pa, unsigned long long target, int *flag_lds) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(pa.bar, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    long long spins = 0;
    int bad = 0;
    while (__hip_atomic_load(pa.bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(1);
      if (++spins > pa.spin_limit) {
        __hip_atomic_store(pa.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bad = 1;
        break;
      }
      if ((spins & 255) == 0 && __hip_atomic_load(pa.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
        bad = 1;
        break;
      }
    }
    *flag_lds = bad;
  }
  __syncthreads();
  return *flag_lds == 0;
}

template <typename WT, bool LEARN, int NW, int NBUF>
__global__ __launch_bounds__(NW * 64) void persistent_kernel(NetDev net, BlockArgs pa) {
  // (aligned: behind a static LDS variable of the kernel the array would otherwise start at an odd word, and every 16-byte
  // access to it would be a misaligned one: the 8 x 4096 fp32 workload ran 8 % slower that way)
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ int flag;
  for (int i = 0; i < pa.n_ticks; ++i) {
    const long long t = pa.t0 + i;
    TickArgs a;
    a.x = pa.x + (size_t)i * pa.in_stride;
    a.out = pa.out + (size_t)i * pa.out_stride;
    a.cur = (int)(t & 1);
    a.rev = pa.serp ? (int)(t & 1) : 0;
    a.tick = (int)(t & 0x3fffffff);
    a.head_target = pa.head_base + (unsigned int)(i + 1) * pa.head_parts;
    a.adam_c1 = a.adam_c2 = 0.f;
    a.learn = LEARN && pa.has_loss && t >= pa.fill;
    a.tgt = i >= pa.k ? pa.tgt + (size_t)(i - pa.k) * pa.tgt_bytes : pa.hist + (size_t)i * pa.tgt_bytes;
    a.lossp = pa.lossp + (size_t)i * pa.pl;
    a.loss1 = pa.loss ? pa.loss + i : pa.dummy;
    for (int tile = blockIdx.x; tile < net.n_tiles; tile += gridDim.x) {
      __syncthreads();   // the previous tile's LDS contents are dead from here on
      dispatch_tile<WT, LEARN, NW, NBUF, true>(net, net.tiles + tile, a, lds);
    }
    if (i + 1 < pa.n_ticks) {
      if (!grid_barrier(pa, pa.bar_base + (unsigned long long)(i + 1) * gridDim.x, &flag)) return;
    }
  }
}

template <typename WT, bool LEARN, int NW, int NBUF, int OPT = 0>
__global__ __launch_bounds__(NW * 64) void tick_kernel(NetDev net, TickArgs a) {
  // (aligned: behind a static LDS variable of the kernel the array would otherwise start at an odd word, and every 16-byte
  // access to it would be a misaligned one: the 8 x 4096 fp32 workload ran 8 % slower that way)
  extern __shared__ __attribute__((aligned(16))) float lds[];
  dispatch_tile<WT, LEARN, NW, NBUF, false, OPT>(net, net.tiles + blockIdx.x, a, lds);
}

__global__ void fill_kernel(float *p, int n, float v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

#include "ms_kernels.h"
#include "rb_kernels.h"
#include "conv_kernels.h"

__global__ void loss_finalize_kernel(const float *lossp, int n_parts, int n, float *loss) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float t = 0.f;
  for (int p = 0; p < n_parts; ++p) t += lossp[(size_t)i * n_parts + p];
  loss[i] = t;
}

// Plain streaming kernels over a private buffer: the bandwidth a kernel with no arithmetic reaches on this
// device, the measured ceiling the weight-streaming kernels are compared with (besides the published peak).
__global__ __launch_bounds__(256) void probe_read_kernel(const float4 *p, size_t n4, float *sink) {
  size_t stride = (size_t)gridDim.x * blockDim.x, i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  float s = 0.f;
  for (; i + 7 * stride < n4; i += 8 * stride) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ldg_f4(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u].x + v[u].y + v[u].z + v[u].w;
  }
  for (; i < n4; i += stride) { float4 v = ldg_f4(p + i); s += v.x + v.y + v.z + v.w; }
  if (s == 12345.678f) sink[0] = s;  // never true for the constant fill; keeps the loads alive
}
__global__ __launch_bounds__(256) void probe_update_kernel(float4 *p, size_t n4, float a) {
  size_t stride = (size_t)gridDim.x * blockDim.x, i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 7 * stride < n4; i += 8 * stride) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ldg_f4(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      v[u].x = v[u].x * a + 1.f; v[u].y = v[u].y * a + 1.f; v[u].z = v[u].z * a + 1.f; v[u].w = v[u].w * a + 1.f;
      stg_f4(p + i + u * stride, v[u]);
    }
  }
  for (; i < n4; i += stride) { float4 v = ldg_f4(p + i); v.x = v.x * a + 1.f; stg_f4(p + i, v); }
}
__global__ __launch_bounds__(256) void probe_write_kernel(float4 *p, size_t n4, float a) {
  size_t stride = (size_t)gridDim.x * blockDim.x, i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  float4 v = make_float4(a, a, a, a);
  for (; i < n4; i += stride) stg_f4(p + i, v);
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------

// Scratch of partime_step_noalloc: the per-tick loss partials of a block of ticks (one float per tile of the last
// stage and tick) followed by one block of dummy loss slots.  It lives in the code object, so every device the
// library runs on holds its own copy from the moment the module is loaded there until the process ends.  Host code
// never uses the symbol as an address: scratch_for() asks the runtime where the array sits on a device.
constexpr int kScratchParts = 256;                                        // most tiles the last stage may have
constexpr size_t kScratchFloats = (size_t)kLossSlots * kScratchParts + kLossSlots;   // 1 MiB + 4 KiB
static __device__ __align__(256) float g_scratch[kScratchFloats];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
float *g_scratch_ptr[kMaxDevices] = {};

// Description of the last failure on this thread.  A plain array on purpose: a thread-local object with a destructor
// is torn down while the process exits, in an order against the runtime's own exit handlers that the library does
// not control.
thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(PT_EHIP, "%s: %s", #expr, hipGetErrorString(e_));    \
  } while (0)

// Address of g_scratch on `device` (which must be the current device): looked up once per device and kept.
int scratch_for(int device, float **out) {
  if (device < 0 || device >= kMaxDevices) return fail(PT_EUNSUPPORTED, "device %d: at most %d devices", device, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur));
    if (cur != device) return fail(PT_EINVAL, "scratch lookup for device %d while device %d is current", device, cur);
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(g_scratch)));
    if (!p) return fail(PT_EHIP, "hipGetSymbolAddress gave a null address for the scratch array");
    g_scratch_ptr[device] = static_cast<float *>(p);
  }
  *out = g_scratch_ptr[device];
  return PT_OK;
}

unsigned short host_bf16_rne(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
  return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
float host_bf16_widen(unsigned short h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

struct StageHost {
  int layer;  // index of the layer this record describes (dense single-stream path: one record per layer)
  int stage = 0, pos = 0, cnt = 1;   // its pipeline stage, its place among the stage's layers, how many those are
  float *mW = nullptr, *vW = nullptr, *mb = nullptr, *vb = nullptr;   // Adam moments (fp32)
  float *skip_ring = nullptr, *serr_ring = nullptr;   // owned by the target layer of a skip: [delay + 1][out_dim] each
  int skip_delay = 0;                                 // stage boundaries the skip crosses
  size_t ring_bytes = 0;                              // size of each ring
  float *out_single = nullptr;       // output of a layer that is not the last of its stage (same tick, no ping-pong)
  float *e_single = nullptr;         // input-error partials of a layer that is not the first of its stage
  int in_dim, out_dim, ld, act, nch, rb;
  void *W = nullptr;
  float *b = nullptr;
  float *act_buf[2] = {nullptr, nullptr};
  float *err_buf[2] = {nullptr, nullptr};
  int n_parts = 0, rows_per_tile = 0;
  // multi-stream path: padded sizes and its extra buffers
  int in_pad = 0, out_pad = 0, n_rt = 0, tr = 0;
  float *zbuf = nullptr;
  float *zp = nullptr;               // multi-stream path: partial pre-activation planes of the coming tick [n_ct][S][out_pad]
  int n_ct = 0;
  bf16_t *dlt = nullptr, *dltT = nullptr, *xT0 = nullptr;
  bf16_t *WTq = nullptr, *xq0 = nullptr;   // batched path: transposed weights; first stage: rnd(x(t)) [S][in_pad]
  bf16_t *xq[2] = {nullptr, nullptr}, *xT[2] = {nullptr, nullptr};   // bf16 copies of what the stage publishes
  size_t act_elems = 0, err_elems = 0;   // elements of one half of act_buf / err_buf
};

struct CvStageHost {   // one record per conv layer
  int c_in = 0, c_out = kCvCo, H = 0, W = 0, act = 0, n_ft = 0, n_wt = 0;
  int ci_pad = kCvCo, co_pad = kCvCo;   // channel counts rounded up to blocks of 64: the kernels work on whole blocks,
                                        // the surplus channels have zero weights and biases and stay zero
  int stage = 0, pos = 0, cnt = 1;   // pipeline stage, place among the stage's layers, how many those are
  float *out_single = nullptr;       // output of a layer that is not the last of its stage (same tick)
  float *Wg = nullptr, *WT = nullptr, *WBT = nullptr, *b = nullptr, *delta = nullptr, *dwp = nullptr, *dbp = nullptr;
  float *mW = nullptr, *vW = nullptr, *mb = nullptr, *vb = nullptr;   // Adam moments, in the order of Wg and b
  float *act_buf[2] = {nullptr, nullptr}, *err_buf[2] = {nullptr, nullptr};
  float *skip_ring = nullptr, *serr_ring = nullptr;   // owned by the target layer of a skip: [delay + 1][co_pad][H][W] each
  int skip_delay = 0;                                 // stage boundaries the skip crosses
  size_t ring_bytes = 0;
};

}  // namespace

struct partime_ctx {
  partime_config cfg{};
  std::vector<pt_layer> layers;
  std::vector<StageHost> stages;
  std::vector<TileDev> tiles;
  std::vector<int> first_node;          // first layer record of every pipeline stage
  int cmax = 1;                         // most layers in one stage; a learning tick is 2 cmax - 1 launches
  std::vector<int> phase_off, phase_cnt;   // tiles of each launch of a tick
  hipStream_t stream = nullptr;
  int device = 0, n_cu = 0;
  int depth = 0, S = 1, esz = 4, fill = 0, k = 0;
  int in_dim = 0, out_dim = 0;
  float lr = 0.f;
  int64_t tick = 0;
  int64_t ring_period = 1;              // least common multiple of the lengths of all skip rings: the kernels choose
                                        // ring slots from the tick number modulo this
  NetDev net{};
  TileRec *d_tiles = nullptr;
  TileRec *d_tiles_inf = nullptr;       // inference-only tile list (bf16 weights: half-size tiles, two per compute unit)
  int n_tiles_inf = 0;
  float *d_lossp = nullptr;
  float *d_dummy = nullptr;
  unsigned char *d_hist[2] = {nullptr, nullptr};  // last k targets, oldest first; [hist_cur] is live
  int hist_cur = 0;
  size_t tgt_bytes = 0;
  size_t lds_bytes = 0;
  int last_launches = 0;
  int serpentine = 1;                   // walk tiles backwards on odd ticks: the rows touched last are touched first next tick
                                        // and are still in the memory-side cache
  int tiles_per_cu = 1;
  int nw = 8, nbuf = 1;                 // waves per work-group, row buffers per wave
  const void *k_learn = nullptr, *k_infer = nullptr;      // one launch per tick
  const void *k_plearn = nullptr, *k_pinfer = nullptr;    // one launch per block of ticks
  int max_grid = 0;                     // co-resident work-groups of the persistent kernels
  unsigned long long *d_bar = nullptr;  // barrier arrival counter
  int *d_err = nullptr;                 // deferred device-side error flag
  float *d_head_o = nullptr;            // softmax head split over several tiles: the stage's outputs of this tick
  unsigned int *d_head_ctr = nullptr;   // ... and the counter of tiles that have published theirs (monotonic)
  unsigned int head_count = 0;          // value of that counter once everything enqueued so far has run
  int head_parts = 0;                   // tiles of a softmax head that is split over several (0: none, or a single tile)
  unsigned long long bar_count = 0;     // arrivals enqueued so far
  long long spin_limit = 4000000;
  bool persistent = false;
  // multi-stream path
  bool ms = false;
  MsNet msnet{};
  MsTileRec *d_ms_tiles = nullptr;
  unsigned int *d_ms_head_ctr = nullptr;
  unsigned int ms_head_count = 0;       // what the counter reads once every head tile launched so far is done
  int ms_n_head = 0;                    // head tiles per learning tick
  float *d_ms_hstat = nullptr, *d_ms_hpart = nullptr;
  int n_prep = 0;                       // the first n_prep tiles of the first vector launch round the first layer's input
  int ms_tiles_f_off = 0;
  int n_tiles_f = 0, n_tiles_f0 = 0;    // forward-only matrix launch over the first layers of all stages; the first
                                        // n_tiles_f0 are the very first layer's
  // launches of a tick by position in the stage (offset into the tile array, count), each over all stages:
  std::vector<std::pair<int, int>> ms_vf, ms_mf, ms_vb, ms_mb, ms_if;   // vector forward [pos], matrix forward-only [pos >= 1],
                                        // vector backward [back >= 1], matrix learning [back] (back = layers behind it
                                        // in its stage; [0] carries the loss head), inference [pos]
  bool ms_zp_valid = false;             // the planes of the stages behind the first one are those of the coming tick
  // batched path (64 .. 1024 streams)
  bool rb = false;
  RbNet rbnet{};
  RbStage *d_rb_stages = nullptr;
  RbTile *d_rb_tiles = nullptr;
  float *d_rb_loss_s = nullptr;
  int rb_nu = 0, rb_u_off = 0, rb_tn = 128, rb_tm = 128, rb_rows = 0;
  std::vector<int> rb_f_off, rb_f_cnt, rb_b_off, rb_b_cnt;   // tiles of the forward / backward launches, by position in the stage
  size_t rb_lds_s = 0, rb_lds_u = 0;
  const void *rb_k_fwd[2] = {nullptr, nullptr}, *rb_k_bwd = nullptr, *rb_k_upd = nullptr;   // [learn]
  // convolutional path
  bool cv = false;
  CvNet cvnet{};
  std::vector<CvStageHost> cvs;
  CvStage *d_cv_stages = nullptr;
  CvTile *d_cv_tiles = nullptr;
  float *hd_W = nullptr, *hd_b = nullptr, *hd_gapv = nullptr, *hd_ge[2] = {nullptr, nullptr};
  float *hd_mW = nullptr, *hd_vW = nullptr, *hd_mb = nullptr, *hd_vb = nullptr;
  int n_cv_f = 0, n_cv_b = 0, n_cv_w = 0, cv_total_w = 0;
  size_t cv_lds_conv = 0, cv_lds_conv2 = 0, cv_lds_wg = 0;   // conv2: padded so that at most two work-groups share a compute unit
  std::vector<int> cv_f_off, cv_f_cnt, cv_b_off, cv_b_cnt;   // tiles of the forward / backward-data launches of a tick
  const void *cv_k_fwd[2] = {nullptr, nullptr}, *cv_k_bwd[2] = {nullptr, nullptr}, *cv_k_wg = nullptr;   // [learn]
};

namespace {

int nch_for(int ld, int epl) {
  const int per_chunk = 64 * epl;
  int need = (ld + per_chunk - 1) / per_chunk, n = 1;
  while (n < need) n *= 2;
  return n;
}

void free_ctx(partime_ctx *c) {
  if (!c) return;
  for (auto &s : c->stages) {
    if (s.W) (void)hipFree(s.W);
    if (s.b) (void)hipFree(s.b);
    if (s.zbuf) (void)hipFree(s.zbuf);
    if (s.zp) (void)hipFree(s.zp);
    if (s.dlt) (void)hipFree(s.dlt);
    if (s.dltT) (void)hipFree(s.dltT);
    if (s.xT0) (void)hipFree(s.xT0);
    if (s.WTq) (void)hipFree(s.WTq);
    if (s.xq0) (void)hipFree(s.xq0);
    for (int p = 0; p < 2; ++p) {
      if (s.xq[p]) (void)hipFree(s.xq[p]);
      if (s.xT[p]) (void)hipFree(s.xT[p]);
    }
    for (int p = 0; p < 2; ++p) {
      if (s.act_buf[p]) (void)hipFree(s.act_buf[p]);
      if (s.err_buf[p]) (void)hipFree(s.err_buf[p]);
    }
    if (s.out_single) (void)hipFree(s.out_single);
    if (s.e_single) (void)hipFree(s.e_single);
    for (float *q : {s.mW, s.vW, s.mb, s.vb, s.skip_ring, s.serr_ring})
      if (q) (void)hipFree(q);
  }
  if (c->d_tiles) (void)hipFree(c->d_tiles);
  if (c->d_tiles_inf) (void)hipFree(c->d_tiles_inf);
  if (c->d_lossp) (void)hipFree(c->d_lossp);
  if (c->d_dummy) (void)hipFree(c->d_dummy);
  for (auto &v : c->cvs) {
    for (float *q : {v.Wg, v.WT, v.WBT, v.b, v.delta, v.dwp, v.dbp, v.act_buf[0], v.act_buf[1], v.err_buf[0], v.err_buf[1], v.out_single, v.mW, v.vW, v.mb, v.vb, v.skip_ring, v.serr_ring})
      if (q) (void)hipFree(q);
  }
  for (float *q : {c->hd_W, c->hd_b, c->hd_gapv, c->hd_ge[0], c->hd_ge[1], c->hd_mW, c->hd_vW, c->hd_mb, c->hd_vb})
    if (q) (void)hipFree(q);
  if (c->d_cv_stages) (void)hipFree(c->d_cv_stages);
  if (c->d_cv_tiles) (void)hipFree(c->d_cv_tiles);
  if (c->d_rb_stages) (void)hipFree(c->d_rb_stages);
  if (c->d_rb_tiles) (void)hipFree(c->d_rb_tiles);
  if (c->d_rb_loss_s) (void)hipFree(c->d_rb_loss_s);
  if (c->d_ms_tiles) (void)hipFree(c->d_ms_tiles);
  if (c->d_ms_head_ctr) (void)hipFree(c->d_ms_head_ctr);
  if (c->d_ms_hstat) (void)hipFree(c->d_ms_hstat);
  if (c->d_ms_hpart) (void)hipFree(c->d_ms_hpart);
  if (c->d_bar) (void)hipFree(c->d_bar);
  if (c->d_head_o) (void)hipFree(c->d_head_o);
  if (c->d_head_ctr) (void)hipFree(c->d_head_ctr);
  if (c->d_err) (void)hipFree(c->d_err);
  for (int p = 0; p < 2; ++p)
    if (c->d_hist[p]) (void)hipFree(c->d_hist[p]);
  delete c;
}

int upload_weights(partime_ctx *c, int h, const float *w_host, const float *b_host) {
  StageHost &s = c->stages[h];
  if (w_host) {
    if (c->cfg.w_dtype == PT_F32) {
      HIP_TRY(hipMemcpy2D(s.W, (size_t)s.ld * 4, w_host, (size_t)s.in_dim * 4, (size_t)s.in_dim * 4, s.out_dim,
                          hipMemcpyHostToDevice));
    } else {
      if (c->ms) {
        // 32-stream path: the weights are kept in the order the matrix tiles request them
        std::vector<unsigned short> tiled((size_t)s.out_pad * s.in_pad, 0);
        for (int r = 0; r < s.out_dim; ++r)
          for (int q = 0; q < s.in_dim; ++q) tiled[ms_woff(r, q, s.out_pad)] = host_bf16_rne(w_host[(size_t)r * s.in_dim + q]);
        HIP_TRY(hipMemcpy(s.W, tiled.data(), tiled.size() * 2, hipMemcpyHostToDevice));
        if (b_host) HIP_TRY(hipMemcpy(s.b, b_host, (size_t)s.out_dim * 4, hipMemcpyHostToDevice));
        return PT_OK;
      }
      std::vector<unsigned short> tmp((size_t)s.out_dim * s.ld, 0);
      for (int r = 0; r < s.out_dim; ++r)
        for (int q = 0; q < s.in_dim; ++q) tmp[(size_t)r * s.ld + q] = host_bf16_rne(w_host[(size_t)r * s.in_dim + q]);
      HIP_TRY(hipMemcpy(s.W, tmp.data(), tmp.size() * 2, hipMemcpyHostToDevice));
      if (s.WTq) {
        // batched path: the backward product reads the transpose [in_pad][out_pad]
        std::vector<unsigned short> tr((size_t)s.in_pad * s.out_pad, 0);
        for (int r = 0; r < s.out_dim; ++r)
          for (int q = 0; q < s.in_dim; ++q) tr[(size_t)q * s.out_pad + r] = tmp[(size_t)r * s.ld + q];
        HIP_TRY(hipMemcpy(s.WTq, tr.data(), tr.size() * 2, hipMemcpyHostToDevice));
      }
    }
  }
  if (b_host) HIP_TRY(hipMemcpy(s.b, b_host, (size_t)s.out_dim * 4, hipMemcpyHostToDevice));
  return PT_OK;
}

// kernel variants: (waves per work-group, row buffers per wave)
template <typename WT, bool LEARN>
const void *pick_kernel(int nw, int nbuf, bool persistent, bool adam = false) {
  if (adam) return nw == 8 && nbuf == 1 ? reinterpret_cast<const void *>(&tick_kernel<WT, true, 8, 1, 1>) : nullptr;
#define PT_VARIANT(NW_, NB_)                                                                               \
  if (nw == NW_ && nbuf == NB_)                                                                            \
    return persistent ? reinterpret_cast<const void *>(&persistent_kernel<WT, LEARN, NW_, NB_>)           \
                      : reinterpret_cast<const void *>(&tick_kernel<WT, LEARN, NW_, NB_>);
  PT_VARIANT(8, 1)
#undef PT_VARIANT
  return nullptr;
}

// A stage with several layers (Eq. 3-5: exact back-propagation inside the stage) cannot do everything in one pass:
// layer j + 1 needs layer j's output of this tick, and layer j's delta needs layer j + 1's input-error of this
// tick.  A tick is therefore a short sequence of grouped launches ("phases"), each over all stages at once:
//   phases 0 .. cmax-2       forward-only passes of the layers that are not the last of their stage,
//   phase  cmax-1            the single-pass forward + backward + update of every stage's last layer,
//   phases cmax .. 2cmax-2   backward + update passes of the earlier layers, last to first; such a pass is the
//                            same fused pass again (z is recomputed from the row that is loaded anyway), with the
//                            error taken from the layer after it instead of from the next stage.
// Stages are aligned at the fused phase, so every launch is of one kind.  With one layer per stage cmax = 1 and a
// tick is the one fused launch.
int learn_phase_of(const StageHost &s, int cmax) { return cmax - 1 + (s.cnt - 1 - s.pos); }
int forward_phase_of(const StageHost &s, int cmax) { return cmax - s.cnt + s.pos; }   // == learn phase for the last layer

int build_plan(partime_ctx *c) {
  const int NL = (int)c->stages.size(), cmax = c->cmax;
  const int epl = c->cfg.w_dtype == PT_F32 ? 4 : 8;
  const int slots = std::max(1, c->n_cu * c->tiles_per_cu);
  int max_rows = 0, xs_len = 0;
  // rows per tile, per learning phase: about equal bytes per tile and never more tiles than work-group slots,
  // so that a launch is one round of work-groups (a single extra tile would cost a whole second round)
  for (int ph = cmax - 1; ph < 2 * cmax - 1; ++ph) {
    double total = 0;
    for (int i = 0; i < NL; ++i) {
      const StageHost &s = c->stages[i];
      if (learn_phase_of(s, cmax) != ph) continue;
      const bool head = i == NL - 1 && c->cfg.loss == PT_LOSS_CE;
      total += (double)s.out_dim * s.ld * c->esz * (head ? 2 : 1);   // the head reads twice
    }
    double per_tile = total / slots;
    for (int attempt = 0; attempt < 200; ++attempt) {
      int n_tiles = 0;
      for (int i = 0; i < NL; ++i) {
        StageHost &s = c->stages[i];
        if (learn_phase_of(s, cmax) != ph) continue;
        const int unit = c->nw * s.rb;
        const bool head = i == NL - 1 && c->cfg.loss == PT_LOSS_CE;
        // (a row of the softmax head counts twice: its tiles read their rows once for the outputs, once to learn)
        long want = std::lround(per_tile / ((double)s.ld * c->esz * (head ? 2 : 1)) / unit) * unit;
        int rows = (int)std::min<long>(std::max<long>(want, unit), kMaxTileRows);
        rows = std::min(rows, (s.out_dim + unit - 1) / unit * unit);
        s.rows_per_tile = rows;
        s.n_parts = (s.out_dim + rows - 1) / rows;
        n_tiles += s.n_parts;
      }
      if (n_tiles <= slots) break;
      per_tile *= 1.03;   // too many tiles: make them larger
    }
  }
  for (int i = 0; i < NL; ++i) {
    const StageHost &s = c->stages[i];
    max_rows = std::max(max_rows, std::min(s.rows_per_tile, s.out_dim));
    xs_len = std::max(xs_len, s.nch * 64 * epl);
  }
  // tiles of every phase, interleaved over the layers of the phase so that neighbouring work-groups (which land
  // on different XCDs) belong to different layers and each layer's input vector stays in few L2s.  A forward-only
  // phase walks the same row blocks as the layer's learning phase.
  c->tiles.clear();
  c->phase_off.assign(2 * cmax - 1, 0);
  c->phase_cnt.assign(2 * cmax - 1, 0);
  for (int ph = 0; ph < 2 * cmax - 1; ++ph) {
    c->phase_off[ph] = (int)c->tiles.size();
    int max_parts = 0;
    auto in_phase = [&](const StageHost &s) {
      return ph < cmax - 1 ? (s.pos < s.cnt - 1 && forward_phase_of(s, cmax) == ph) : learn_phase_of(s, cmax) == ph;
    };
    for (auto &s : c->stages)
      if (in_phase(s)) max_parts = std::max(max_parts, s.n_parts);
    auto push = [&](int i, int p) {
      const StageHost &s = c->stages[i];
      TileDev t;
      t.stage = i;
      t.row0 = p * s.rows_per_tile;
      t.nrows = std::min(s.rows_per_tile, s.out_dim - t.row0);
      t.part = p;
      c->tiles.push_back(t);
    };
    // The tiles of a softmax head wait for each other inside the launch: they come first, so that all of them are
    // running before any tile that could keep a compute unit from them.
    const int head_i = c->cfg.loss == PT_LOSS_CE && ph == cmax - 1 ? NL - 1 : -1;
    if (head_i >= 0)
      for (int p = 0; p < c->stages[head_i].n_parts; ++p) push(head_i, p);
    for (int p = 0; p < max_parts; ++p)
      for (int i = 0; i < NL; ++i)
        if (i != head_i && in_phase(c->stages[i]) && p < c->stages[i].n_parts) push(i, p);
    c->phase_cnt[ph] = (int)c->tiles.size() - c->phase_off[ph];
  }
  c->net.xs_len = xs_len;
  c->net.max_rows = max_rows;
  c->head_parts = c->cfg.loss == PT_LOSS_CE && c->stages[NL - 1].n_parts > 1 ? c->stages[NL - 1].n_parts : 0;
  c->net.head_parts = c->head_parts;
  // (a tile of the softmax head keeps all outputs of the stage where the error shares are reduced later)
  c->net.red_len = std::max({(c->nw / 2) * xs_len, (max_rows + 63) / 64 * 64, c->nw * 64,
                             c->cfg.loss == PT_LOSS_CE ? (c->stages[NL - 1].out_dim + 63) / 64 * 64 : 0});
  c->lds_bytes = ((size_t)xs_len + c->net.red_len + (size_t)max_rows * 5 + 2 * c->nw) * sizeof(float);
  if (c->lds_bytes > 160 * 1024) return fail(PT_EUNSUPPORTED, "tile needs %zu bytes of LDS", c->lds_bytes);
  return PT_OK;
}


// a skip ring of n slots joins the pipeline: the tick number handed to the kernels is taken modulo a common multiple
// of all ring lengths, so that slot = tick mod n stays right however long the stream runs
int add_ring_length(partime_ctx *c, int n) {
  int64_t a = c->ring_period, b = n;
  while (b) { const int64_t r = a % b; a = b; b = r; }
  const int64_t l = c->ring_period / a * n;
  if (l > (int64_t)1 << 30) return fail(PT_EUNSUPPORTED, "partime_init: the delays of the skip connections have no common period below 2^30 ticks");
  c->ring_period = l;
  return PT_OK;
}

// ---- multi-stream path: allocation and tile lists ------------------------------------------------

#define MS_TRY(expr)                                                                                   \
  do {                                                                                                 \
    hipError_t e_ = (expr);                                                                            \
    if (e_ != hipSuccess)                                                                              \
      return fail(e_ == hipErrorOutOfMemory ? PT_ENOMEM : PT_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

template <typename T>
int alloc_zero(T **p, size_t n) {
  MS_TRY(hipMalloc(reinterpret_cast<void **>(p), std::max<size_t>(n, 1) * sizeof(T)));
  MS_TRY(hipMemset(*p, 0, std::max<size_t>(n, 1) * sizeof(T)));
  return PT_OK;
}

int init_multistream(partime_ctx *c, const float *const *w_host, const float *const *b_host, const int *balance) {
  const int D = c->depth, NL = (int)c->layers.size(), S = c->S;
  c->ms = true;
  c->stages.resize(NL);               // one record per layer; a stage is a run of layers
  c->first_node.assign(D, 0);
  c->cmax = 1;
  for (int h = 0, i = 0; h < D; ++h) {
    const int cnt = balance ? balance[h] : 1;
    c->first_node[h] = i;
    c->cmax = std::max(c->cmax, cnt);
    for (int j = 0; j < cnt; ++j, ++i) {
      c->stages[i].stage = h; c->stages[i].pos = j; c->stages[i].cnt = cnt;
    }
  }
  const int cmax = c->cmax;
  auto pad512 = [](int v) { return (v + kMsTC - 1) / kMsTC * kMsTC; };   // every layer size is padded to whole column tiles
  for (int i = 0; i < NL; ++i) {
    StageHost &s = c->stages[i];
    const pt_layer &l = c->layers[i];
    s.layer = i;
    s.in_dim = l.in_dim;
    s.out_dim = l.out_dim;
    s.act = l.act;
    s.in_pad = pad512(l.in_dim);
    s.out_pad = pad512(l.out_dim);
    s.ld = s.in_pad;
    s.n_ct = s.in_pad / kMsTC;                     // column tiles = pre-activation planes
    s.act_elems = (size_t)S * s.out_pad;
  }
  // Tile height of a matrix launch.  A work-group holds one wave per SIMD, so a launch of more tiles than compute units
  // runs in rounds and the last one is rarely full: where taller tiles (fewer error planes as well) make the launch a
  // single round they are taken, per launch.  The last layer keeps the short tiles: they start only once the loss head is
  // done.  (The head tiles are not counted: they are gone within a few microseconds.)
  auto back_of = [&](const StageHost &s) { return s.cnt - 1 - s.pos; };
  for (int back = 0; back < cmax; ++back) {
    auto count_tiles = [&](int tr) {
      int n = 0;
      for (int i = 0; i < NL; ++i) {
        const StageHost &s = c->stages[i];
        if (back_of(s) != back) continue;
        const int t = i == NL - 1 ? std::min(tr, kMsTR) : tr;
        n += (s.out_pad + t - 1) / t * s.n_ct;
      }
      return n;
    };
    int tr_all = kMsTR;
    if (count_tiles(kMsTR) > c->n_cu)
      for (int tr = 2 * kMsTR; tr <= 8 * kMsTR; tr *= 2)
        if (count_tiles(tr) <= c->n_cu) { tr_all = tr; break; }
    for (int i = 0; i < NL; ++i) {
      StageHost &s = c->stages[i];
      if (back_of(s) != back) continue;
      s.tr = i == NL - 1 ? std::min(tr_all, kMsTR) : tr_all;
      s.n_rt = (s.out_pad + s.tr - 1) / s.tr;        // row tiles = error planes
      s.n_parts = s.n_rt;
      s.err_elems = (size_t)s.n_rt * S * s.in_pad;
    }
  }
  int rc;
  for (int i = 0; i < NL; ++i) {
    StageHost &s = c->stages[i];
    const bool last_in_stage = s.pos == s.cnt - 1;
    bf16_t *W = nullptr;
    if ((rc = alloc_zero(&W, (size_t)s.out_pad * s.in_pad)) != PT_OK) return rc;
    s.W = W;
    if ((rc = alloc_zero(&s.b, (size_t)s.out_pad)) != PT_OK) return rc;
    if (c->cfg.optimizer == PT_OPT_ADAM) {
      const size_t nw = (size_t)s.out_pad * s.in_pad;
      if ((rc = alloc_zero(&s.mW, nw)) != PT_OK || (rc = alloc_zero(&s.vW, nw)) != PT_OK) return rc;
      if ((rc = alloc_zero(&s.mb, (size_t)s.out_pad)) != PT_OK || (rc = alloc_zero(&s.vb, (size_t)s.out_pad)) != PT_OK) return rc;
    }
    if ((rc = alloc_zero(&s.zp, (size_t)s.n_ct * s.act_elems)) != PT_OK) return rc;
    if ((i == NL - 1 || !last_in_stage) && (rc = alloc_zero(&s.zbuf, s.act_elems)) != PT_OK) return rc;
    if ((rc = alloc_zero(&s.dlt, s.act_elems)) != PT_OK) return rc;
    if ((rc = alloc_zero(&s.dltT, s.act_elems)) != PT_OK) return rc;
    if (i == 0 && ((rc = alloc_zero(&s.xT0, (size_t)s.in_pad * S)) != PT_OK || (rc = alloc_zero(&s.xq0, (size_t)s.in_pad * S)) != PT_OK)) return rc;
    // what a layer publishes crosses a stage boundary as a ping-pong pair; inside a stage it is a single buffer of the
    // same tick (kept in half 0)
    for (int p = 0; p < 2; ++p) {
      if (i < NL - 1 && (p == 0 || last_in_stage)) {
        if ((rc = alloc_zero(&s.act_buf[p], s.act_elems)) != PT_OK) return rc;
        if ((rc = alloc_zero(&s.xq[p], s.act_elems)) != PT_OK) return rc;
        if ((rc = alloc_zero(&s.xT[p], s.act_elems)) != PT_OK) return rc;
      }
      if (i > 0 && (p == 0 || s.pos == 0) && (rc = alloc_zero(&s.err_buf[p], s.err_elems)) != PT_OK) return rc;
    }
    if (c->layers[i].skip_from >= 0) {
      // target of a skip: the rings of the skipped tensor and of its gradient, one slot per tick of delay and one more
      s.skip_delay = s.stage - c->stages[c->layers[i].skip_from].stage;
      const size_t n = (size_t)(s.skip_delay + 1) * S * s.out_pad;
      s.ring_bytes = n * 4;
      if ((rc = alloc_zero(&s.skip_ring, n)) != PT_OK || (rc = alloc_zero(&s.serr_ring, n)) != PT_OK) return rc;
      if ((rc = add_ring_length(c, s.skip_delay + 1)) != PT_OK) return rc;
    }
    if ((rc = upload_weights(c, i, w_host[i], b_host[i])) != PT_OK) return rc;
  }
  auto half = [](auto *const (&pair)[2], int p) { return pair[p] ? pair[p] : pair[0]; };
  std::vector<MsStage> sd(NL);
  for (int i = 0; i < NL; ++i) {
    StageHost &s = c->stages[i];
    MsStage &d = sd[i];
    std::memset(&d, 0, sizeof d);
    d.W = static_cast<bf16_t *>(s.W);
    d.b = s.b;
    d.mW = s.mW; d.vW = s.vW; d.mb = s.mb; d.vb = s.vb;
    d.in_dim = s.in_dim; d.out_dim = s.out_dim; d.in_pad = s.in_pad; d.out_pad = s.out_pad;
    d.act = s.act; d.is_last = i == NL - 1; d.is_first = i == 0; d.fold = s.pos == 0;
    d.zp = s.zp; d.n_ct = s.n_ct;
    d.zbuf = s.zbuf; d.dlt = s.dlt; d.dltT = s.dltT; d.xT0 = s.xT0; d.xq0 = s.xq0;
    for (int p = 0; p < 2; ++p) {
      d.out_act[p] = half(s.act_buf, p);
      d.xq_in[p] = i > 0 ? half(c->stages[i - 1].xq, p) : nullptr;
      d.xq_out[p] = half(s.xq, p);
      d.xT_in[p] = i > 0 ? half(c->stages[i - 1].xT, p) : nullptr;
      d.xT_out[p] = half(s.xT, p);
      d.gin[p] = i < NL - 1 ? half(c->stages[i + 1].err_buf, p) : nullptr;
      d.eout[p] = half(s.err_buf, p);
    }
    d.n_gparts = i < NL - 1 ? c->stages[i + 1].n_rt : 0;
    d.n_rt = s.n_rt; d.tr = s.tr;
    if (s.skip_ring) {
      d.skip_in = s.skip_ring; d.serr_out = s.serr_ring; d.skip_n = s.skip_delay + 1; d.skip_d = s.skip_delay;
    }
    for (int t = i + 1; t < NL; ++t)
      if (c->layers[t].skip_from == i) {   // the layer that adds this layer's output
        const StageHost &q = c->stages[t];
        d.skip_out = q.skip_ring; d.serr_in = q.serr_ring; d.src_n = q.skip_delay + 1; d.src_d = q.skip_delay;
      }
  }
  // tile lists, one per launch
  std::vector<MsTile> all;
  auto close_list = [&](std::vector<std::pair<int, int>> &lists, int at) {
    if ((int)lists.size() <= at) lists.resize(at + 1, {(int)all.size(), 0});
    lists[at].second = (int)all.size() - lists[at].first;
  };
  auto open_list = [&](std::vector<std::pair<int, int>> &lists, int at) {
    if ((int)lists.size() <= at) lists.resize(at + 1);
    lists[at] = {(int)all.size(), 0};
  };
  auto mat_tiles = [&](int i) {
    const StageHost &s = c->stages[i];
    for (int p = 0; p < s.n_rt; ++p)
      for (int q = 0; q < s.n_ct; ++q) all.push_back(MsTile{i, p, q, 0});
  };
  for (int pos = 0; pos < cmax; ++pos) {
    // vector launch of the layers at this position: forward and delta for a stage's last layer (its error signal is one
    // tick old, or comes from the loss head), forward alone otherwise
    open_list(c->ms_vf, pos);
    if (pos == 0) {
      for (int k0 = 0; k0 < c->stages[0].in_pad; k0 += kMsVR) all.push_back(MsTile{0, k0, 0, 1});   // the input of the first layer
      c->n_prep = (int)all.size() - c->ms_vf[0].first;
    }
    for (int i = 0; i < NL; ++i) {
      const StageHost &s = c->stages[i];
      if (s.pos != pos) continue;
      for (int r = 0; r < s.out_pad; r += kMsVR) all.push_back(MsTile{i, r, 0, s.pos == s.cnt - 1 ? 0 : 3});
    }
    close_list(c->ms_vf, pos);
    open_list(c->ms_mf, pos);
    if (pos > 0)
      for (int i = 0; i < NL; ++i)
        if (c->stages[i].pos == pos) mat_tiles(i);
    close_list(c->ms_mf, pos);
    open_list(c->ms_if, pos);
    for (int i = 0; i < NL; ++i) {
      const StageHost &s = c->stages[i];
      if (s.pos != pos) continue;
      for (int r = 0; r < s.out_pad; r += kMsRowsF) all.push_back(MsTile{i, r, kMsRowsF, 0});
    }
    close_list(c->ms_if, pos);
  }
  for (int back = 0; back < cmax; ++back) {
    open_list(c->ms_vb, back);
    if (back > 0)
      for (int i = 0; i < NL; ++i) {
        const StageHost &s = c->stages[i];
        if (back_of(s) != back) continue;
        for (int r = 0; r < s.out_pad; r += kMsVR) all.push_back(MsTile{i, r, 0, 4});
      }
    close_list(c->ms_vb, back);
    // matrix launch of a learning tick; the first one carries the loss head of the last layer in front and the last
    // layer's own tiles (which wait for the delta it provides) at its end
    open_list(c->ms_mb, back);
    if (back == 0) {
      for (int r = 0; r < c->stages[NL - 1].out_pad; r += kMsVR) all.push_back(MsTile{NL - 1, r, kMsVR, 2});
      c->ms_n_head = (int)all.size() - c->ms_mb[0].first;
    }
    {
      // Work-group i of a launch runs on die i mod 8, each die with its own L2, and the column tiles of one row tile read
      // the same deltas: row tiles are dealt out eight at a time (then four, two, one for what is left), column tile by
      // column tile, so that the column tiles of a row tile are 8 (4, 2) places apart and land on one die (two, four).
      auto deal = [&](const std::vector<std::pair<int, int>> &groups) {   // (layer, row tile)
        size_t g = 0;
        while (g < groups.size()) {
          size_t n = 8;
          for (;; n /= 2) {
            bool ok = g + n <= groups.size();
            for (size_t u = 1; ok && u < n; ++u) ok = c->stages[groups[g + u].first].n_ct == c->stages[groups[g].first].n_ct;
            if (ok) break;
          }
          for (int q = 0; q < c->stages[groups[g].first].n_ct; ++q)
            for (size_t u = 0; u < n; ++u) all.push_back(MsTile{groups[g + u].first, groups[g + u].second, q, 0});
          g += n;
        }
      };
      std::vector<std::pair<int, int>> groups, last;
      for (int i = 0; i < NL; ++i)
        if (back_of(c->stages[i]) == back)
          for (int p = 0; p < c->stages[i].n_rt; ++p) (i == NL - 1 ? last : groups).push_back({i, p});
      deal(groups);
      deal(last);   // (the last layer's tiles wait for the loss head: at the end of the launch)
    }
    close_list(c->ms_mb, back);
  }
  {
    // forward-only matrix launch for the planes a folded pass could not form: the very first layer's, then the other
    // stages' first layers
    const int at = (int)all.size();
    mat_tiles(0);
    c->n_tiles_f0 = (int)all.size() - at;
    for (int i = 1; i < NL; ++i)
      if (c->stages[i].pos == 0) mat_tiles(i);
    c->n_tiles_f = (int)all.size() - at;
    c->ms_tiles_f_off = at;
  }
  {
    // every tile carries a copy of its layer's record (one memory round trip less at the start of every work-group)
    std::vector<MsTileRec> recs(all.size());
    for (size_t q = 0; q < all.size(); ++q) { recs[q].t = all[q]; recs[q].s = sd[all[q].stage]; }
    MS_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_ms_tiles), sizeof(MsTileRec) * recs.size()));
    MS_TRY(hipMemcpy(c->d_ms_tiles, recs.data(), sizeof(MsTileRec) * recs.size(), hipMemcpyHostToDevice));
  }
  c->msnet.tiles_v = c->msnet.tiles_m = c->msnet.tiles_f = c->msnet.tiles_i = c->d_ms_tiles;   // set per launch
  c->msnet.loss = c->cfg.loss;
  c->msnet.out_dim = c->out_dim;
  c->msnet.lr_over_s = c->lr / (float)S;
  c->msnet.inv_s = 1.f / (float)S;
  c->msnet.adam = c->cfg.optimizer == PT_OPT_ADAM;
  c->msnet.beta1 = c->cfg.beta1; c->msnet.beta2 = c->cfg.beta2; c->msnet.eps = c->cfg.eps;
  MS_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_ms_head_ctr), sizeof(unsigned int)));
  MS_TRY(hipMemset(c->d_ms_head_ctr, 0, sizeof(unsigned int)));
  c->msnet.head_flag = c->d_ms_head_ctr;
  c->ms_head_count = 0;
  if ((rc = alloc_zero(&c->d_ms_hstat, (size_t)c->ms_n_head * S * 2)) != PT_OK) return rc;
  if ((rc = alloc_zero(&c->d_ms_hpart, (size_t)c->ms_n_head)) != PT_OK) return rc;
  c->msnet.hstat = c->d_ms_hstat;
  c->msnet.hpart = c->d_ms_hpart;
  c->msnet.spin_limit = c->spin_limit;
  if ((rc = alloc_zero(&c->d_dummy, (size_t)std::max(kLossSlots, c->out_dim))) != PT_OK) return rc;
  for (int p = 0; p < 2; ++p)
    if ((rc = alloc_zero(&c->d_hist[p], std::max<size_t>(1, (size_t)c->k) * c->tgt_bytes)) != PT_OK) return rc;
  if ((rc = alloc_zero(&c->d_err, 1)) != PT_OK) return rc;
  c->msnet.err = c->d_err;
  c->ms_zp_valid = false;
  MS_TRY(hipDeviceSynchronize());
  return PT_OK;
}

// ---- batched path (64 .. 1024 streams): allocation and tile lists ------------------------------------

int init_batched(partime_ctx *c, const float *const *w_host, const float *const *b_host, const int *balance) {
  const int D = c->depth, NL = (int)c->layers.size(), S = c->S;
  const bool adam = c->cfg.optimizer == PT_OPT_ADAM;
  c->rb = true;
  c->stages.resize(NL);               // one record per layer; a stage is a run of layers
  c->first_node.assign(D, 0);
  c->cmax = 1;
  for (int h = 0, i = 0; h < D; ++h) {
    const int cnt = balance ? balance[h] : 1;
    c->first_node[h] = i;
    c->cmax = std::max(c->cmax, cnt);
    for (int j = 0; j < cnt; ++j, ++i) {
      c->stages[i].stage = h; c->stages[i].pos = j; c->stages[i].cnt = cnt;
    }
  }
  auto pad = [](int v) { return (v + kRbTM - 1) / kRbTM * kRbTM; };
  int rc;
  for (int h = 0; h < NL; ++h) {
    StageHost &s = c->stages[h];
    const pt_layer &l = c->layers[h];
    const bool last_of_stage = s.pos == s.cnt - 1, final = h == NL - 1;
    s.layer = h;
    s.in_dim = l.in_dim; s.out_dim = l.out_dim; s.act = l.act;
    s.in_pad = pad(l.in_dim); s.out_pad = pad(l.out_dim);
    s.ld = s.in_pad;
    s.n_rt = s.n_parts = 1;
    s.act_elems = (size_t)S * s.out_pad;
    s.err_elems = (size_t)S * s.in_pad;
    const size_t nw = (size_t)s.out_pad * s.in_pad;
    bf16_t *W = nullptr;
    if ((rc = alloc_zero(&W, nw)) != PT_OK) return rc;
    s.W = W;
    if ((rc = alloc_zero(&s.WTq, nw)) != PT_OK) return rc;
    if ((rc = alloc_zero(&s.b, (size_t)s.out_pad)) != PT_OK) return rc;
    if (adam) {
      if ((rc = alloc_zero(&s.mW, nw)) != PT_OK || (rc = alloc_zero(&s.vW, nw)) != PT_OK) return rc;
      if ((rc = alloc_zero(&s.mb, (size_t)s.out_pad)) != PT_OK || (rc = alloc_zero(&s.vb, (size_t)s.out_pad)) != PT_OK) return rc;
    }
    if ((rc = alloc_zero(&s.dlt, s.act_elems)) != PT_OK || (rc = alloc_zero(&s.dltT, s.act_elems)) != PT_OK) return rc;
    if ((final || !last_of_stage) && (rc = alloc_zero(&s.zbuf, s.act_elems)) != PT_OK) return rc;
    if (h == 0 && ((rc = alloc_zero(&s.xq0, s.err_elems)) != PT_OK || (rc = alloc_zero(&s.xT0, s.err_elems)) != PT_OK)) return rc;
    // what the layer hands on: across a stage boundary a ping-pong pair (read one tick later), inside a stage one
    // buffer of the same tick; the error of a stage's first layer likewise
    for (int p = 0; p < (last_of_stage ? 2 : 1); ++p)
      if (!final && ((rc = alloc_zero(&s.xq[p], s.act_elems)) != PT_OK || (rc = alloc_zero(&s.xT[p], s.act_elems)) != PT_OK)) return rc;
    for (int p = 0; p < 2; ++p)
      if (h > 0 && s.pos == 0 && (rc = alloc_zero(&s.err_buf[p], s.err_elems)) != PT_OK) return rc;
    if (l.skip_from >= 0) {
      // target of a skip: the rings of the skipped tensor and of its gradient, one slot per tick of delay and one more
      s.skip_delay = s.stage - c->stages[l.skip_from].stage;
      const size_t n = (size_t)(s.skip_delay + 1) * S * s.out_pad;
      s.ring_bytes = n * 4;
      if ((rc = alloc_zero(&s.skip_ring, n)) != PT_OK || (rc = alloc_zero(&s.serr_ring, n)) != PT_OK) return rc;
      if ((rc = add_ring_length(c, s.skip_delay + 1)) != PT_OK) return rc;
    }
    if ((rc = upload_weights(c, h, w_host[h], b_host[h])) != PT_OK) return rc;
  }
  // stream tiles are 128 wide when the streams fill them, else 64.  Tiles are 128 rows tall: 256-row tiles (8 waves per
  // work-group, one work-group per compute unit) were measured 10-20 % slower at 1024 streams and no faster at 256,
  // although they pull a quarter less out of the L2 per product
  c->rb_tn = S % 128 == 0 ? 128 : 64;
  if (c->rb_tn == 128) {
    // a forward launch covers the layers of one position: when 128-wide tiles would not even give every compute unit
    // one (few stages, small batch), 64-wide ones are faster (two-stage 8 x 4096 network, 256 streams: +8 %)
    std::vector<int> per_pos(c->cmax, 0);
    for (int h = 0; h < NL; ++h) per_pos[c->stages[h].pos] += (c->stages[h].out_pad / kRbTM) * (S / 128);
    if (*std::max_element(per_pos.begin(), per_pos.end()) < c->n_cu) c->rb_tn = 64;
    if (const char *e = std::getenv("PARTIME_RB_TN")) c->rb_tn = std::atoi(e) == 64 ? 64 : 128;
  }
  c->rb_tm = kRbTM;
  const int TM = c->rb_tm;
  std::vector<RbStage> sd(NL);
  std::vector<std::vector<RbTile>> tfp(c->cmax), tbp(c->cmax);   // forward / backward launches by position in the stage
  std::vector<RbTile> tu;
  c->rb_rows = 0;
  for (int h = 0; h < NL; ++h) {
    StageHost &s = c->stages[h];
    RbStage &d = sd[h];
    const bool first_of_stage = s.pos == 0, last_of_stage = s.pos == s.cnt - 1, final = h == NL - 1;
    std::memset(&d, 0, sizeof d);
    d.W = static_cast<bf16_t *>(s.W); d.WT = s.WTq;
    d.b = s.b; d.mW = s.mW; d.vW = s.vW; d.mb = s.mb; d.vb = s.vb;
    d.in_dim = s.in_dim; d.out_dim = s.out_dim; d.in_pad = s.in_pad; d.out_pad = s.out_pad;
    d.act = s.act; d.is_last = final;
    d.dlt = s.dlt; d.dltT = s.dltT; d.zbuf = s.zbuf;
    d.fuse_delta = last_of_stage && !final;
    auto target_of = [&](int src) -> const StageHost * {   // the layer that adds layer src's output, if any
      for (int t = src + 1; t < NL; ++t)
        if (c->layers[t].skip_from == src) return &c->stages[t];
      return nullptr;
    };
    if (s.skip_ring) {
      d.skip_in = s.skip_ring; d.serr_out = s.serr_ring; d.skip_n = s.skip_delay + 1; d.skip_d = s.skip_delay;
    }
    if (const StageHost *t = target_of(h)) {
      d.skip_out = t->skip_ring; d.serr_in = t->serr_ring; d.src_n = t->skip_delay + 1; d.src_d = t->skip_delay;
    }
    if (!first_of_stage) {
      const StageHost &q = c->stages[h - 1];
      d.pred_dlt = q.dlt; d.pred_dltT = q.dltT; d.pred_z = q.zbuf; d.pred_act = q.act;
      if (q.skip_ring) { d.pred_serr_out = q.serr_ring; d.pred_skip_n = q.skip_delay + 1; }
      if (const StageHost *t = target_of(h - 1)) {
        d.pred_serr_in = t->serr_ring; d.pred_src_n = t->skip_delay + 1; d.pred_src_d = t->skip_delay;
      }
    }
    for (int p = 0; p < 2; ++p) {
      // inputs: the caller's batch, the previous stage's pair, or the single buffer of the layer in front
      d.xq_in[p] = h == 0 ? s.xq0 : (first_of_stage ? c->stages[h - 1].xq[p] : c->stages[h - 1].xq[0]);
      d.xT_in[p] = h == 0 ? s.xT0 : (first_of_stage ? c->stages[h - 1].xT[p] : c->stages[h - 1].xT[0]);
      d.xq_out[p] = last_of_stage ? s.xq[p] : s.xq[0];
      d.xT_out[p] = last_of_stage ? s.xT[p] : s.xT[0];
      d.gin[p] = d.fuse_delta ? c->stages[h + 1].err_buf[p] : nullptr;
      d.eout[p] = s.err_buf[p];
    }
    c->rb_rows += s.out_pad;
    // squares of up to 8 x 8 tiles, one after the other: 64 tiles that follow each other share 8 + 8 operand panels
    auto blocked = [&](std::vector<RbTile> &dst, int m_end, int n_end, int tn) {
      for (int mb = 0; mb < m_end; mb += 8 * TM)
        for (int nb = 0; nb < n_end; nb += 8 * tn)
          for (int m = mb; m < std::min(m_end, mb + 8 * TM); m += TM)
            for (int n = nb; n < std::min(n_end, nb + 8 * tn); n += tn) dst.push_back(RbTile{h, m, n});
    };
    blocked(tfp[s.pos], s.out_pad, S, c->rb_tn);
    if (h > 0) blocked(tbp[s.pos], s.in_pad, S, c->rb_tn);
    // the update streams the weights and moments once and its operands are small: tiles simply walk along the rows
    for (int n = 0; n < s.out_pad; n += 128)
      for (int m = 0; m < s.in_pad; m += TM) tu.push_back(RbTile{h, m, n});
  }
  // Work-groups go to the 8 dies of the chip in turn (work-group i to die i % 8), and each die has its own L2.  The
  // launch order of the forward and backward products therefore deals the list out in 8 contiguous shares, one per
  // die, so that the 64 work-groups a die runs at a time are one of the squares above and fetch each operand panel
  // into that L2 once: measured at 1024 streams, 2.1 -> 0.9 GB (forward) and 1.7 -> 0.6 GB (backward) from HBM per
  // tick, at the same speed (the products are not bound by HBM).  The update launch keeps its plain order: dealt out
  // like this it was measured 7 % slower.
  auto per_die = [](std::vector<RbTile> &t) {
    const size_t n = t.size(), share = (n + 7) / 8;
    std::vector<RbTile> out(share * 8, RbTile{-1, 0, 0});
    for (size_t i = 0; i < n; ++i) out[(i % share) * 8 + i / share] = t[i];
    t.swap(out);
  };
  std::vector<RbTile> all;
  c->rb_f_off.clear(); c->rb_f_cnt.clear(); c->rb_b_off.clear(); c->rb_b_cnt.clear();
  for (auto &t : tfp) {
    per_die(t);
    c->rb_f_off.push_back((int)all.size()); c->rb_f_cnt.push_back((int)t.size());
    all.insert(all.end(), t.begin(), t.end());
  }
  for (auto &t : tbp) {
    if (!t.empty()) per_die(t);
    c->rb_b_off.push_back((int)all.size()); c->rb_b_cnt.push_back((int)t.size());
    all.insert(all.end(), t.begin(), t.end());
  }
  c->rb_u_off = (int)all.size();
  c->rb_nu = (int)tu.size();
  all.insert(all.end(), tu.begin(), tu.end());
  MS_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_rb_stages), sizeof(RbStage) * NL));
  MS_TRY(hipMemcpy(c->d_rb_stages, sd.data(), sizeof(RbStage) * NL, hipMemcpyHostToDevice));
  MS_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_rb_tiles), sizeof(RbTile) * all.size()));
  MS_TRY(hipMemcpy(c->d_rb_tiles, all.data(), sizeof(RbTile) * all.size(), hipMemcpyHostToDevice));
  if ((rc = alloc_zero(&c->d_rb_loss_s, (size_t)S)) != PT_OK) return rc;
  RbNet &n = c->rbnet;
  n.stages = c->d_rb_stages;
  n.tiles = c->d_rb_tiles;
  n.S = S; n.n_stages = NL; n.loss = c->cfg.loss; n.out_dim = c->out_dim; n.in_dim = c->in_dim; n.adam = adam;
  n.lr = c->lr; n.inv_s = 1.f / (float)S;
  n.beta1 = c->cfg.beta1; n.beta2 = c->cfg.beta2; n.eps = c->cfg.eps;
  n.xq0 = c->stages[0].xq0; n.xT0 = c->stages[0].xT0; n.in_pad0 = c->stages[0].in_pad;
  n.loss_s = c->d_rb_loss_s;
#define RB_SET(TM_, TN_)                                                                                        \
  do {                                                                                                            \
    c->rb_k_fwd[0] = reinterpret_cast<const void *>(&rb_gemm_kernel<RB_FWD, TM_, TN_, false, 0>);                 \
    c->rb_k_fwd[1] = reinterpret_cast<const void *>(&rb_gemm_kernel<RB_FWD, TM_, TN_, true, 0>);                  \
    c->rb_k_bwd = reinterpret_cast<const void *>(&rb_gemm_kernel<RB_BWD, TM_, TN_, true, 0>);                     \
    c->rb_k_upd = adam ? reinterpret_cast<const void *>(&rb_gemm_kernel<RB_UPD, TM_, 128, true, 1>)               \
                       : reinterpret_cast<const void *>(&rb_gemm_kernel<RB_UPD, TM_, 128, true, 0>);              \
  } while (0)
  if (c->rb_tn == 128) RB_SET(kRbTM, 128);
  else RB_SET(kRbTM, 64);
#undef RB_SET
  // the operand buffers, or the fp32 tile of the epilogue, whichever is larger
  auto lds_for = [&](int tn) { return std::max((size_t)(2 * TM + 2 * tn) * kRbPitch * 2, (size_t)tn * (TM + 4) * 4); };
  c->rb_lds_s = lds_for(c->rb_tn);
  c->rb_lds_u = lds_for(128);
  for (const void *k : {c->rb_k_fwd[0], c->rb_k_fwd[1], c->rb_k_bwd})
    MS_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->rb_lds_s));
  MS_TRY(hipFuncSetAttribute(c->rb_k_upd, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->rb_lds_u));
  if ((rc = alloc_zero(&c->d_dummy, (size_t)std::max(kLossSlots, c->out_dim))) != PT_OK) return rc;
  for (int p = 0; p < 2; ++p)
    if ((rc = alloc_zero(&c->d_hist[p], std::max<size_t>(1, (size_t)c->k) * c->tgt_bytes)) != PT_OK) return rc;
  if ((rc = alloc_zero(&c->d_err, 1)) != PT_OK) return rc;
  MS_TRY(hipDeviceSynchronize());
  return PT_OK;
}

// ---- convolutional path: allocation and tile lists -----------------------------------------------

// host copies of the two tap-major weight layouts the forward and the backward-data products read
// (wg: [co_pad][c_in * 9], rows >= c_out zero)
void cv_make_layouts(const float *wg, int c_in, int co_pad, int ci_pad, std::vector<float> &wt, std::vector<float> &wbt) {
  const int cin_p = (c_in + 1) & ~1;
  wt.assign((size_t)cin_p * 9 * co_pad, 0.f);
  wbt.assign((size_t)co_pad * 9 * ci_pad, 0.f);
  for (int co = 0; co < co_pad; ++co)
    for (int ci = 0; ci < c_in; ++ci)
      for (int tap = 0; tap < 9; ++tap) {
        const float w = wg[((size_t)co * c_in + ci) * 9 + tap];
        wt[((size_t)(co / kCvCo) * (cin_p * 9) + ci * 9 + tap) * kCvCo + co % kCvCo] = w;
        wbt[((size_t)(ci / kCvCo) * (co_pad * 9) + co * 9 + (8 - tap)) * kCvCo + ci % kCvCo] = w;
      }
}

int cv_upload(partime_ctx *c, int layer, const float *w_host, const float *b_host) {
  const int n_conv = (int)c->cvs.size();
  if (layer < n_conv) {
    CvStageHost &v = c->cvs[layer];
    if (w_host) {
      // the caller's [c_out][c_in][3][3], padded with zero rows to whole blocks of output channels
      std::vector<float> wg((size_t)v.co_pad * v.c_in * 9, 0.f), wt, wbt;
      std::memcpy(wg.data(), w_host, (size_t)v.c_out * v.c_in * 9 * 4);
      cv_make_layouts(wg.data(), v.c_in, v.co_pad, v.ci_pad, wt, wbt);
      MS_TRY(hipMemcpy(v.Wg, wg.data(), wg.size() * 4, hipMemcpyHostToDevice));
      MS_TRY(hipMemcpy(v.WT, wt.data(), wt.size() * 4, hipMemcpyHostToDevice));
      MS_TRY(hipMemcpy(v.WBT, wbt.data(), wbt.size() * 4, hipMemcpyHostToDevice));
    }
    if (b_host) {
      std::vector<float> bb(v.co_pad, 0.f);
      std::memcpy(bb.data(), b_host, (size_t)v.c_out * 4);
      MS_TRY(hipMemcpy(v.b, bb.data(), bb.size() * 4, hipMemcpyHostToDevice));
    }
  } else {
    const pt_layer &l = c->layers[layer];
    if (w_host) MS_TRY(hipMemcpy(c->hd_W, w_host, (size_t)l.out_dim * l.c_in * 4, hipMemcpyHostToDevice));
    if (b_host) MS_TRY(hipMemcpy(c->hd_b, b_host, (size_t)l.out_dim * 4, hipMemcpyHostToDevice));
  }
  return PT_OK;
}

inline int total_pieces(int n16) { return (n16 + 255) / 256; }

// launch through a kernel address chosen at init (two by-value arguments)
template <typename A, typename B>
hipError_t launch2(const void *k, int grid, int block, size_t lds, hipStream_t s, A &a, B &b) {
  void *args[2] = {&a, &b};
  return hipLaunchKernel(k, dim3(grid), dim3(block), args, lds, s);
}

// the conv kernels are compiled per frame width (every LDS offset is then an immediate)
template <int LW, bool RES>
void cv_set_kernels(partime_ctx *c) {
  c->cv_k_fwd[0] = reinterpret_cast<const void *>(&cv_conv_kernel<CV_FWD, false, LW, RES>);
  c->cv_k_fwd[1] = reinterpret_cast<const void *>(&cv_conv_kernel<CV_FWD, true, LW, RES>);
  c->cv_k_bwd[0] = reinterpret_cast<const void *>(&cv_conv_kernel<CV_BWD, false, LW, RES>);
  c->cv_k_bwd[1] = reinterpret_cast<const void *>(&cv_conv_kernel<CV_BWD, true, LW, RES>);
  c->cv_k_wg = LW >= 6 ? reinterpret_cast<const void *>(&cv_wgrad_kernel<64>) : reinterpret_cast<const void *>(&cv_wgrad_kernel<32>);
}
template <bool RES>
void cv_pick_width(partime_ctx *c, int W) {
  switch (W) {
    case 32: cv_set_kernels<5, RES>(c); break;
    case 64: cv_set_kernels<6, RES>(c); break;
    case 128: cv_set_kernels<7, RES>(c); break;
    default: cv_set_kernels<8, RES>(c); break;
  }
}
void cv_pick_kernels(partime_ctx *c, int W) {
  bool res = false;
  for (const pt_layer &l : c->layers) res = res || l.skip_from >= 0;
  if (res) cv_pick_width<true>(c, W);
  else cv_pick_width<false>(c, W);
}

int init_conv(partime_ctx *c, const float *const *w_host, const float *const *b_host, const int *balance) {
  const int D = c->depth, NL = (int)c->layers.size(), n_conv = NL - 1;
  const pt_layer &hl = c->layers[NL - 1];
  const int H = c->layers[0].h, W = c->layers[0].w, HW = H * W;
  if (hl.kind != PT_GAP_DENSE || n_conv < 1) return fail(PT_EUNSUPPORTED, "partime_init: a conv pipeline ends with one pooled dense layer");
  if (balance && balance[D - 1] != 1) return fail(PT_EUNSUPPORTED, "partime_init: the pooled dense layer must be a stage of its own");
  if (c->S != 1 || c->cfg.w_dtype != PT_F32) return fail(PT_EUNSUPPORTED, "partime_init: conv pipelines are built for one fp32 stream");
  if (W % 32 || kCvPx % W || H % (kCvPx / W)) return fail(PT_EUNSUPPORTED, "partime_init: conv frames need w in {32,64,128,256} and h a multiple of 256/w");
  if (hl.c_in != c->layers[n_conv - 1].c_out || hl.h != H || hl.w != W || hl.out_dim <= 0 || hl.out_dim > 1024)
    return fail(PT_ESHAPE, "partime_init: the pooled head must take %d x %d x %d", c->layers[n_conv - 1].c_out, H, W);
  for (int h = 0; h < n_conv; ++h) {
    const pt_layer &l = c->layers[h];
    if (l.kind != PT_CONV3X3 || l.c_out <= 0 || l.c_out > kCvMaxC || l.c_in <= 0 || l.c_in > kCvMaxC || l.h != H || l.w != W)
      return fail(PT_EUNSUPPORTED, "partime_init: layer %d: conv stages are 3x3 with at most %d channels in and out, one frame size", h, kCvMaxC);
    if (h > 0 && l.c_in != c->layers[h - 1].c_out)
      return fail(PT_ESHAPE, "partime_init: layer %d takes %d channels, layer %d gives %d", h, l.c_in, h - 1, c->layers[h - 1].c_out);
    if (l.skip_from >= 0 && c->layers[l.skip_from].c_out != l.c_out)
      return fail(PT_ESHAPE, "partime_init: layer %d adds the output of layer %d: %d channels != %d", h, l.skip_from, l.c_out, c->layers[l.skip_from].c_out);
  }
  c->cv = true;
  c->in_dim = c->layers[0].c_in * HW;
  c->out_dim = hl.out_dim;
  c->tgt_bytes = c->cfg.loss == PT_LOSS_MSE ? (size_t)c->out_dim * 4 : 4;
  c->cvs.resize(n_conv);
  c->first_node.assign(D, 0);
  c->cmax = 1;
  for (int h = 0, i = 0; h < D - 1; ++h) {
    const int cnt = balance ? balance[h] : 1;
    c->first_node[h] = i;
    c->cmax = std::max(c->cmax, cnt);
    for (int j = 0; j < cnt; ++j, ++i) {
      c->cvs[i].stage = h;
      c->cvs[i].pos = j;
      c->cvs[i].cnt = cnt;
    }
  }
  c->first_node[D - 1] = n_conv;
  const int TR = kCvPx / W;
  const bool adam = c->cfg.optimizer == PT_OPT_ADAM;
  int rc;
  for (int h = 0; h < n_conv; ++h) {
    CvStageHost &v = c->cvs[h];
    v.c_in = c->layers[h].c_in; v.c_out = c->layers[h].c_out; v.H = H; v.W = W; v.act = c->layers[h].act;
    v.ci_pad = (v.c_in + kCvCo - 1) / kCvCo * kCvCo;
    v.co_pad = (v.c_out + kCvCo - 1) / kCvCo * kCvCo;
    v.n_ft = H / TR;
    v.n_wt = (H + kCvWgRows - 1) / kCvWgRows;
    const size_t nw = (size_t)v.co_pad * v.c_in * 9;
    if ((rc = alloc_zero(&v.Wg, nw)) || (rc = alloc_zero(&v.WT, (size_t)((v.c_in + 1) & ~1) * 9 * v.co_pad)) ||
        (rc = alloc_zero(&v.WBT, (size_t)v.co_pad * 9 * v.ci_pad)) || (rc = alloc_zero(&v.b, (size_t)v.co_pad)) ||
        (rc = alloc_zero(&v.delta, (size_t)v.co_pad * HW)) || (rc = alloc_zero(&v.dwp, (size_t)v.n_wt * nw)) ||
        (rc = alloc_zero(&v.dbp, (size_t)v.n_ft * v.co_pad)))
      return rc;
    if (adam && ((rc = alloc_zero(&v.mW, nw)) || (rc = alloc_zero(&v.vW, nw)) || (rc = alloc_zero(&v.mb, (size_t)v.co_pad)) ||
                 (rc = alloc_zero(&v.vb, (size_t)v.co_pad))))
      return rc;
    if (v.pos < v.cnt - 1 && (rc = alloc_zero(&v.out_single, (size_t)v.co_pad * HW))) return rc;
    if (c->layers[h].skip_from >= 0) {
      // target of a skip: the rings of the skipped map and of its gradient, one frame per tick of delay and one more
      v.skip_delay = v.stage - c->cvs[c->layers[h].skip_from].stage;
      const size_t n = (size_t)(v.skip_delay + 1) * v.co_pad * HW;
      v.ring_bytes = n * 4;
      if ((rc = alloc_zero(&v.skip_ring, n)) || (rc = alloc_zero(&v.serr_ring, n))) return rc;
      if ((rc = add_ring_length(c, v.skip_delay + 1)) != PT_OK) return rc;
    }
    for (int p = 0; p < 2; ++p) {
      if (v.pos == v.cnt - 1 && (rc = alloc_zero(&v.act_buf[p], (size_t)v.co_pad * HW))) return rc;
      if (v.pos == 0 && v.stage > 0 && (rc = alloc_zero(&v.err_buf[p], (size_t)v.ci_pad * HW))) return rc;
    }
  }
  const int c_last = c->layers[n_conv - 1].c_out, c_last_pad = c->cvs[n_conv - 1].co_pad;
  if ((rc = alloc_zero(&c->hd_W, (size_t)hl.out_dim * c_last)) || (rc = alloc_zero(&c->hd_b, (size_t)hl.out_dim)) ||
      (rc = alloc_zero(&c->hd_gapv, (size_t)c_last_pad)) || (rc = alloc_zero(&c->hd_ge[0], (size_t)c_last_pad)) ||
      (rc = alloc_zero(&c->hd_ge[1], (size_t)c_last_pad)))
    return rc;
  if (adam && ((rc = alloc_zero(&c->hd_mW, (size_t)hl.out_dim * c_last)) || (rc = alloc_zero(&c->hd_vW, (size_t)hl.out_dim * c_last)) ||
               (rc = alloc_zero(&c->hd_mb, (size_t)hl.out_dim)) || (rc = alloc_zero(&c->hd_vb, (size_t)hl.out_dim))))
    return rc;
  for (int h = 0; h < NL; ++h)
    if ((rc = cv_upload(c, h, w_host[h], b_host[h])) != PT_OK) return rc;

  // links: across a stage boundary through the ping-pong halves (previous tick), inside a stage through
  // single buffers of this tick (both "halves" name the same buffer)
  std::vector<CvStage> sd(n_conv);
  std::vector<CvTile> tw;
  std::vector<std::vector<CvTile>> tf(c->cmax), tb(c->cmax);
  c->cv_total_w = 0;
  for (int h = 0; h < n_conv; ++h) {
    CvStageHost &v = c->cvs[h];
    CvStage &d = sd[h];
    std::memset(&d, 0, sizeof d);
    d.Wg = v.Wg; d.WT = v.WT; d.WBT = v.WBT; d.b = v.b; d.mW = v.mW; d.vW = v.vW; d.mb = v.mb; d.vb = v.vb; d.c_in = v.c_in; d.c_out = v.c_out; d.ci_pad = v.ci_pad; d.co_pad = v.co_pad; d.H = H; d.W = W; d.act = v.act;
    d.delta = v.delta; d.dwp = v.dwp; d.dbp = v.dbp; d.n_ft = v.n_ft; d.n_wt = v.n_wt;
    const bool first = v.pos == 0, last = v.pos == v.cnt - 1, before_head = h == n_conv - 1;
    d.fuse_delta = last;
    d.pred_delta = first ? nullptr : c->cvs[h - 1].delta;
    d.pred_dbp = first ? nullptr : c->cvs[h - 1].dbp;
    d.pred_act = first ? PT_ID : c->cvs[h - 1].act;
    if (v.skip_ring) {
      d.skip_in = v.skip_ring; d.serr_out = v.serr_ring; d.skip_n = v.skip_delay + 1; d.skip_d = v.skip_delay;
    }
    for (int t = h + 1; t < n_conv; ++t)
      if (c->layers[t].skip_from == h) {   // this layer's output is skipped to layer t
        const CvStageHost &q = c->cvs[t];
        d.skip_out = q.skip_ring; d.serr_in = q.serr_ring; d.src_n = q.skip_delay + 1; d.src_d = q.skip_delay;
      }
    for (int p = 0; p < 2; ++p) {
      d.in_act[p] = h == 0 ? nullptr : (first ? c->cvs[h - 1].act_buf[p] : c->cvs[h - 1].out_single);
      d.out_act[p] = last ? v.act_buf[p] : v.out_single;
      d.gin[p] = last && !before_head ? c->cvs[h + 1].err_buf[p] : nullptr;
      d.ge[p] = before_head ? c->hd_ge[p] : nullptr;
      d.eout[p] = v.err_buf[p];
    }
    // forward launch number pos; backward-data launch number cnt - 1 - pos (none for the very first layer:
    // nobody needs the error of the frame)
    // Work-group i of a launch runs on die i mod 8 and neighbouring row tiles of a layer read the same halo rows: the n row
    // tiles of a layer are dealt out so that a die gets n / 8 neighbours (position j * 8 + d <-> row tile d * (n / 8) + j)
    auto dealt = [](int n, int i) { return n % 8 ? i : (i % 8) * (n / 8) + i / 8; };
    const int n_rows = H / TR;
    for (int ob = 0; ob < v.co_pad / kCvCo; ++ob)
      for (int i = 0; i < n_rows; ++i) tf[v.pos].push_back(CvTile{h, dealt(n_rows, i) * TR, ob, 0});
    if (h > 0)
      for (int ib = 0; ib < v.ci_pad / kCvCo; ++ib)
        for (int i = 0; i < n_rows; ++i) tb[v.cnt - 1 - v.pos].push_back(CvTile{h, dealt(n_rows, i) * TR, ib, 0});
    for (int i = 0; i < v.n_wt; ++i)
      for (int ib = 0; ib < v.ci_pad / kCvCo; ++ib)
        for (int ob = 0; ob < v.co_pad / kCvCo; ++ob) tw.push_back(CvTile{h, dealt(v.n_wt, i), ib, ob});
    c->cv_total_w += v.co_pad * v.c_in * 9 + v.co_pad;
  }
  {
    // the pooling tiles go first: they are short, and behind the conv tiles they would start a round of their own
    std::vector<CvTile> pool;
    for (int ch = 0; ch < c_last; ++ch) pool.push_back(CvTile{0, ch, 0, 1});
    tf[0].insert(tf[0].begin(), pool.begin(), pool.end());
  }
  tb[0].insert(tb[0].begin(), CvTile{0, 0, 0, 2});   // the head first: an inference tick launches that tile alone
  std::vector<CvTile> all;
  c->cv_f_off.clear(); c->cv_f_cnt.clear(); c->cv_b_off.clear(); c->cv_b_cnt.clear();
  for (auto &t : tf) { c->cv_f_off.push_back((int)all.size()); c->cv_f_cnt.push_back((int)t.size()); all.insert(all.end(), t.begin(), t.end()); }
  for (auto &t : tb) { c->cv_b_off.push_back((int)all.size()); c->cv_b_cnt.push_back((int)t.size()); all.insert(all.end(), t.begin(), t.end()); }
  const int w_off = (int)all.size();
  all.insert(all.end(), tw.begin(), tw.end());
  c->n_cv_f = c->cv_f_cnt[0]; c->n_cv_b = c->cv_b_cnt[0]; c->n_cv_w = (int)tw.size();
  MS_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_cv_stages), sizeof(CvStage) * n_conv));
  MS_TRY(hipMemcpy(c->d_cv_stages, sd.data(), sizeof(CvStage) * n_conv, hipMemcpyHostToDevice));
  MS_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_cv_tiles), sizeof(CvTile) * all.size()));
  MS_TRY(hipMemcpy(c->d_cv_tiles, all.data(), sizeof(CvTile) * all.size(), hipMemcpyHostToDevice));
  CvNet &n = c->cvnet;
  n.stages = c->d_cv_stages;
  n.tiles_f = c->d_cv_tiles + c->cv_f_off[0];
  n.tiles_b = c->d_cv_tiles + c->cv_b_off[0];
  n.tiles_w = c->d_cv_tiles + w_off;
  n.n_conv = n_conv; n.loss = c->cfg.loss; n.lr = c->lr;
  n.adam = adam; n.beta1 = c->cfg.beta1; n.beta2 = c->cfg.beta2; n.eps = c->cfg.eps;
  n.head.mW = c->hd_mW; n.head.vW = c->hd_vW; n.head.mb = c->hd_mb; n.head.vb = c->hd_vb;
  n.head.W = c->hd_W; n.head.b = c->hd_b; n.head.c = c_last; n.head.out = hl.out_dim; n.head.hw = HW;
  n.head.gapv = c->hd_gapv;
  for (int p = 0; p < 2; ++p) {
    n.head.in_act[p] = c->cvs[n_conv - 1].act_buf[p];
    n.head.ge[p] = c->hd_ge[p];
  }
  // conv kernel: two buffers of kCvCiCh channels x (tile rows + 2) x (W + 8); the head tile needs 3200 floats.
  // weight-gradient kernel: eight rings of 3 rows x 16 channels x (columns + 12).
  const int PR = TR + 2;
  if (total_pieces(kCvCiCh * PR * (W / 4)) > kCvNQ) return fail(PT_EUNSUPPORTED, "partime_init: conv frame shape needs more staging pieces than the kernel holds");
  c->cv_lds_conv = std::max<size_t>((size_t)2 * kCvCiCh * PR * (W + 8) * 4, 3200 * 4);
  c->cv_lds_wg = (size_t)8 * 3 * kCvWgCi * (std::min(W, kCvWgXC) + 12) * 4;
  // A launch of up to two tiles per compute unit must not pack three work-groups into some units and none into
  // others (the dispatcher fills a unit before it moves on): asking for more than a third of the LDS caps it at two.
  c->cv_lds_conv2 = std::max<size_t>(c->cv_lds_conv, 56 * 1024);
  cv_pick_kernels(c, W);
  for (const void *k : {c->cv_k_fwd[0], c->cv_k_fwd[1], c->cv_k_bwd[0], c->cv_k_bwd[1]})
    MS_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->cv_lds_conv2));
  MS_TRY(hipFuncSetAttribute(c->cv_k_wg, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->cv_lds_wg));
  if ((rc = alloc_zero(&c->d_dummy, (size_t)std::max(kLossSlots, c->out_dim))) != PT_OK) return rc;
  for (int p = 0; p < 2; ++p)
    if ((rc = alloc_zero(&c->d_hist[p], std::max<size_t>(1, (size_t)c->k) * c->tgt_bytes)) != PT_OK) return rc;
  if ((rc = alloc_zero(&c->d_err, 1)) != PT_OK) return rc;
  MS_TRY(hipDeviceSynchronize());
  return PT_OK;
}

}  // namespace

extern "C" {

const char *partime_last_error(void) { return g_err; }

int partime_init(const partime_config *cfg, const float *const *w_host, const float *const *b_host,
                 partime_ctx **out) {
  if (!cfg || !w_host || !b_host || !out) return fail(PT_EINVAL, "partime_init: null argument");
  *out = nullptr;
  if (cfg->n_layers <= 0 || !cfg->layers || cfg->depth <= 0) return fail(PT_EINVAL, "partime_init: empty network");
  if (cfg->n_streams <= 0) return fail(PT_EINVAL, "partime_init: n_streams must be positive");
  if (cfg->w_dtype != PT_F32 && cfg->w_dtype != PT_BF16) return fail(PT_EINVAL, "partime_init: bad w_dtype");
  if (cfg->loss != PT_LOSS_MSE && cfg->loss != PT_LOSS_CE && cfg->loss != PT_LOSS_NONE)
    return fail(PT_EINVAL, "partime_init: bad loss");
  if (cfg->target_delay < 0) return fail(PT_EINVAL, "partime_init: negative target_delay");
  if (cfg->exec_mode < PT_EXEC_AUTO || cfg->exec_mode > PT_EXEC_PERSISTENT)
    return fail(PT_EINVAL, "partime_init: bad exec_mode");
  int nsum = 0;
  for (int h = 0; h < cfg->depth; ++h) {
    const int n = cfg->balance ? cfg->balance[h] : 1;
    if (n <= 0) return fail(PT_EINVAL, "partime_init: balance[%d] = %d", h, n);
    nsum += n;
  }
  if (nsum != cfg->n_layers) return fail(PT_ESHAPE, "partime_init: balance sums to %d, n_layers is %d", nsum, cfg->n_layers);
  bool any_conv = false;
  for (int i = 0; i < cfg->n_layers; ++i) any_conv = any_conv || cfg->layers[i].kind != PT_DENSE;
  for (int i = 0; i < cfg->n_layers; ++i) {
    const pt_layer &l = cfg->layers[i];
    if (!w_host[i] || !b_host[i]) return fail(PT_EINVAL, "partime_init: null weights for layer %d", i);
    if (l.kind < PT_DENSE || l.kind > PT_GAP_DENSE) return fail(PT_EINVAL, "partime_init: layer %d: bad kind", i);
    if (l.act < PT_ID || l.act > PT_GELU) return fail(PT_EINVAL, "partime_init: layer %d: bad activation", i);
    if (l.kind == PT_DENSE && (l.in_dim <= 0 || l.out_dim <= 0))
      return fail(PT_EINVAL, "partime_init: layer %d: non-positive size", i);
    if (l.kind != PT_DENSE && (l.c_in <= 0 || l.h <= 0 || l.w <= 0 || (l.kind == PT_CONV3X3 ? l.c_out : l.out_dim) <= 0))
      return fail(PT_EINVAL, "partime_init: layer %d: non-positive size", i);
    if (any_conv) continue;   // the conv pipeline checks its own chain of shapes
    if (i > 0 && cfg->layers[i - 1].out_dim != l.in_dim)
      return fail(PT_ESHAPE, "partime_init: layer %d takes %d inputs, layer %d gives %d", i, l.in_dim, i - 1,
                  cfg->layers[i - 1].out_dim);
    if (cfg->n_streams == 1 && l.in_dim > kMaxIn)
      return fail(PT_EUNSUPPORTED, "partime_init: layer %d: in_dim %d > %d", i, l.in_dim, kMaxIn);
  }
  for (int i = 0; i < cfg->n_layers; ++i) {
    const int sf = cfg->layers[i].skip_from;
    if (sf < -1 || sf >= i) return fail(PT_EINVAL, "partime_init: layer %d: skip_from must name an earlier layer or be -1", i);
    if (sf < 0) continue;
    if (cfg->exec_mode == PT_EXEC_PERSISTENT)
      return fail(PT_EUNSUPPORTED, "partime_init: skip connections take one launch per tick, not the persistent kernel");
    if (i == cfg->n_layers - 1) return fail(PT_EUNSUPPORTED, "partime_init: the last layer cannot be the target of a skip");
    if (!any_conv && cfg->layers[sf].out_dim != cfg->layers[i].out_dim)
      return fail(PT_ESHAPE, "partime_init: layer %d adds the output of layer %d: %d != %d", i, sf, cfg->layers[i].out_dim, cfg->layers[sf].out_dim);
    for (int q = 0; q < i; ++q)
      if (cfg->layers[q].skip_from == sf) return fail(PT_EUNSUPPORTED, "partime_init: layer %d is the source of two skips", sf);
  }
  if (cfg->optimizer != PT_OPT_SGD && cfg->optimizer != PT_OPT_ADAM) return fail(PT_EINVAL, "partime_init: bad optimizer");
  if (cfg->optimizer == PT_OPT_ADAM) {
    if (cfg->exec_mode == PT_EXEC_PERSISTENT)
      return fail(PT_EUNSUPPORTED, "partime_init: Adam takes one launch per tick, not the persistent kernel");
    if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f && cfg->beta2 >= 0.f && cfg->beta2 < 1.f && cfg->eps > 0.f))
      return fail(PT_EINVAL, "partime_init: Adam needs 0 <= beta1, beta2 < 1 and eps > 0");
  }
  if (cfg->depth != cfg->n_layers && cfg->exec_mode == PT_EXEC_PERSISTENT)
    return fail(PT_EUNSUPPORTED, "partime_init: the persistent kernel takes one layer per stage");
  const bool batched = cfg->n_streams >= 64 && cfg->n_streams % 64 == 0 && cfg->n_streams <= kRbMaxS;
  if (cfg->n_streams != 1 && ((cfg->n_streams != kMsS && !batched) || cfg->w_dtype != PT_BF16))
    return fail(PT_EUNSUPPORTED, "partime_init: several streams are built for n_streams = %d or a multiple of 64 up to %d, with bf16 weights only", kMsS, kRbMaxS);
  if (cfg->target_delay > kLossSlots) return fail(PT_EUNSUPPORTED, "partime_init: target_delay > %d", kLossSlots);
  if (!any_conv && cfg->loss == PT_LOSS_CE && cfg->layers[cfg->n_layers - 1].out_dim > kMaxHeadRows)
    return fail(PT_EUNSUPPORTED, "partime_init: softmax head wider than %d", kMaxHeadRows);

  partime_ctx *c = new (std::nothrow) partime_ctx;
  if (!c) return fail(PT_ENOMEM, "partime_init: out of host memory");
  c->cfg = *cfg;
  c->layers.assign(cfg->layers, cfg->layers + cfg->n_layers);
  c->cfg.layers = c->layers.data();
  c->cfg.balance = nullptr;
  c->stream = static_cast<hipStream_t>(cfg->hip_stream);
  c->depth = cfg->depth;
  c->S = cfg->n_streams;
  c->esz = cfg->w_dtype == PT_F32 ? 4 : 2;
  c->k = cfg->target_delay;
  c->fill = std::max(cfg->depth - 1, cfg->target_delay);
  c->lr = cfg->lr;
  c->in_dim = c->layers.front().in_dim;
  c->out_dim = c->layers.back().out_dim;

  auto bail = [&](int code) { free_ctx(c); return code; };
#define INIT_TRY(expr)                                                                                   \
  do {                                                                                                   \
    hipError_t e_ = (expr);                                                                              \
    if (e_ != hipSuccess)                                                                                \
      return bail(fail(e_ == hipErrorOutOfMemory ? PT_ENOMEM : PT_EHIP, "%s: %s", #expr, hipGetErrorString(e_))); \
  } while (0)

  INIT_TRY(hipGetDevice(&c->device));
  {
    float *scr = nullptr;   // the static scratch of partime_step_noalloc, looked up once per device while it is current
    if (int rcs = scratch_for(c->device, &scr)) return bail(rcs);
  }
  hipDeviceProp_t prop;
  INIT_TRY(hipGetDeviceProperties(&prop, c->device));
  c->n_cu = prop.multiProcessorCount;

  c->tgt_bytes = c->cfg.loss == PT_LOSS_MSE ? (size_t)c->S * c->out_dim * 4 : (size_t)c->S * 4;
  if (const char *e = std::getenv("PARTIME_SPIN_LIMIT")) c->spin_limit = std::atoll(e);
  if (any_conv) {
    int rcc = init_conv(c, w_host, b_host, cfg->balance);
    if (rcc != PT_OK) return bail(rcc);
    *out = c;
    g_err[0] = 0;
    return PT_OK;
  }
  if (c->S > kMsS) {
    int rcb = init_batched(c, w_host, b_host, cfg->balance);
    if (rcb != PT_OK) return bail(rcb);
    *out = c;
    g_err[0] = 0;
    return PT_OK;
  }
  if (c->S > 1) {
    int rcm = init_multistream(c, w_host, b_host, cfg->balance);
    if (rcm != PT_OK) return bail(rcm);
    *out = c;
    g_err[0] = 0;
    return PT_OK;
  }
  // one record per layer ("node"); a stage is a run of nodes
  const int D = c->depth, NL = (int)c->layers.size(), epl = c->cfg.w_dtype == PT_F32 ? 4 : 8;
  c->stages.resize(NL);
  c->first_node.assign(D, 0);
  c->cmax = 1;
  for (int h = 0, i = 0; h < D; ++h) {
    const int cnt = cfg->balance ? cfg->balance[h] : 1;
    c->first_node[h] = i;
    c->cmax = std::max(c->cmax, cnt);
    for (int j = 0; j < cnt; ++j, ++i) {
      c->stages[i].stage = h;
      c->stages[i].pos = j;
      c->stages[i].cnt = cnt;
    }
  }
  for (int h = 0; h < NL; ++h) {
    StageHost &s = c->stages[h];
    const pt_layer &l = c->layers[h];
    s.layer = h;
    s.in_dim = l.in_dim;
    s.out_dim = l.out_dim;
    s.act = l.act;
    s.ld = (l.in_dim + epl - 1) / epl * epl;
    s.nch = nch_for(s.ld, epl);
    s.rb = c->cfg.w_dtype == PT_F32 ? rows_per_iter<float>(s.nch) : rows_per_iter<bf16_t>(s.nch);
    if (c->cfg.w_dtype == PT_BF16 && s.nch > 8) return bail(fail(PT_EUNSUPPORTED, "partime_init: internal nch"));
  }
  if (c->cfg.w_dtype == PT_F32) {
    c->k_learn = pick_kernel<float, true>(c->nw, c->nbuf, false);
    c->k_infer = pick_kernel<float, false>(c->nw, c->nbuf, false);
    c->k_plearn = pick_kernel<float, true>(c->nw, c->nbuf, true);
    c->k_pinfer = pick_kernel<float, false>(c->nw, c->nbuf, true);
  } else {
    c->k_learn = pick_kernel<bf16_t, true>(c->nw, c->nbuf, false);
    c->k_infer = pick_kernel<bf16_t, false>(c->nw, c->nbuf, false);
    c->k_plearn = pick_kernel<bf16_t, true>(c->nw, c->nbuf, true);
    c->k_pinfer = pick_kernel<bf16_t, false>(c->nw, c->nbuf, true);
  }
  if (c->cfg.optimizer == PT_OPT_ADAM) {
    c->nw = 8;
    c->nbuf = 1;
    c->k_learn = c->cfg.w_dtype == PT_F32 ? pick_kernel<float, true>(8, 1, false, true) : pick_kernel<bf16_t, true>(8, 1, false, true);
    c->k_infer = c->cfg.w_dtype == PT_F32 ? pick_kernel<float, false>(8, 1, false) : pick_kernel<bf16_t, false>(8, 1, false);
  }
  if (!c->k_learn || !c->k_infer) return bail(fail(PT_EINVAL, "no kernel variant %dx%d", c->nw, c->nbuf));
  int rc = build_plan(c);
  if (rc != PT_OK) return bail(rc);

  for (int h = 0; h < NL; ++h) {
    StageHost &s = c->stages[h];
    const size_t wbytes = (size_t)s.out_dim * s.ld * c->esz;
    INIT_TRY(hipMalloc(&s.W, wbytes));
    INIT_TRY(hipMemset(s.W, 0, wbytes));
    INIT_TRY(hipMalloc(&s.b, (size_t)s.out_dim * 4));
    const bool last_of_stage = s.pos == s.cnt - 1, first_of_stage = s.pos == 0;
    for (int p = 0; p < 2; ++p) {
      if (last_of_stage && s.stage < D - 1) {      // what the stage publishes for the next tick
        INIT_TRY(hipMalloc(&s.act_buf[p], (size_t)s.out_dim * 4));
        INIT_TRY(hipMemset(s.act_buf[p], 0, (size_t)s.out_dim * 4));
      }
      if (first_of_stage && s.stage > 0) {         // the input-error the stage publishes for the next tick
        INIT_TRY(hipMalloc(&s.err_buf[p], (size_t)s.n_parts * s.ld * 4));
        INIT_TRY(hipMemset(s.err_buf[p], 0, (size_t)s.n_parts * s.ld * 4));
      }
    }
    if (!last_of_stage) {
      INIT_TRY(hipMalloc(&s.out_single, (size_t)s.out_dim * 4));
      INIT_TRY(hipMemset(s.out_single, 0, (size_t)s.out_dim * 4));
    }
    if (!first_of_stage) {
      INIT_TRY(hipMalloc(&s.e_single, (size_t)s.n_parts * s.ld * 4));
      INIT_TRY(hipMemset(s.e_single, 0, (size_t)s.n_parts * s.ld * 4));
    }
    if (c->cfg.optimizer == PT_OPT_ADAM) {
      const size_t nw = (size_t)s.out_dim * s.ld;
      for (float **q : {&s.mW, &s.vW}) {
        INIT_TRY(hipMalloc(q, nw * 4));
        INIT_TRY(hipMemset(*q, 0, nw * 4));
      }
      for (float **q : {&s.mb, &s.vb}) {
        INIT_TRY(hipMalloc(q, (size_t)s.out_dim * 4));
        INIT_TRY(hipMemset(*q, 0, (size_t)s.out_dim * 4));
      }
    }
    if (c->layers[h].skip_from >= 0) {
      s.skip_delay = s.stage - c->stages[c->layers[h].skip_from].stage;
      const size_t n = (size_t)(s.skip_delay + 1) * s.out_dim;
      s.ring_bytes = n * 4;
      for (float **q : {&s.skip_ring, &s.serr_ring}) {
        INIT_TRY(hipMalloc(q, n * 4));
        INIT_TRY(hipMemset(*q, 0, n * 4));
      }
      if ((rc = add_ring_length(c, s.skip_delay + 1)) != PT_OK) return bail(rc);
    }
    rc = upload_weights(c, h, w_host[h], b_host[h]);
    if (rc != PT_OK) return bail(rc);
  }

  // links between the records: across a stage boundary through the ping-pong halves (previous tick), inside a
  // stage through single buffers of this tick (both "halves" name the same buffer)
  std::vector<StageDev> sd(NL);
  for (int h = 0; h < NL; ++h) {
    StageHost &s = c->stages[h];
    StageDev &d = sd[h];
    std::memset(&d, 0, sizeof d);
    d.W = s.W; d.b = s.b;
    d.in_dim = s.in_dim; d.out_dim = s.out_dim; d.ld = s.ld;
    d.act = s.act; d.nch = s.nch; d.is_last = h == NL - 1;
    for (int p = 0; p < 2; ++p) {
      d.in_act[p] = h == 0 ? nullptr : (s.pos > 0 ? c->stages[h - 1].out_single : c->stages[h - 1].act_buf[p]);
      d.out_act[p] = s.pos < s.cnt - 1 ? s.out_single : s.act_buf[p];
      d.gin[p] = h == NL - 1 ? nullptr : (s.pos < s.cnt - 1 ? c->stages[h + 1].e_single : c->stages[h + 1].err_buf[p]);
      d.eout[p] = s.pos > 0 ? s.e_single : s.err_buf[p];
    }
    d.n_gparts = h < NL - 1 ? c->stages[h + 1].n_parts : 0;
    d.gin_ld = h < NL - 1 ? c->stages[h + 1].ld : 0;
    d.n_parts = s.n_parts;
    d.mW = s.mW; d.vW = s.vW; d.mb = s.mb; d.vb = s.vb;
    if (s.skip_ring) {   // this layer is the target of a skip: it reads the tensor ring and writes the gradient ring
      d.skip_in = s.skip_ring; d.skip_in_n = s.skip_delay + 1; d.skip_in_d = s.skip_delay;
      d.serr_out = s.serr_ring; d.serr_out_n = s.skip_delay + 1;
    }
    for (int q = h + 1; q < NL; ++q)
      if (c->layers[q].skip_from == h) {   // ... and the source writes the tensor ring and reads the gradient ring
        const StageHost &t = c->stages[q];
        d.skip_out = t.skip_ring; d.skip_out_n = t.skip_delay + 1;
        d.serr_in = t.serr_ring; d.serr_in_n = t.skip_delay + 1; d.serr_in_d = t.skip_delay;
      }
  }
  auto with_layers = [&](const std::vector<TileDev> &tl) {
    std::vector<TileRec> r(tl.size());
    for (size_t q = 0; q < tl.size(); ++q) { r[q].t = tl[q]; r[q].s = sd[tl[q].stage]; }
    return r;
  };
  {
    const std::vector<TileRec> recs = with_layers(c->tiles);
    INIT_TRY(hipMalloc(&c->d_tiles, sizeof(TileRec) * recs.size()));
    INIT_TRY(hipMemcpy(c->d_tiles, recs.data(), sizeof(TileRec) * recs.size(), hipMemcpyHostToDevice));
  }
  if (c->cmax == 1 && c->cfg.w_dtype == PT_BF16 && c->tiles_per_cu == 1 && c->cfg.exec_mode != PT_EXEC_PERSISTENT) {
    // Inference with bf16 rows: a wave has half the bytes of an fp32 row in flight and nothing to write, and two
    // work-groups of half the rows per compute unit were measured 20 % faster (16 x 2048 x 2048: 25.9 against 30.9 us
    // per tick); for learning, and for fp32 rows either way, one tile per compute unit is the faster split.
    std::vector<TileDev> ti;
    std::vector<int> rows(NL), parts(NL);
    int max_parts = 0;
    for (int i = 0; i < NL; ++i) {
      const StageHost &s = c->stages[i];
      const int unit = c->nw * s.rb;
      rows[i] = std::max(unit, s.rows_per_tile / 2 / unit * unit);
      parts[i] = (s.out_dim + rows[i] - 1) / rows[i];
      max_parts = std::max(max_parts, parts[i]);
    }
    for (int p = 0; p < max_parts; ++p)
      for (int i = 0; i < NL; ++i) {
        if (p >= parts[i]) continue;
        TileDev t;
        t.stage = i;
        t.row0 = p * rows[i];
        t.nrows = std::min(rows[i], c->stages[i].out_dim - t.row0);
        t.part = 0;                       // error planes are not written by inference
        ti.push_back(t);
      }
    c->n_tiles_inf = (int)ti.size();
    const std::vector<TileRec> recs = with_layers(ti);
    INIT_TRY(hipMalloc(&c->d_tiles_inf, sizeof(TileRec) * recs.size()));
    INIT_TRY(hipMemcpy(c->d_tiles_inf, recs.data(), sizeof(TileRec) * recs.size(), hipMemcpyHostToDevice));
  }
  const int pl = c->stages[NL - 1].n_parts;
  INIT_TRY(hipMalloc(&c->d_lossp, sizeof(float) * kLossSlots * pl));
  INIT_TRY(hipMalloc(&c->d_dummy, sizeof(float) * std::max(kLossSlots, c->out_dim)));
  c->tgt_bytes = c->cfg.loss == PT_LOSS_MSE ? (size_t)c->S * c->out_dim * 4 : (size_t)c->S * 4;
  for (int p = 0; p < 2; ++p) {
    INIT_TRY(hipMalloc(&c->d_hist[p], std::max<size_t>(1, (size_t)c->k) * c->tgt_bytes));
    INIT_TRY(hipMemset(c->d_hist[p], 0, std::max<size_t>(1, (size_t)c->k) * c->tgt_bytes));
  }

  c->net.tiles = c->d_tiles;
  c->net.depth = NL;
  c->net.n_tiles = (int)c->tiles.size();
  c->net.loss = c->cfg.loss;
  c->net.out_dim = c->out_dim;
  c->net.lr = c->lr;
  c->net.beta1 = cfg->beta1; c->net.beta2 = cfg->beta2; c->net.eps = cfg->eps;

  for (const void *k : {c->k_learn, c->k_infer, c->k_plearn, c->k_pinfer})
    INIT_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->lds_bytes));
  {
    // the persistent kernels wait for each other: only as many work-groups as are resident at once
    int nb_l = 0, nb_i = 0;
    INIT_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb_l, c->k_plearn, c->nw * 64, c->lds_bytes));
    INIT_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb_i, c->k_pinfer, c->nw * 64, c->lds_bytes));
    c->max_grid = std::min(nb_l, nb_i) * c->n_cu;
    if (c->max_grid <= 0) return bail(fail(PT_EHIP, "partime_init: the persistent kernel does not fit a compute unit"));
  }
  INIT_TRY(hipMalloc(&c->d_bar, sizeof(unsigned long long)));
  INIT_TRY(hipMemset(c->d_bar, 0, sizeof(unsigned long long)));
  INIT_TRY(hipMalloc(&c->d_err, sizeof(int)));
  INIT_TRY(hipMemset(c->d_err, 0, sizeof(int)));
  INIT_TRY(hipMalloc(&c->d_head_o, sizeof(float) * std::max(1, c->out_dim)));
  INIT_TRY(hipMemset(c->d_head_o, 0, sizeof(float) * std::max(1, c->out_dim)));
  INIT_TRY(hipMalloc(&c->d_head_ctr, sizeof(unsigned int)));
  INIT_TRY(hipMemset(c->d_head_ctr, 0, sizeof(unsigned int)));
  c->net.head_o = c->d_head_o; c->net.head_ctr = c->d_head_ctr; c->net.err = c->d_err; c->net.spin_limit = c->spin_limit;
  c->persistent = c->cfg.exec_mode == PT_EXEC_PERSISTENT;
  // (a work-group of the persistent kernel that takes several tiles in turn could wait for a head tile of its own)
  if (c->head_parts > 1 && c->tiles.size() > (size_t)c->max_grid) c->persistent = false;
  if (c->cmax > 1 || c->cfg.optimizer == PT_OPT_ADAM) c->persistent = false;   // no single-kernel form for these
  for (auto &l : c->layers)
    if (l.skip_from >= 0) c->persistent = false;
  INIT_TRY(hipDeviceSynchronize());
#undef INIT_TRY
  *out = c;
  g_err[0] = 0;
  return PT_OK;
}

void partime_destroy(partime_ctx *ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);
  free_ctx(ctx);
}

// lossp / dummy: where the dense single-stream path keeps the loss partials of a block of ticks and the loss slots
// nobody asked for (the context's own buffers, or the static scratch array)
static int run_ticks(partime_ctx *c, const float *x_dev, const void *target_dev, int n_ticks, float *out_dev,
                     float *loss_dev, bool learn, float *lossp = nullptr, float *dummy = nullptr) {
  const int pl = c->stages.empty() ? 1 : c->stages.back().n_parts;   // (the conv path keeps no dense stages)
  if (!lossp) lossp = c->d_lossp;
  if (!dummy) dummy = c->d_dummy;
  const dim3 grid((unsigned)c->tiles.size()), block(c->nw * 64);
  const unsigned char *tgt = static_cast<const unsigned char *>(target_dev);
  c->last_launches = 0;
  if (c->cv) {
    // convolutional path: forward, backward-data, weight-gradient and update launches per tick
    for (int i = 0; i < n_ticks; ++i) {
      const int64_t t = c->tick + i;
      CvTick a;
      a.x = x_dev + (size_t)i * c->in_dim;
      a.out = out_dev + (size_t)i * c->out_dim;
      a.cur = (int)(t & 1);
      a.tick = (int)(t % c->ring_period);
      a.adam_c1 = a.adam_c2 = 0.f;
      if (c->cfg.optimizer == PT_OPT_ADAM) {
        const double n = (double)(t + 1);
        a.adam_c1 = (float)((double)c->lr / (1.0 - std::pow((double)c->cfg.beta1, n)));
        a.adam_c2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)c->cfg.beta2, n)));
      }
      a.learn = learn && t >= c->fill && c->cfg.loss != PT_LOSS_NONE;
      a.tgt = nullptr;
      if (learn && c->cfg.loss != PT_LOSS_NONE)
        a.tgt = i >= c->k ? tgt + (size_t)(i - c->k) * c->tgt_bytes
                          : c->d_hist[c->hist_cur] + (size_t)i * c->tgt_bytes;
      a.loss1 = loss_dev ? loss_dev + i : c->d_dummy;
      const bool lrn = learn && c->cfg.loss != PT_LOSS_NONE;
      // forward launches front to back (one per layer position inside the stages) ...
      for (int ph = 0; ph < c->cmax; ++ph) {
        CvNet net = c->cvnet;
        net.tiles_f = c->d_cv_tiles + c->cv_f_off[ph];
        HIP_TRY(launch2(c->cv_k_fwd[lrn], c->cv_f_cnt[ph], 256, c->cv_f_cnt[ph] <= 2 * c->n_cu + kCvMaxC ? c->cv_lds_conv2 : c->cv_lds_conv,
                        c->stream, net, a));
        ++c->last_launches;
      }
      if (lrn) {
        // ... backward-data launches back to front (the first one also runs the head stage), then the weight
        // gradients of all layers and the update
        for (int ph = 0; ph < c->cmax; ++ph) {
          if (c->cv_b_cnt[ph] == 0) continue;
          CvNet net = c->cvnet;
          net.tiles_b = c->d_cv_tiles + c->cv_b_off[ph];
          HIP_TRY(launch2(c->cv_k_bwd[1], c->cv_b_cnt[ph], 256, c->cv_b_cnt[ph] <= 2 * c->n_cu + 1 ? c->cv_lds_conv2 : c->cv_lds_conv,
                          c->stream, net, a));
          ++c->last_launches;
        }
        HIP_TRY(launch2(c->cv_k_wg, c->n_cv_w, 512, c->cv_lds_wg, c->stream, c->cvnet, a));
        hipLaunchKernelGGL(cv_update_kernel, dim3((c->cv_total_w + 255) / 256), dim3(256), 0, c->stream, c->cvnet, c->cv_total_w, a.adam_c1, a.adam_c2);
        c->last_launches += 2;
      } else {
        HIP_TRY(launch2(c->cv_k_bwd[0], 1, 256, c->cv_lds_conv, c->stream, c->cvnet, a));
        ++c->last_launches;
      }
    }
    HIP_TRY(hipGetLastError());
  } else if (c->rb) {
    // batched path: every product of the tick is a grouped launch of the same tiled kernel
    for (int i = 0; i < n_ticks; ++i) {
      const int64_t t = c->tick + i;
      RbTick a;
      a.x = x_dev + (size_t)i * c->S * c->in_dim;
      a.out = out_dev + (size_t)i * c->S * c->out_dim;
      a.cur = (int)(t & 1);
      a.learn = learn && t >= c->fill && c->cfg.loss != PT_LOSS_NONE;
      a.tgt = nullptr;
      if (learn && c->cfg.loss != PT_LOSS_NONE)
        a.tgt = i >= c->k ? tgt + (size_t)(i - c->k) * c->tgt_bytes
                          : c->d_hist[c->hist_cur] + (size_t)i * c->tgt_bytes;
      a.loss1 = loss_dev ? loss_dev + i : c->d_dummy;
      a.tick = (int)(t % c->ring_period);
      a.adam_c1 = a.adam_c2 = 0.f;
      if (c->cfg.optimizer == PT_OPT_ADAM) {
        const double n = (double)(t + 1);
        a.adam_c1 = (float)((double)c->lr / (1.0 - std::pow((double)c->cfg.beta1, n)));
        a.adam_c2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)c->cfg.beta2, n)));
      }
      const bool lrn = learn && c->cfg.loss != PT_LOSS_NONE;
      RbNet net = c->rbnet;
      hipLaunchKernelGGL(rb_input_kernel, dim3((c->S / 64) * (net.in_pad0 / 64)), dim3(256), 0, c->stream, net, a);
      ++c->last_launches;
      // forward: one launch per position in the stage (a layer needs the output of the layer in front of it) ...
      for (int ph = 0; ph < c->cmax; ++ph) {
        net.tiles = c->d_rb_tiles + c->rb_f_off[ph];
        HIP_TRY(launch2(c->rb_k_fwd[lrn], c->rb_f_cnt[ph], 2 * c->rb_tm, c->rb_lds_s, c->stream, net, a));
        ++c->last_launches;
      }
      if (lrn) {
        hipLaunchKernelGGL(rb_head_kernel, dim3(c->S), dim3(256), 0, c->stream, net, a);
        // ... backward from the last position to the first (a layer's delta comes from the layer behind it), then
        // the biases and the weights of all layers
        for (int ph = c->cmax - 1; ph >= 0; --ph) {
          if (c->rb_b_cnt[ph] == 0) continue;
          net.tiles = c->d_rb_tiles + c->rb_b_off[ph];
          HIP_TRY(launch2(c->rb_k_bwd, c->rb_b_cnt[ph], 2 * c->rb_tm, c->rb_lds_s, c->stream, net, a));
          ++c->last_launches;
        }
        hipLaunchKernelGGL(rb_bias_kernel, dim3(c->rb_rows / 16 + 1), dim3(256), 0, c->stream, net, a, c->rb_rows);   // 4 waves x 4 rows + the loss
        net.tiles = c->d_rb_tiles + c->rb_u_off;
        HIP_TRY(launch2(c->rb_k_upd, c->rb_nu, 2 * c->rb_tm, c->rb_lds_u, c->stream, net, a));
        c->last_launches += 3;
      }
    }
    HIP_TRY(hipGetLastError());
  } else if (c->ms) {
    // multi-stream path.  A learning tick is a vector launch and a matrix launch; the matrix launch of tick t also forms
    // the pre-activation planes of tick t + 1.  What it could not form (the first stage's at the last tick of the previous
    // call: the caller's next sample was not known; everything after inference ticks or after the state was changed from
    // outside) is formed here first by a forward-only matrix launch.  An inference tick is one launch of its own kernel.
    MsNet net = c->msnet;
    auto vec = [&](bool lrn, const std::pair<int, int> &l, int count, const MsTick &a) {
      if (count <= 0) return;
      net.tiles_v = c->d_ms_tiles + l.first;
      if (lrn) hipLaunchKernelGGL(ms_vec_kernel<true>, dim3(count), dim3(256), 0, c->stream, net, a);
      else hipLaunchKernelGGL(ms_vec_kernel<false>, dim3(count), dim3(256), 0, c->stream, net, a);
      ++c->last_launches;
    };
    auto mat_fwd = [&](int off, int count, const MsTick &a) {
      if (count <= 0) return;
      net.tiles_f = c->d_ms_tiles + off;
      hipLaunchKernelGGL((ms_mat_kernel<1, 0>), dim3(count), dim3(64 * kMsNWM), 0, c->stream, net, a);
      ++c->last_launches;
    };
    auto mat_learn = [&](const std::pair<int, int> &l, const MsTick &a) {
      if (l.second <= 0) return;
      net.tiles_m = c->d_ms_tiles + l.first;
      if (c->cfg.optimizer == PT_OPT_ADAM)
        hipLaunchKernelGGL((ms_mat_kernel<0, 1>), dim3(l.second), dim3(64 * kMsNWM), 0, c->stream, net, a);
      else
        hipLaunchKernelGGL((ms_mat_kernel<0, 0>), dim3(l.second), dim3(64 * kMsNWM), 0, c->stream, net, a);
      ++c->last_launches;
    };
    if (learn) {
      MsTick a{};
      a.x = x_dev;
      a.x_next = x_dev;                       // the prep tiles round "the coming tick's" samples: here this tick's
      a.cur = (int)(c->tick & 1);
      a.fhalf = a.cur ^ 1;                    // inputs of tick t are what the stages published at tick t - 1
      vec(false, c->ms_vf[0], c->n_prep, a);
      mat_fwd(c->ms_tiles_f_off, c->ms_zp_valid ? c->n_tiles_f0 : c->n_tiles_f, a);
    }
    for (int i = 0; i < n_ticks; ++i) {
      const int64_t t = c->tick + i;
      MsTick a{};
      a.x = x_dev + (size_t)i * c->S * c->in_dim;
      a.x_next = i + 1 < n_ticks ? a.x + (size_t)c->S * c->in_dim : nullptr;
      a.out = out_dev + (size_t)i * c->S * c->out_dim;
      a.cur = (int)(t & 1);
      a.tick = (int)(t % c->ring_period);
      a.fhalf = a.cur;                        // inputs of tick t + 1 are what the stages publish in this tick
      a.learn = learn && t >= c->fill && c->cfg.loss != PT_LOSS_NONE;
      a.tgt = nullptr;
      if (learn && c->cfg.loss != PT_LOSS_NONE)
        a.tgt = i >= c->k ? tgt + (size_t)(i - c->k) * c->tgt_bytes
                          : c->d_hist[c->hist_cur] + (size_t)i * c->tgt_bytes;
      a.loss1 = loss_dev ? loss_dev + i : c->d_dummy;
      if (learn) c->ms_head_count += (unsigned int)c->ms_n_head;
      a.seq = c->ms_head_count;
      a.adam_c1 = a.adam_c2 = 0.f;
      if (c->cfg.optimizer == PT_OPT_ADAM) {
        const double n = (double)(t + 1);
        a.adam_c1 = (float)((double)c->lr / (1.0 - std::pow((double)c->cfg.beta1, n)));
        a.adam_c2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)c->cfg.beta2, n)));
      }
      if (learn) {
        // forward through the positions of a stage: the planes of the first layers were left by the previous tick's matrix
        // launch, those of the others are formed now, after the layer in front has published its output of this tick
        for (int pos = 0; pos < c->cmax; ++pos) {
          MsTick f = a;
          f.fhalf = a.cur ^ 1;                // (within a stage both halves name the same buffer)
          if (pos > 0) mat_fwd(c->ms_mf[pos].first, c->ms_mf[pos].second, f);
          vec(true, c->ms_vf[pos], c->ms_vf[pos].second, a);
        }
        // backward: every stage's last layer first, then the layers in front of it, each after the layer behind it has
        // left its input-error of this tick
        for (int back = 0; back < c->cmax; ++back) {
          if (back > 0) vec(true, c->ms_vb[back], c->ms_vb[back].second, a);
          mat_learn(c->ms_mb[back], a);
        }
      } else {
        for (int pos = 0; pos < c->cmax; ++pos) {
          if (c->ms_if[pos].second <= 0) continue;
          net.tiles_i = c->d_ms_tiles + c->ms_if[pos].first;
          hipLaunchKernelGGL(ms_infer_kernel, dim3(c->ms_if[pos].second), dim3(256), 0, c->stream, net, a);
          ++c->last_launches;
        }
      }
    }
    c->ms_zp_valid = learn;   // (an inference tick forms no planes for the tick after it)
    HIP_TRY(hipGetLastError());
  } else
  for (int base = 0; base < n_ticks; base += kLossSlots) {
    const int n = std::min(kLossSlots, n_ticks - base);
    if (c->persistent && n > 1) {
      // the whole block in one launch; ticks are separated by a grid barrier inside the kernel
      BlockArgs pa;
      pa.x = x_dev + (size_t)base * c->S * c->in_dim;
      pa.out = out_dev + (size_t)base * c->S * c->out_dim;
      pa.tgt = tgt ? tgt + (size_t)base * c->tgt_bytes : nullptr;
      // ticks [base, base+k) of the call are scored against targets that precede the block
      pa.hist = base == 0 ? c->d_hist[c->hist_cur] : (tgt ? tgt + (size_t)(base - c->k) * c->tgt_bytes : nullptr);
      pa.lossp = lossp;
      pa.loss = loss_dev ? loss_dev + base : nullptr;
      pa.dummy = dummy;
      pa.bar = c->d_bar;
      pa.err = c->d_err;
      pa.bar_base = c->bar_count;
      pa.head_base = c->head_count;
      pa.head_parts = learn ? (unsigned int)c->head_parts : 0u;
      c->head_count += pa.head_parts * (unsigned int)n;
      pa.t0 = c->tick + base;
      pa.spin_limit = c->spin_limit;
      pa.n_ticks = n;
      pa.fill = c->fill;
      pa.k = c->k;
      pa.serp = c->serpentine;
      pa.has_loss = learn && c->cfg.loss != PT_LOSS_NONE;
      pa.pl = pl;
      pa.tgt_bytes = (int)c->tgt_bytes;
      pa.in_stride = c->S * c->in_dim;
      pa.out_stride = c->S * c->out_dim;
      const unsigned g = (unsigned)std::min<size_t>(c->tiles.size(), (size_t)c->max_grid);
      void *kargs[2] = {&c->net, &pa};
      HIP_TRY(hipLaunchCooperativeKernel(learn ? c->k_plearn : c->k_pinfer, dim3(g), block, kargs,
                                         (unsigned)c->lds_bytes, c->stream));
      c->bar_count += (unsigned long long)(n - 1) * g;
      ++c->last_launches;
    } else
    for (int j = 0; j < n; ++j) {
      const int i = base + j;
      const int64_t t = c->tick + i;
      TickArgs a;
      a.x = x_dev + (size_t)i * c->S * c->in_dim;
      a.out = out_dev + (size_t)i * c->S * c->out_dim;
      a.cur = (int)(t & 1);
      a.rev = c->serpentine ? (int)(t & 1) : 0;
      a.tick = (int)(t % c->ring_period);
      if (learn) c->head_count += (unsigned int)c->head_parts;
      a.head_target = c->head_count;
      a.learn = learn && t >= c->fill && c->cfg.loss != PT_LOSS_NONE;
      a.tgt = nullptr;
      if (learn && c->cfg.loss != PT_LOSS_NONE)
        a.tgt = i >= c->k ? tgt + (size_t)(i - c->k) * c->tgt_bytes
                          : c->d_hist[c->hist_cur] + (size_t)i * c->tgt_bytes;
      a.lossp = lossp + (size_t)j * pl;
      a.loss1 = loss_dev ? loss_dev + i : dummy;
      a.adam_c1 = a.adam_c2 = 0.f;
      if (c->cfg.optimizer == PT_OPT_ADAM) {
        // every tick is one optimiser step of every stage, counted from the first tick after init or reset
        const double n = (double)(t + 1);
        a.adam_c1 = (float)((double)c->lr / (1.0 - std::pow((double)c->cfg.beta1, n)));
        a.adam_c2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)c->cfg.beta2, n)));
      }
      if (c->cmax == 1 && !learn && c->d_tiles_inf) {
        NetDev net = c->net;
        net.tiles = c->d_tiles_inf;
        net.n_tiles = c->n_tiles_inf;
        void *kargs[2] = {&net, &a};
        HIP_TRY(hipLaunchKernel(c->k_infer, dim3((unsigned)c->n_tiles_inf), block, kargs, c->lds_bytes, c->stream));
        ++c->last_launches;
      } else if (c->cmax == 1) {
        void *kargs[2] = {&c->net, &a};
        HIP_TRY(hipLaunchKernel(learn ? c->k_learn : c->k_infer, grid, block, kargs, c->lds_bytes, c->stream));
        ++c->last_launches;
      } else {
        // several layers per stage: forward-only phases, the fused phase, then the backward phases
        const int n_ph = learn ? 2 * c->cmax - 1 : c->cmax;
        for (int ph = 0; ph < n_ph; ++ph) {
          if (c->phase_cnt[ph] == 0) continue;
          NetDev net = c->net;
          net.tiles = c->d_tiles + c->phase_off[ph];
          net.n_tiles = c->phase_cnt[ph];
          void *kargs[2] = {&net, &a};
          HIP_TRY(hipLaunchKernel(learn && ph >= c->cmax - 1 ? c->k_learn : c->k_infer, dim3((unsigned)c->phase_cnt[ph]),
                                  block, kargs, c->lds_bytes, c->stream));
          ++c->last_launches;
        }
      }
    }
    if (learn && c->cfg.loss == PT_LOSS_MSE && loss_dev) {
      hipLaunchKernelGGL(loss_finalize_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, lossp, pl, n,
                         loss_dev + base);
      ++c->last_launches;
    }
    HIP_TRY(hipGetLastError());
  }
  if (learn && c->cfg.loss == PT_LOSS_NONE && loss_dev)
    hipLaunchKernelGGL(fill_kernel, dim3((n_ticks + 255) / 256), dim3(256), 0, c->stream, loss_dev, n_ticks, 0.f);
  // keep the last k targets for the ticks of the next call
  if (learn && c->k > 0 && c->cfg.loss != PT_LOSS_NONE) {
    const int k = c->k;
    unsigned char *oldh = c->d_hist[c->hist_cur], *newh = c->d_hist[c->hist_cur ^ 1];
    if (n_ticks >= k) {
      HIP_TRY(hipMemcpyAsync(newh, tgt + (size_t)(n_ticks - k) * c->tgt_bytes, (size_t)k * c->tgt_bytes,
                             hipMemcpyDeviceToDevice, c->stream));
    } else {
      HIP_TRY(hipMemcpyAsync(newh, oldh + (size_t)n_ticks * c->tgt_bytes, (size_t)(k - n_ticks) * c->tgt_bytes,
                             hipMemcpyDeviceToDevice, c->stream));
      HIP_TRY(hipMemcpyAsync(newh + (size_t)(k - n_ticks) * c->tgt_bytes, tgt, (size_t)n_ticks * c->tgt_bytes,
                             hipMemcpyDeviceToDevice, c->stream));
    }
    c->hist_cur ^= 1;
  }
  c->tick += n_ticks;
  return PT_OK;
}

int partime_step(partime_ctx *ctx, const float *x_dev, const void *target_dev, int n_ticks, float *out_dev,
                 float *loss_dev) {
  if (!ctx) return fail(PT_EINVAL, "partime_step: null context");
  if (n_ticks < 0) return fail(PT_EINVAL, "partime_step: n_ticks < 0");
  if (n_ticks == 0) return PT_OK;
  if (!x_dev || !out_dev) return fail(PT_EINVAL, "partime_step: null x_dev / out_dev");
  if (!target_dev && ctx->cfg.loss != PT_LOSS_NONE) return fail(PT_EINVAL, "partime_step: null target_dev");
  return run_ticks(ctx, x_dev, target_dev, n_ticks, out_dev, loss_dev, true);
}

int partime_infer(partime_ctx *ctx, const float *x_dev, int n_ticks, float *out_dev) {
  if (!ctx) return fail(PT_EINVAL, "partime_infer: null context");
  if (n_ticks < 0) return fail(PT_EINVAL, "partime_infer: n_ticks < 0");
  if (n_ticks == 0) return PT_OK;
  if (!x_dev || !out_dev) return fail(PT_EINVAL, "partime_infer: null x_dev / out_dev");
  return run_ticks(ctx, x_dev, nullptr, n_ticks, out_dev, nullptr, false);
}

int partime_step_noalloc(partime_ctx *ctx, const float *x_dev, const void *target_dev, int n_ticks, float *out_dev,
                         float *loss_dev) {
  if (!ctx) return fail(PT_EINVAL, "partime_step_noalloc: null context");
  if (n_ticks < 0) return fail(PT_EINVAL, "partime_step_noalloc: n_ticks < 0");
  if (n_ticks == 0) return PT_OK;
  if (!x_dev || !out_dev) return fail(PT_EINVAL, "partime_step_noalloc: null x_dev / out_dev");
  if (!target_dev && ctx->cfg.loss != PT_LOSS_NONE) return fail(PT_EINVAL, "partime_step_noalloc: null target_dev");
  if (ctx->cv || ctx->rb || ctx->ms || ctx->persistent)
    return fail(PT_EUNSUPPORTED, "partime_step_noalloc: built for dense pipelines of one stream, one launch per tick");
  const int pl = ctx->stages.back().n_parts;
  if (pl > kScratchParts)
    return fail(PT_EUNSUPPORTED, "partime_step_noalloc: the last stage has %d tiles, the static scratch holds %d", pl, kScratchParts);
  float *scr = nullptr;
  if (int rc = scratch_for(ctx->device, &scr)) return rc;
  return run_ticks(ctx, x_dev, target_dev, n_ticks, out_dev, loss_dev, true, scr, scr + (size_t)kLossSlots * kScratchParts);
}

// wait for the stream and report an error a kernel raised on the device (a grid barrier that ran out)
static int sync_and_check(partime_ctx *ctx) {
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  int flag = 0;
  HIP_TRY(hipMemcpy(&flag, ctx->d_err, sizeof(int), hipMemcpyDeviceToHost));
  if (flag) return fail(PT_EHIP, "a bounded wait inside a kernel ran out (grid barrier of the persistent kernel, the tiles of a softmax head waiting for each other, or the loss-head flag of the multi-stream matrix launch); results after that tick are invalid");
  return PT_OK;
}

int partime_sync(partime_ctx *ctx) {
  if (!ctx) return fail(PT_EINVAL, "partime_sync: null context");
  return sync_and_check(ctx);
}

int partime_get_state(partime_ctx *ctx, int layer, float *w_host, float *b_host) {
  if (!ctx) return fail(PT_EINVAL, "partime_get_state: null context");
  if (layer < 0 || layer >= (int)ctx->layers.size()) return fail(PT_EINVAL, "partime_get_state: layer %d out of range", layer);
  if (int rc = sync_and_check(ctx)) return rc;
  if (ctx->cv) {
    const int n_conv = (int)ctx->cvs.size();
    if (layer < n_conv) {
      CvStageHost &v = ctx->cvs[layer];
      if (w_host) HIP_TRY(hipMemcpy(w_host, v.Wg, (size_t)v.c_out * v.c_in * 9 * 4, hipMemcpyDeviceToHost));
      if (b_host) HIP_TRY(hipMemcpy(b_host, v.b, (size_t)v.c_out * 4, hipMemcpyDeviceToHost));
    } else {
      const pt_layer &l = ctx->layers[layer];
      if (w_host) HIP_TRY(hipMemcpy(w_host, ctx->hd_W, (size_t)l.out_dim * l.c_in * 4, hipMemcpyDeviceToHost));
      if (b_host) HIP_TRY(hipMemcpy(b_host, ctx->hd_b, (size_t)l.out_dim * 4, hipMemcpyDeviceToHost));
    }
    return PT_OK;
  }
  StageHost &s = ctx->stages[layer];
  if (w_host) {
    if (ctx->cfg.w_dtype == PT_F32) {
      HIP_TRY(hipMemcpy2D(w_host, (size_t)s.in_dim * 4, s.W, (size_t)s.ld * 4, (size_t)s.in_dim * 4, s.out_dim,
                          hipMemcpyDeviceToHost));
    } else if (ctx->ms) {
      std::vector<unsigned short> tiled((size_t)s.out_pad * s.in_pad);
      HIP_TRY(hipMemcpy(tiled.data(), s.W, tiled.size() * 2, hipMemcpyDeviceToHost));
      for (int r = 0; r < s.out_dim; ++r)
        for (int q = 0; q < s.in_dim; ++q) w_host[(size_t)r * s.in_dim + q] = host_bf16_widen(tiled[ms_woff(r, q, s.out_pad)]);
    } else {
      std::vector<unsigned short> tmp((size_t)s.out_dim * s.ld);
      HIP_TRY(hipMemcpy(tmp.data(), s.W, tmp.size() * 2, hipMemcpyDeviceToHost));
      for (int r = 0; r < s.out_dim; ++r)
        for (int q = 0; q < s.in_dim; ++q) w_host[(size_t)r * s.in_dim + q] = host_bf16_widen(tmp[(size_t)r * s.ld + q]);
    }
  }
  if (b_host) HIP_TRY(hipMemcpy(b_host, s.b, (size_t)s.out_dim * 4, hipMemcpyDeviceToHost));
  return PT_OK;
}

int partime_set_state(partime_ctx *ctx, int layer, const float *w_host, const float *b_host) {
  if (!ctx) return fail(PT_EINVAL, "partime_set_state: null context");
  if (layer < 0 || layer >= (int)ctx->layers.size()) return fail(PT_EINVAL, "partime_set_state: layer %d out of range", layer);
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  ctx->ms_zp_valid = false;   // (32 streams: the pre-activation planes formed ahead of the coming tick are stale now)
  if (ctx->cv) return cv_upload(ctx, layer, w_host, b_host);
  return upload_weights(ctx, layer, w_host, b_host);
}

static int buffer_args(partime_ctx *ctx, int which, int stage, int half, const void *host, const char *fn) {
  if (!ctx || !host) return fail(PT_EINVAL, "%s: null argument", fn);
  if (which == 2) return PT_OK;   // the target history: stage and half are not used
  if (which == 3 || which == 4) return PT_OK;   // delay lines of a skip connection: checked by ring_slot
  if (which < 0 || which > 4 || half < 0 || half > 1 || stage < 0 || stage >= ctx->depth)
    return fail(PT_EINVAL, "%s: which/stage/half out of range", fn);
  if (which == 0 && stage == ctx->depth - 1) return fail(PT_EINVAL, "%s: the last stage publishes no activation", fn);
  if (which == 1 && stage == 0) return fail(PT_EINVAL, "%s: the first stage publishes no error", fn);
  return PT_OK;
}

// Delay lines of the skip connection that ends in layer `layer` (which = 3: the skipped tensor, 4: the gradient that
// travels back): where the entry written `age` ticks before the coming tick's predecessor sits (age 0 = written during
// the last tick), how many streams and values per stream it has and how far apart the streams are in memory.
struct RingSlot {
  float *p;
  int S, n, pitch;
};
static int ring_slot(partime_ctx *ctx, int which, int layer, int age, const char *fn, RingSlot *out) {
  if (layer < 0 || layer >= (int)ctx->layers.size() || ctx->layers[layer].skip_from < 0)
    return fail(PT_EINVAL, "%s: layer %d is not the target of a skip connection", fn, layer);
  float *ring = nullptr;
  int d = 0;
  size_t slot = 0;
  if (ctx->cv) {
    CvStageHost &v = ctx->cvs[layer];
    ring = which == 3 ? v.skip_ring : v.serr_ring;
    d = v.skip_delay;
    slot = (size_t)v.co_pad * v.H * v.W;
    out->S = 1; out->n = v.c_out * v.H * v.W; out->pitch = out->n;   // the real channels come first
  } else {
    StageHost &s = ctx->stages[layer];
    ring = which == 3 ? s.skip_ring : s.serr_ring;
    d = s.skip_delay;
    const bool padded = ctx->ms || ctx->rb;
    out->S = ctx->S; out->n = s.out_dim; out->pitch = padded ? s.out_pad : s.out_dim;
    slot = (size_t)ctx->S * out->pitch;
  }
  if (age < 0 || age >= d)
    return fail(PT_EINVAL, "%s: the skip into layer %d crosses %d stage boundaries: ages 0 .. %d", fn, layer, d, d - 1);
  // slot of tick t = t mod (d + 1), as in the kernels (before tick 0 nothing was written: those slots hold their zeros)
  const int64_t n = d + 1, t = ctx->tick - 1 - age;
  out->p = ring + (size_t)(((t % n) + n) % n) * slot;
  return PT_OK;
}

int partime_get_buffer(partime_ctx *ctx, int which, int stage, int half, float *host) {
  int rc = buffer_args(ctx, which, stage, half, host, "partime_get_buffer");
  if (rc != PT_OK) return rc;
  if ((rc = sync_and_check(ctx)) != PT_OK) return rc;
  if (which == 3 || which == 4) {
    RingSlot r;
    if ((rc = ring_slot(ctx, which, stage, half, "partime_get_buffer", &r)) != PT_OK) return rc;
    HIP_TRY(hipMemcpy2D(host, (size_t)r.n * 4, r.p, (size_t)r.pitch * 4, (size_t)r.n * 4, r.S, hipMemcpyDeviceToHost));
    return PT_OK;
  }
  if (which == 2) {
    // the last target_delay targets, oldest first, as the 4-byte elements the caller supplied them in
    if (ctx->k > 0 && ctx->cfg.loss != PT_LOSS_NONE)
      HIP_TRY(hipMemcpy(host, ctx->d_hist[ctx->hist_cur], (size_t)ctx->k * ctx->tgt_bytes, hipMemcpyDeviceToHost));
    return PT_OK;
  }
  if (ctx->cv) {
    // a stage's activation is its last layer's, its error its first layer's; the last stage is the head
    const int HW = ctx->cvs[0].H * ctx->cvs[0].W, fl = ctx->first_node[stage];
    if (which == 0) {
      HIP_TRY(hipMemcpy(host, ctx->cvs[ctx->first_node[stage + 1] - 1].act_buf[half], (size_t)ctx->cvs[ctx->first_node[stage + 1] - 1].c_out * HW * 4, hipMemcpyDeviceToHost));
    } else if (stage < ctx->depth - 1) {
      HIP_TRY(hipMemcpy(host, ctx->cvs[fl].err_buf[half], (size_t)ctx->cvs[fl].c_in * HW * 4, hipMemcpyDeviceToHost));
    } else {
      // the head's error is one value per channel, the same at every pixel
      std::vector<float> ge(ctx->cvs.back().co_pad);
      HIP_TRY(hipMemcpy(ge.data(), ctx->hd_ge[half], ge.size() * 4, hipMemcpyDeviceToHost));
      for (int ch = 0; ch < ctx->cvs.back().c_out; ++ch)
        for (int p = 0; p < HW; ++p) host[(size_t)ch * HW + p] = ge[ch];
    }
    return PT_OK;
  }
  // dense single-stream path: a stage's activation is its last layer's, its error its first layer's
  StageHost &s = ctx->stages[which == 0 ? ctx->first_node[stage] + ctx->stages[ctx->first_node[stage]].cnt - 1
                                       : ctx->first_node[stage]];
  if (ctx->rb) {
    // activations live as bf16 [S][out_pad] (what the next stage's products read), errors as fp32 [S][in_pad]
    StageHost &r = s;   // activation: the stage's last layer; error: its first layer
    const int S = ctx->S;
    if (which == 0) {
      std::vector<unsigned short> tmp(r.act_elems);
      HIP_TRY(hipMemcpy(tmp.data(), r.xq[half], tmp.size() * 2, hipMemcpyDeviceToHost));
      for (int q = 0; q < S; ++q)
        for (int k = 0; k < r.out_dim; ++k) host[(size_t)q * r.out_dim + k] = host_bf16_widen(tmp[(size_t)q * r.out_pad + k]);
    } else {
      std::vector<float> tmp(r.err_elems);
      HIP_TRY(hipMemcpy(tmp.data(), r.err_buf[half], tmp.size() * 4, hipMemcpyDeviceToHost));
      for (int q = 0; q < S; ++q) std::memcpy(host + (size_t)q * r.in_dim, &tmp[(size_t)q * r.in_pad], (size_t)r.in_dim * 4);
    }
    return PT_OK;
  }
  if (ctx->ms) {
    // padded [S][pad] (activations) or [planes][S][pad] (errors, summed over the planes) -> [S][size]
    const int S = ctx->S;
    if (which == 0) {
      std::vector<float> tmp(s.act_elems);
      HIP_TRY(hipMemcpy(tmp.data(), s.act_buf[half], tmp.size() * 4, hipMemcpyDeviceToHost));
      for (int q = 0; q < S; ++q) std::memcpy(host + (size_t)q * s.out_dim, &tmp[(size_t)q * s.out_pad], (size_t)s.out_dim * 4);
    } else {
      std::vector<float> tmp(s.err_elems);
      HIP_TRY(hipMemcpy(tmp.data(), s.err_buf[half], tmp.size() * 4, hipMemcpyDeviceToHost));
      for (int q = 0; q < S; ++q)
        for (int k = 0; k < s.in_dim; ++k) {
          float t = 0.f;
          for (int p = 0; p < s.n_rt; ++p) t += tmp[(size_t)p * S * s.in_pad + ms_poff(q, k)];
          host[(size_t)q * s.in_dim + k] = t;
        }
    }
    return PT_OK;
  }
  if (which == 0) {
    HIP_TRY(hipMemcpy(host, s.act_buf[half], (size_t)s.out_dim * 4, hipMemcpyDeviceToHost));
  } else {
    std::vector<float> tmp((size_t)s.n_parts * s.ld);
    HIP_TRY(hipMemcpy(tmp.data(), s.err_buf[half], tmp.size() * 4, hipMemcpyDeviceToHost));
    for (int q = 0; q < s.in_dim; ++q) {
      float t = 0.f;
      for (int p = 0; p < s.n_parts; ++p) t += tmp[(size_t)p * s.ld + q];
      host[q] = t;
    }
  }
  return PT_OK;
}

int partime_set_buffer(partime_ctx *ctx, int which, int stage, int half, const float *host) {
  int rc = buffer_args(ctx, which, stage, half, host, "partime_set_buffer");
  if (rc != PT_OK) return rc;
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  ctx->ms_zp_valid = false;
  if (which == 3 || which == 4) {
    RingSlot r;
    if ((rc = ring_slot(ctx, which, stage, half, "partime_set_buffer", &r)) != PT_OK) return rc;
    HIP_TRY(hipMemcpy2D(r.p, (size_t)r.pitch * 4, host, (size_t)r.n * 4, (size_t)r.n * 4, r.S, hipMemcpyHostToDevice));
    return PT_OK;
  }
  if (which == 2) {
    if (ctx->k > 0 && ctx->cfg.loss != PT_LOSS_NONE)
      HIP_TRY(hipMemcpy(ctx->d_hist[ctx->hist_cur], host, (size_t)ctx->k * ctx->tgt_bytes, hipMemcpyHostToDevice));
    return PT_OK;
  }
  if (ctx->cv) {
    const int HW = ctx->cvs[0].H * ctx->cvs[0].W, fl = ctx->first_node[stage];
    if (which == 0) {
      HIP_TRY(hipMemcpy(ctx->cvs[ctx->first_node[stage + 1] - 1].act_buf[half], host, (size_t)ctx->cvs[ctx->first_node[stage + 1] - 1].c_out * HW * 4, hipMemcpyHostToDevice));
    } else if (stage < ctx->depth - 1) {
      HIP_TRY(hipMemcpy(ctx->cvs[fl].err_buf[half], host, (size_t)ctx->cvs[fl].c_in * HW * 4, hipMemcpyHostToDevice));
    } else {
      std::vector<float> ge(ctx->cvs.back().co_pad, 0.f);   // the head's error is constant over the pixels of a channel: keep pixel 0
      for (int ch = 0; ch < ctx->cvs.back().c_out; ++ch) ge[ch] = host[(size_t)ch * HW];
      HIP_TRY(hipMemcpy(ctx->hd_ge[half], ge.data(), ge.size() * 4, hipMemcpyHostToDevice));
    }
    return PT_OK;
  }
  StageHost &s = ctx->stages[which == 0 ? ctx->first_node[stage] + ctx->stages[ctx->first_node[stage]].cnt - 1
                                       : ctx->first_node[stage]];
  if (ctx->rb) {
    StageHost &r = s;   // activation: the stage's last layer; error: its first layer
    const int S = ctx->S;
    if (which == 0) {
      // rounded to bf16, in both orientations
      std::vector<unsigned short> q16(r.act_elems, 0), t16(r.act_elems, 0);
      for (int q = 0; q < S; ++q)
        for (int k = 0; k < r.out_dim; ++k) {
          const unsigned short v = host_bf16_rne(host[(size_t)q * r.out_dim + k]);
          q16[(size_t)q * r.out_pad + k] = v;
          t16[(size_t)k * S + q] = v;
        }
      HIP_TRY(hipMemcpy(r.xq[half], q16.data(), q16.size() * 2, hipMemcpyHostToDevice));
      HIP_TRY(hipMemcpy(r.xT[half], t16.data(), t16.size() * 2, hipMemcpyHostToDevice));
    } else {
      std::vector<float> tmp(r.err_elems, 0.f);
      for (int q = 0; q < S; ++q) std::memcpy(&tmp[(size_t)q * r.in_pad], host + (size_t)q * r.in_dim, (size_t)r.in_dim * 4);
      HIP_TRY(hipMemcpy(r.err_buf[half], tmp.data(), tmp.size() * 4, hipMemcpyHostToDevice));
    }
    return PT_OK;
  }
  if (ctx->ms) {
    const int S = ctx->S;
    if (which == 0) {
      std::vector<float> tmp(s.act_elems, 0.f);
      for (int q = 0; q < S; ++q) std::memcpy(&tmp[(size_t)q * s.out_pad], host + (size_t)q * s.out_dim, (size_t)s.out_dim * 4);
      HIP_TRY(hipMemcpy(s.act_buf[half], tmp.data(), tmp.size() * 4, hipMemcpyHostToDevice));
      // the bf16 copies the next stage's products read
      std::vector<unsigned short> q16(s.act_elems, 0), t16(s.act_elems, 0);
      for (int q = 0; q < S; ++q)
        for (int r = 0; r < s.out_dim; ++r) {
          const unsigned short v = host_bf16_rne(tmp[(size_t)q * s.out_pad + r]);
          q16[(size_t)q * s.out_pad + r] = v;
          t16[(size_t)r * S + q] = v;
        }
      HIP_TRY(hipMemcpy(s.xq[half], q16.data(), q16.size() * 2, hipMemcpyHostToDevice));
      HIP_TRY(hipMemcpy(s.xT[half], t16.data(), t16.size() * 2, hipMemcpyHostToDevice));
    } else {
      std::vector<float> tmp(s.err_elems, 0.f);   // plane 0 carries the values, the other planes are zero
      for (int q = 0; q < S; ++q)
        for (int k = 0; k < s.in_dim; ++k) tmp[ms_poff(q, k)] = host[(size_t)q * s.in_dim + k];
      HIP_TRY(hipMemcpy(s.err_buf[half], tmp.data(), tmp.size() * 4, hipMemcpyHostToDevice));
    }
    return PT_OK;
  }
  if (which == 0) {
    HIP_TRY(hipMemcpy(s.act_buf[half], host, (size_t)s.out_dim * 4, hipMemcpyHostToDevice));
  } else {
    std::vector<float> tmp((size_t)s.n_parts * s.ld, 0.f);
    std::memcpy(tmp.data(), host, (size_t)s.in_dim * 4);
    HIP_TRY(hipMemcpy(s.err_buf[half], tmp.data(), tmp.size() * 4, hipMemcpyHostToDevice));
  }
  return PT_OK;
}

int partime_get_tick(partime_ctx *ctx, int64_t *tick) {
  if (!ctx || !tick) return fail(PT_EINVAL, "partime_get_tick: null argument");
  *tick = ctx->tick;
  return PT_OK;
}

int partime_set_tick(partime_ctx *ctx, int64_t tick) {
  if (!ctx || tick < 0) return fail(PT_EINVAL, "partime_set_tick: bad argument");
  if (ctx->d_ms_head_ctr) {
    // the head-tile counter starts over together with the count the host keeps of it
    HIP_TRY(hipStreamSynchronize(ctx->stream));
    HIP_TRY(hipMemset(ctx->d_ms_head_ctr, 0, sizeof(unsigned int)));
    ctx->ms_head_count = 0;
  }
  ctx->tick = tick;
  ctx->ms_zp_valid = false;   // which half of the published activations feeds the coming tick depends on its parity
  return PT_OK;
}

int partime_set_lr(partime_ctx *ctx, float lr) {
  if (!ctx) return fail(PT_EINVAL, "partime_set_lr: null context");
  ctx->lr = lr;
  ctx->net.lr = lr;
  ctx->msnet.lr_over_s = lr / (float)ctx->S;
  ctx->rbnet.lr = lr;
  ctx->cvnet.lr = lr;
  return PT_OK;
}

int partime_reset(partime_ctx *ctx) {
  if (!ctx) return fail(PT_EINVAL, "partime_reset: null context");
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  if (ctx->d_ms_head_ctr) {
    HIP_TRY(hipMemset(ctx->d_ms_head_ctr, 0, sizeof(unsigned int)));
    ctx->ms_head_count = 0;
  }
  if (ctx->d_head_ctr) {
    HIP_TRY(hipMemset(ctx->d_head_ctr, 0, sizeof(unsigned int)));
    ctx->head_count = 0;
  }
  for (auto &v : ctx->cvs)
    for (int p = 0; p < 2; ++p) {
      if (v.act_buf[p]) HIP_TRY(hipMemset(v.act_buf[p], 0, (size_t)v.co_pad * v.H * v.W * 4));
      if (v.err_buf[p]) HIP_TRY(hipMemset(v.err_buf[p], 0, (size_t)v.ci_pad * v.H * v.W * 4));
    }
  for (auto &v : ctx->cvs)
    if (v.skip_ring) {
      HIP_TRY(hipMemset(v.skip_ring, 0, v.ring_bytes));
      HIP_TRY(hipMemset(v.serr_ring, 0, v.ring_bytes));
    }
  if (ctx->cv)
    for (int p = 0; p < 2; ++p) HIP_TRY(hipMemset(ctx->hd_ge[p], 0, (size_t)ctx->cvs.back().co_pad * 4));
  for (auto &s : ctx->stages)
    for (int p = 0; p < 2; ++p) {
      if (s.act_buf[p]) HIP_TRY(hipMemset(s.act_buf[p], 0, ((ctx->ms || ctx->rb) ? s.act_elems : (size_t)s.out_dim) * 4));
      if (s.err_buf[p]) HIP_TRY(hipMemset(s.err_buf[p], 0, ((ctx->ms || ctx->rb) ? s.err_elems : (size_t)s.n_parts * s.ld) * 4));
      if (s.xq[p]) HIP_TRY(hipMemset(s.xq[p], 0, s.act_elems * 2));
      if (s.xT[p]) HIP_TRY(hipMemset(s.xT[p], 0, s.act_elems * 2));
    }
  for (auto &v : ctx->cvs)
    if (v.mW) {
      HIP_TRY(hipMemset(v.mW, 0, (size_t)v.co_pad * v.c_in * 9 * 4));
      HIP_TRY(hipMemset(v.vW, 0, (size_t)v.co_pad * v.c_in * 9 * 4));
      HIP_TRY(hipMemset(v.mb, 0, (size_t)v.co_pad * 4));
      HIP_TRY(hipMemset(v.vb, 0, (size_t)v.co_pad * 4));
    }
  if (ctx->hd_mW) {
    const pt_layer &hl = ctx->layers.back();
    HIP_TRY(hipMemset(ctx->hd_mW, 0, (size_t)hl.out_dim * hl.c_in * 4));
    HIP_TRY(hipMemset(ctx->hd_vW, 0, (size_t)hl.out_dim * hl.c_in * 4));
    HIP_TRY(hipMemset(ctx->hd_mb, 0, (size_t)hl.out_dim * 4));
    HIP_TRY(hipMemset(ctx->hd_vb, 0, (size_t)hl.out_dim * 4));
  }
  for (auto &s : ctx->stages) {
    if (s.mW) {
      const size_t nw = ctx->ms ? (size_t)s.out_pad * s.in_pad : (size_t)s.out_dim * s.ld;
      HIP_TRY(hipMemset(s.mW, 0, nw * 4));
      HIP_TRY(hipMemset(s.vW, 0, nw * 4));
      HIP_TRY(hipMemset(s.mb, 0, (size_t)s.out_dim * 4));
      HIP_TRY(hipMemset(s.vb, 0, (size_t)s.out_dim * 4));
    }
    if (s.skip_ring) {
      HIP_TRY(hipMemset(s.skip_ring, 0, s.ring_bytes));
      HIP_TRY(hipMemset(s.serr_ring, 0, s.ring_bytes));
    }
    if (s.out_single) HIP_TRY(hipMemset(s.out_single, 0, (size_t)s.out_dim * 4));
    if (s.e_single) HIP_TRY(hipMemset(s.e_single, 0, (size_t)s.n_parts * s.ld * 4));
  }
  for (int p = 0; p < 2; ++p)
    HIP_TRY(hipMemset(ctx->d_hist[p], 0, std::max<size_t>(1, (size_t)ctx->k) * ctx->tgt_bytes));
  ctx->tick = 0;
  ctx->ms_zp_valid = false;
  return PT_OK;
}

int partime_last_launch_count(partime_ctx *ctx) { return ctx ? ctx->last_launches : 0; }

static int opt_state_args(partime_ctx *ctx, int layer, const char *fn) {
  if (!ctx) return fail(PT_EINVAL, "%s: null context", fn);
  if (ctx->cfg.optimizer != PT_OPT_ADAM) return fail(PT_EINVAL, "%s: the pipeline has no optimiser state (plain SGD)", fn);
  if (layer < 0 || layer >= (int)ctx->layers.size()) return fail(PT_EINVAL, "%s: layer %d out of range", fn, layer);
  return PT_OK;
}

// conv pipelines: where the moments of a layer live and how many there are (weights in the caller's order, biases)
static void cv_moments(partime_ctx *ctx, int layer, float *dev[4], size_t &nw, size_t &nb) {
  const int n_conv = (int)ctx->cvs.size();
  if (layer < n_conv) {
    CvStageHost &v = ctx->cvs[layer];
    dev[0] = v.mW; dev[1] = v.vW; dev[2] = v.mb; dev[3] = v.vb;
    nw = (size_t)v.c_out * v.c_in * 9; nb = (size_t)v.c_out;   // the real output channels come first in both arrays
  } else {
    const pt_layer &l = ctx->layers[layer];
    dev[0] = ctx->hd_mW; dev[1] = ctx->hd_vW; dev[2] = ctx->hd_mb; dev[3] = ctx->hd_vb;
    nw = (size_t)l.out_dim * l.c_in; nb = (size_t)l.out_dim;
  }
}

int partime_get_opt_state(partime_ctx *ctx, int layer, float *m_w_host, float *v_w_host, float *m_b_host, float *v_b_host) {
  int rc = opt_state_args(ctx, layer, "partime_get_opt_state");
  if (rc != PT_OK) return rc;
  if ((rc = sync_and_check(ctx)) != PT_OK) return rc;
  if (ctx->cv) {
    float *dev[4], *host[4] = {m_w_host, v_w_host, m_b_host, v_b_host};
    size_t nw, nb;
    cv_moments(ctx, layer, dev, nw, nb);
    for (int q = 0; q < 4; ++q)
      if (host[q]) HIP_TRY(hipMemcpy(host[q], dev[q], (q < 2 ? nw : nb) * 4, hipMemcpyDeviceToHost));
    return PT_OK;
  }
  StageHost &s = ctx->stages[layer];
  const float *src[2] = {s.mW, s.vW};
  float *dst[2] = {m_w_host, v_w_host};
  for (int q = 0; q < 2; ++q) {
    if (!dst[q]) continue;
    if (ctx->ms) {   // the moments are stored like the weights
      std::vector<float> tiled((size_t)s.out_pad * s.in_pad);
      HIP_TRY(hipMemcpy(tiled.data(), src[q], tiled.size() * 4, hipMemcpyDeviceToHost));
      for (int r = 0; r < s.out_dim; ++r)
        for (int k = 0; k < s.in_dim; ++k) dst[q][(size_t)r * s.in_dim + k] = tiled[ms_woff(r, k, s.out_pad)];
      continue;
    }
    HIP_TRY(hipMemcpy2D(dst[q], (size_t)s.in_dim * 4, src[q], (size_t)s.ld * 4, (size_t)s.in_dim * 4, s.out_dim,
                        hipMemcpyDeviceToHost));
  }
  if (m_b_host) HIP_TRY(hipMemcpy(m_b_host, s.mb, (size_t)s.out_dim * 4, hipMemcpyDeviceToHost));
  if (v_b_host) HIP_TRY(hipMemcpy(v_b_host, s.vb, (size_t)s.out_dim * 4, hipMemcpyDeviceToHost));
  return PT_OK;
}

int partime_set_opt_state(partime_ctx *ctx, int layer, const float *m_w_host, const float *v_w_host,
                          const float *m_b_host, const float *v_b_host) {
  int rc = opt_state_args(ctx, layer, "partime_set_opt_state");
  if (rc != PT_OK) return rc;
  HIP_TRY(hipStreamSynchronize(ctx->stream));
  if (ctx->cv) {
    float *dev[4];
    const float *host[4] = {m_w_host, v_w_host, m_b_host, v_b_host};
    size_t nw, nb;
    cv_moments(ctx, layer, dev, nw, nb);
    for (int q = 0; q < 4; ++q)
      if (host[q]) HIP_TRY(hipMemcpy(dev[q], host[q], (q < 2 ? nw : nb) * 4, hipMemcpyHostToDevice));
    return PT_OK;
  }
  StageHost &s = ctx->stages[layer];
  float *dst[2] = {s.mW, s.vW};
  const float *src[2] = {m_w_host, v_w_host};
  for (int q = 0; q < 2; ++q) {
    if (!src[q]) continue;
    if (ctx->ms) {
      std::vector<float> tiled((size_t)s.out_pad * s.in_pad, 0.f);
      for (int r = 0; r < s.out_dim; ++r)
        for (int k = 0; k < s.in_dim; ++k) tiled[ms_woff(r, k, s.out_pad)] = src[q][(size_t)r * s.in_dim + k];
      HIP_TRY(hipMemcpy(dst[q], tiled.data(), tiled.size() * 4, hipMemcpyHostToDevice));
      continue;
    }
    HIP_TRY(hipMemcpy2D(dst[q], (size_t)s.ld * 4, src[q], (size_t)s.in_dim * 4, (size_t)s.in_dim * 4, s.out_dim,
                        hipMemcpyHostToDevice));
  }
  if (m_b_host) HIP_TRY(hipMemcpy(s.mb, m_b_host, (size_t)s.out_dim * 4, hipMemcpyHostToDevice));
  if (v_b_host) HIP_TRY(hipMemcpy(s.vb, v_b_host, (size_t)s.out_dim * 4, hipMemcpyHostToDevice));
  return PT_OK;
}

int partime_bandwidth_probe(size_t bytes, int mode, int iters, double *gbps_out) {
  if (!gbps_out || iters <= 0 || mode < 0 || mode > 2) return fail(PT_EINVAL, "bandwidth probe: bad argument");
  if (bytes < (1u << 20) || bytes > ((size_t)64 << 30)) return fail(PT_EINVAL, "bandwidth probe: 1 MiB <= bytes <= 64 GiB");
  size_t n4 = bytes / 16;
  float4 *buf = nullptr;
  float *sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = PT_OK;
  float ms = 0.f;
  double best = 0.0;
  const int grids[3] = {256, 512, 2048};  // one work-group per compute unit is usually the fastest
  auto launch = [&](int grid) {
    if (mode == 0) hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, 0, buf, n4, sink);
    else if (mode == 1) hipLaunchKernelGGL(probe_write_kernel, dim3(grid), dim3(256), 0, 0, buf, n4, 1.f);
    else hipLaunchKernelGGL(probe_update_kernel, dim3(grid), dim3(256), 0, 0, buf, n4, 0.999f);
  };
#define PROBE_TRY(expr)                                                                  \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) { rc = fail(PT_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); goto done; } \
  } while (0)
  PROBE_TRY(hipMalloc((void **)&buf, n4 * 16));
  PROBE_TRY(hipMalloc((void **)&sink, 4));
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  hipLaunchKernelGGL(probe_write_kernel, dim3(2048), dim3(256), 0, 0, buf, n4, 1.f);
  for (int g = 0; g < 3; ++g) {
    for (int i = 0; i < 3; ++i) launch(grids[g]);
    PROBE_TRY(hipDeviceSynchronize());
    PROBE_TRY(hipEventRecord(e0, 0));
    for (int i = 0; i < iters; ++i) launch(grids[g]);
    PROBE_TRY(hipEventRecord(e1, 0));
    PROBE_TRY(hipEventSynchronize(e1));
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
    best = std::max(best, (double)(n4 * 16) * (mode == 2 ? 2.0 : 1.0) * iters / (ms * 1e-3) / 1e9);
  }
  *gbps_out = best;
done:
#undef PROBE_TRY
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (sink) (void)hipFree(sink);
  if (buf) (void)hipFree(buf);
  return rc;
}

}  // extern "C"
