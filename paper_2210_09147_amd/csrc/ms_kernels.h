// Multi-stream (S = 32) stages: every stage product is a dense contraction with the S streams as its
// narrow dimension, computed on the matrix cores (v_mfma_f32_16x16x32_bf16, gfx950) from bf16 weights.
// Included by partime.hip only.
//
// The weights are the traffic (arithmetic intensity 48 flop per byte), so a learning tick reads every weight once and
// writes it once.  A stage's delta needs the stage's complete pre-activations, which would force a second pass; the
// pass is therefore folded across the tick boundary: the launch that updates the weights of tick t also forms, from
// the updated tile it still holds in registers, the tile's share of the NEXT tick's pre-activations.
//
// One learning tick = two launches over all stages:
//   ms_vec_kernel   (vectors only)  z(t) = b + sum of the partial planes the previous matrix launch left (Eq. 6),
//                   o = phi(z), published in fp32 and as bf16 in both orientations; g = the error the next stage
//                   published one tick earlier (sum of its planes, Eq. 11), delta = rnd(g * phi'(z)) (Eq. 9) in both
//                   orientations, bias update; the last stage's softmax statistics per 64 rows; rnd(x(t)) transposed and
//                   rnd(x(t+1)) for the first stage
//   ms_mat_kernel   tile = a block of rows x 512 columns of one stage's W, one pass: E = W^T delta with the old W
//                   (error plane of this row tile), W <- rnd(W - eta/S * delta rnd(x)^T)  (Algorithm 1, last two
//                   steps), then Z(t+1) partial = W_new * rnd(x(t+1)) over the tile's columns (plane of this column
//                   tile).  Its first work-groups are the loss head of the last stage, 64 rows each (softmax / squared
//                   error, delta, bias); the tiles of the last stage, which come last in the launch, start once all
//                   of them have counted themselves in.
// x(t+1) of a stage is what the stage in front of it has just published, and for the first stage the caller's next
// sample; at the last tick of a call that sample is not known yet, so the first stage's planes are formed by a
// forward-only launch of the same kernel over that stage when the next call begins.  The same forward-only mode
// forms every stage's planes for the first learning tick after inference ticks or after the state was changed from
// outside.  An inference tick writes no weights, so nothing is gained by folding: it is one launch of ms_infer_kernel.
// rnd() is round-to-nearest-even to bf16: what enters a matrix-core product is bf16, sums are fp32.
//
// Several layers per stage (Eq. 3-5: exact back-propagation inside a stage).  Layer j + 1 of a stage needs layer j's output
// of this tick and layer j's delta needs layer j + 1's input-error of this tick, so a tick becomes a sequence of launches
// by position in the stage, each over all stages: vector launch of the first layers (their planes come from the previous
// tick's matrix launch: the fold works for them alone), then for every further position a forward-only matrix launch and
// a vector launch; the matrix launch of every stage's last layer (with the loss head); then, going back through the
// positions, a vector launch that forms delta from the pre-activations kept earlier and the error planes the layer
// behind has just written, and that layer's matrix launch.  Links inside a stage are single buffers of the same tick
// (both halves of a record's ping-pong pair name the same memory), stage boundaries keep their pairs.
//
// Matrix-core operand layout used throughout (16x16x32, D = A * B + C, wave of 64 lanes, lane l, g = l / 16):
//   A (16 x 32): lane holds A[l % 16][8 g .. 8 g + 7]          (8 bf16 = 16 bytes)
//   B (32 x 16): lane holds B[8 g .. 8 g + 7][l % 16]
//   C (16 x 16): lane holds C[4 g .. 4 g + 3][l % 16]          (4 fp32)
// The contraction index may be permuted freely as long as A and B use the same permutation, and the rows
// of A (columns of B) may be any rows we like: both freedoms are used below so that registers loaded
// with 16 contiguous bytes of a weight row serve as A operand, and line up element by element with the
// C-layout result of the update product.

#pragma once

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kMsS = 32;          // streams (fixed by the kernels' register layouts)
constexpr int kMsTR = 512;        // rows per matrix tile, unless taller tiles make the launch one round of work-groups
constexpr int kMsNWM = 4;         // waves of a matrix work-group: one per SIMD
constexpr int kMsSB = 4;          // groups of 32 columns a wave takes: 128 columns, its share of E is 64 registers
constexpr int kMsRing = 2;        // register sets of a matrix tile: blocks of 32 rows in flight or being worked on (tile heights are multiples of 32 * kMsRing)
constexpr int kMsTC = 32 * kMsSB * kMsNWM;   // columns per matrix tile (stage sizes are padded to whole column tiles)
constexpr int kMsVR = 64;         // rows per tile of the vector kernel
constexpr int kMsRW = 16;         // inference kernel: rows per wave
constexpr int kMsRowsF = 4 * kMsRW;   // rows per inference tile (4 waves)
constexpr int kMsKC = 512;        // columns of X staged in LDS at a time by the inference kernel
constexpr int kMsXPitch = kMsKC + 8;

// Storage order of W (and of the Adam moments, which are shaped like it).  A matrix tile streams its rows block by block
// and a wave asks for 16 bytes per lane and request, so the weights are kept in the order the requests want them:
//   [column tile of 512][block of 32 rows][wave: 128 columns][group of 32 columns][16-row half][lane = 16 * (column / 8 % 4) + row % 16][8]
// One request of a wave is 1 KiB of consecutive memory, a block of 32 rows x 512 columns is 32 KiB, and a tile walks one
// consecutive region from its first row to its last.  (With plain row-major storage a tile reads 1 KiB pieces 8 KiB
// apart; measured with a no-arithmetic kernel, that streams at 4.7 TB/s against 6.9 TB/s as soon as the tiles of a launch
// do not march in step.)  The caller's row-major order is restored at the boundary.
constexpr int kMsBlk = 32 * kMsTC;   // elements of one block of 32 rows x 512 columns
__host__ __device__ inline size_t ms_woff(int row, int col, int out_pad) {
  const size_t blk = (size_t)(col / kMsTC) * (out_pad >> 5) + (row >> 5);
  const int c = col % kMsTC;
  return blk * kMsBlk + (c >> 5) * 1024 + ((row >> 4) & 1) * 512 + ((c >> 3) & 3) * 128 + (row & 15) * 8 + (c & 7);
}

struct MsStage {
  bf16_t *W;                 // out_pad x in_pad, in the order of ms_woff
  float *b;                  // [out_pad]
  float *mW, *vW, *mb, *vb;  // Adam moments, fp32, shaped like W and b (NULL under plain SGD)
  int in_dim, out_dim, in_pad, out_pad, act, is_last, is_first;
  int fold;                  // first layer of its stage: its matrix launch also forms the coming tick's pre-activations
  float *out_act[2];         // [S][out_pad] (NULL: last stage, output goes to the caller)
  float *zp;                 // [n_ct] planes of S x out_pad partial pre-activations of the coming tick (order: ms_poff), one per column tile
  int n_ct;
  float *zbuf;               // [S][out_pad] pre-activations of this tick: last layer (the loss head reads them) and layers
                             // that are not the last of their stage (their delta is formed later in the tick)
  bf16_t *dlt;               // delta as the matrix tiles' operand of E: [block of 32 rows][16 streams half h][lane][8], see ms_put_delta
  bf16_t *dltT;              // [out_pad][S]
  const bf16_t *xq_in[2];    // rnd(stage input) [S][in_pad], published by the previous stage (NULL: first stage)
  bf16_t *xq_out[2];         // rnd(stage output) [S][out_pad] for the next stage (NULL: last stage)
  const bf16_t *xT_in[2];    // rnd(stage input) transposed [in_pad][S]
  bf16_t *xT_out[2];         // rnd(stage output) transposed [out_pad][S] (NULL: last stage)
  bf16_t *xT0;               // first stage only: rnd(x(t)) transposed [in_pad][S]
  bf16_t *xq0;               // first stage only: rnd(x of the coming tick) [S][in_pad]
  const float *gin[2];       // error planes of the next stage: [n_gparts] planes of S x out_pad (order: ms_poff)
  int n_gparts;
  float *eout[2];            // this stage's error planes: [n_rt] planes of S x in_pad (NULL for the first stage)
  int n_rt, tr;              // row tiles of the matrix launch (= error planes) and their height
  // skip connections (Sec. V-C): a layer that adds the output of an earlier layer reads it with the delay of the stage
  // boundaries in between and hands the gradient at its own output back with the same delay.  Both wait in rings of
  // d + 1 slots of fp32 [S][out_pad], slot = tick mod (d + 1); the rings belong to the target.
  const float *skip_in;      // target: ring of the source's outputs
  float *serr_out;           // target: ring of gradients for the source
  int skip_n, skip_d;        // target: slots, delay
  float *skip_out;           // source: the ring it writes its output to ...
  const float *serr_in;      // ... and the ring it reads its extra gradient from
  int src_n, src_d;
};

// what one tick of one stage needs, with the ping-pong halves already chosen: plain scalars and pointers, so the
// whole thing lives in registers (a by-reference view of MsStage would be re-read from memory after every
// store, and a by-value copy with runtime-indexed arrays would live in scratch memory)
struct MsView {
  bf16_t *W;
  float *b;
  float *mW, *vW, *mb, *vb;
  int in_dim, out_dim, in_pad, out_pad, act, is_last, is_first, fold;
  float *out_cur;
  float *zp;
  int n_ct;
  float *zbuf;
  bf16_t *dlt, *dltT;
  const bf16_t *xq_fwd;      // operand of the forward product (the half the launch was told to use; first stage: xq0)
  bf16_t *xq_cur;
  const bf16_t *xT_prev;     // operand of the update product (first stage: xT0)
  bf16_t *xT_cur;
  bf16_t *xT0, *xq0;
  const float *gin_prev;
  int n_gparts;
  float *eout_cur;
  int n_rt, tr;
  const float *skip_in, *serr_in;   // ring slots of this tick, already chosen (NULL: no skip)
  float *skip_out, *serr_out;
};
__device__ __forceinline__ MsView ms_view(const MsStage *sp, int cur, int fhalf, int tick = 0) {
  MsView v;
  v.W = sp->W; v.b = sp->b;
  v.mW = sp->mW; v.vW = sp->vW; v.mb = sp->mb; v.vb = sp->vb;
  v.in_dim = sp->in_dim; v.out_dim = sp->out_dim; v.in_pad = sp->in_pad; v.out_pad = sp->out_pad;
  v.act = sp->act; v.is_last = sp->is_last; v.is_first = sp->is_first; v.fold = sp->fold;
  v.out_cur = cur ? sp->out_act[1] : sp->out_act[0];
  v.zp = sp->zp; v.n_ct = sp->n_ct;
  v.zbuf = sp->zbuf; v.dlt = sp->dlt; v.dltT = sp->dltT;
  v.xT0 = sp->xT0; v.xq0 = sp->xq0;
  v.xq_fwd = sp->is_first ? sp->xq0 : (fhalf ? sp->xq_in[1] : sp->xq_in[0]);
  v.xq_cur = cur ? sp->xq_out[1] : sp->xq_out[0];
  v.xT_prev = sp->is_first ? sp->xT0 : (cur ? sp->xT_in[0] : sp->xT_in[1]);
  v.xT_cur = cur ? sp->xT_out[1] : sp->xT_out[0];
  v.gin_prev = cur ? sp->gin[0] : sp->gin[1];
  v.n_gparts = sp->n_gparts;
  v.eout_cur = cur ? sp->eout[1] : sp->eout[0];
  v.n_rt = sp->n_rt; v.tr = sp->tr;
  const size_t slot = (size_t)kMsS * sp->out_pad;
  v.skip_in = sp->skip_in ? sp->skip_in + (size_t)((tick + sp->skip_n - sp->skip_d) % sp->skip_n) * slot : nullptr;
  v.serr_out = sp->serr_out ? sp->serr_out + (size_t)(tick % sp->skip_n) * slot : nullptr;
  v.skip_out = sp->skip_out ? sp->skip_out + (size_t)(tick % sp->src_n) * slot : nullptr;
  v.serr_in = sp->serr_in ? sp->serr_in + (size_t)((tick + sp->src_n - sp->src_d) % sp->src_n) * slot : nullptr;
  return v;
}

struct MsTile {
  int stage, a, b, kind;     // `stage` is the layer's record.  Vector kernel: rows [a, a + 64); kind 0: forward and delta, kind 3:
                             // forward only, the pre-activations are kept (a layer that is not the last of its stage), kind 4: delta
                             // from the kept pre-activations; kind 1: columns [a, a + 64) of the first layer's input.
                             // matrix kernel: kind 0: a = row tile, b = column tile; kind 2: loss head, rows [a, a + 64)
};

// What a work-group reads first: its tile and, in the same record, a copy of the layer's record.  With the layer records
// in an array of their own a work-group would read the tile, then the layer, then its data: three memory round trips
// in a row at the start of every launch, each of them cold.
struct MsTileRec {
  MsTile t;
  MsStage s;
};

struct MsNet {
  const MsTileRec *tiles_v, *tiles_m, *tiles_f;   // vector launch; matrix launch of a learning tick; forward-only matrix launch
  const MsTileRec *tiles_i;                       // inference launch (tile: a = first of 64 rows)
  int loss, out_dim, adam;
  float lr_over_s, inv_s, beta1, beta2, eps;
  unsigned int *head_flag;  // number of head tiles that have finished since the counter was last cleared
  float *hstat;             // last stage: [tiles of 64 rows][S][2] softmax statistics left by the vector launch
  float *hpart;             // last stage: the head tiles' shares of the squared error
  int *err;                 // raised when a bounded wait runs out
  long long spin_limit;
};

struct MsTick {
  const float *x;       // [S][in_dim] this tick's samples
  const float *x_next;  // the coming tick's samples, or NULL when the caller has not supplied them yet
  const void *tgt;      // [S] int32 or [S][out_dim] fp32
  float *out;           // [S][out_dim]
  float *loss1;
  int cur, learn;
  int tick;             // tick number modulo the common period of all skip rings: their slots
  int fhalf;            // which half of the published activations the forward product of this launch reads
  unsigned int seq;     // what head_flag reads once every head tile of this tick is done
  float adam_c1, adam_c2;   // lr / (1 - beta1^n), 1 / sqrt(1 - beta2^n)
};

__device__ __forceinline__ f32x4_t mfma16(uint4 a, uint4 b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                 0, 0, 0);
}
// two fp32 -> two bf16 (round to nearest even) in one 32-bit word: gfx950 converts a pair in one instruction
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned int pack_bf16(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float bf16_lo(unsigned int u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int u) { return __uint_as_float(u & 0xffff0000u); }

// one step of the update rule on one parameter; gsum = gradient summed over the streams.  Plain SGD, or Adam on the
// mean gradient with the moments passed by reference
__device__ __forceinline__ float ms_step(const MsNet &net, const MsTick &a, float w, float gsum, float &m, float &v) {
  if (!net.adam) return w - net.lr_over_s * gsum;
  const float g = gsum * net.inv_s;
  m = fmaf(net.beta1, m, (1.f - net.beta1) * g);
  v = fmaf(net.beta2, v, (1.f - net.beta2) * g * g);
  return w - a.adam_c1 * m / (sqrtf(v) * a.adam_c2 + net.eps);
}

// delta in the order the matrix tiles load it as operand of E = W^T delta: per block of 32 rows and half h of the streams one
// 16-byte piece per lane (g = lane / 16, li = lane % 16): rows 4 g .. 4 g + 3 and 16 + 4 g .. 16 + 4 g + 3 of the block at
// stream 16 h + li -- 1 KiB of consecutive memory per request of a wave.  (Kept as [S][out_pad] the same operand took
// four 8-byte requests per lane over 16 rows of memory 8 KiB apart.)  A vector thread holds rows r .. r + 7 of stream s,
// r a multiple of 8: two 8-byte pieces of neighbouring lanes.
__device__ __forceinline__ void ms_put_delta(bf16_t *dlt, int s, int r, const unsigned int (&pd)[4]) {
  const int rr = r & 31, g0 = (rr >> 2) & 3, hi = rr >> 4;
  bf16_t *p = dlt + ((size_t)((r >> 5) * 2 + (s >> 4)) * 64 + g0 * 16 + (s & 15)) * 8 + hi * 4;
  stg8(p, make_uint2(pd[0], pd[1]));
  stg8(p + 16 * 8, make_uint2(pd[2], pd[3]));   // rows r + 4 .. r + 7: the next g
}

// Partial-sum planes (pre-activations per column tile, errors per row tile) are [S][pad] values kept in the order the
// matrix tiles produce them: per 16 values of the padded axis and half h of the streams one 16-byte piece per lane of
// the matrix-core result layout (lane = 16 g + li holds values 4 g .. 4 g + 3 at stream 16 h + li), so a wave writes
// 1 KiB of consecutive memory (rows of [S][pad] would take 64-byte pieces 16 KiB apart).  Element (stream s, index i):
__host__ __device__ inline size_t ms_poff(int s, int i) {
  return ((size_t)((i >> 4) * 2 + (s >> 4)) * 64 + ((i >> 2) & 3) * 16 + (s & 15)) * 4 + (i & 3);
}
// acc[0..7] += the values i .. i + 7 (i a multiple of 8) of stream s in planes q = 0 .. n - 1, added in ascending order.
// The planes are requested CH at a time, at clamped addresses: one request per trip of a loop with a run-time bound would
// be one memory round trip after the other.
template <int CH>
__device__ __forceinline__ void ms_add_planes(const float *planes, int s, int i, int n, size_t plane, float (&acc)[8]) {
  const float *p0 = planes + ms_poff(s, i);   // values i .. i + 3; i + 4 .. i + 7 sit one g further: 64 floats on
  for (int q0 = 0; q0 < n; q0 += CH) {
    float4 u[CH][2];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const float *p = p0 + (size_t)min(q0 + i, n - 1) * plane;
      u[i][0] = ldg_f4(p);
      u[i][1] = ldg_f4(p + 64);
    }
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const bool on = q0 + i < n;
      acc[0] += on ? u[i][0].x : 0.f; acc[1] += on ? u[i][0].y : 0.f; acc[2] += on ? u[i][0].z : 0.f; acc[3] += on ? u[i][0].w : 0.f;
      acc[4] += on ? u[i][1].x : 0.f; acc[5] += on ? u[i][1].y : 0.f; acc[6] += on ? u[i][1].z : 0.f; acc[7] += on ? u[i][1].w : 0.f;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// vector kernel: everything of a tick that is a vector per stream.  Tile = 64 rows of one stage x the 32 streams;
// thread (stream s, group of 8 rows).  The transposed bf16 copies go through LDS so that every store is 16 bytes.
// ------------------------------------------------------------------------------------------------
template <bool LEARN>
__global__ __launch_bounds__(256) void ms_vec_kernel(MsNet net, MsTick a) {
  __shared__ __attribute__((aligned(16))) unsigned short tr[2][kMsVR * kMsS];   // bf16 [row][stream]: outputs, deltas
  const MsTileRec *rec = net.tiles_v + blockIdx.x;
  const MsTile tl = rec->t;
  const MsView st = ms_view(&rec->s, a.cur, a.cur, a.tick);
  const int tid = threadIdx.x, s = tid >> 3, rq = tid & 7;
  const int trow = tid >> 2, tq = tid & 3;           // transposed phase: row of the tile, group of 8 streams

  if (tl.kind == 1) {
    // first stage: the caller's fp32 samples rounded on the way in; columns [k0, k0 + 64) of the padded input.
    // rnd(x(t)) transposed feeds the update product, rnd(x(t+1)) the forward product of the coming tick.
    const int k = tl.a + 8 * rq;
    auto round8 = [&](const float *x, unsigned int (&p)[4]) {
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = ldg_f(x + (size_t)s * st.in_dim + min(k + j, st.in_dim - 1));   // clamped, unconditional
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = k + j < st.in_dim ? v[j] : 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) p[j] = pack_bf16(v[2 * j], v[2 * j + 1]);
    };
    if (a.x_next) {
      unsigned int p[4];
      round8(a.x_next, p);
      stg16(st.xq0 + (size_t)s * st.in_pad + k, make_uint4(p[0], p[1], p[2], p[3]));
    }
    if (LEARN) {
      unsigned int p[4];
      round8(a.x, p);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        tr[0][(8 * rq + 2 * j) * kMsS + s] = (unsigned short)(p[j] & 0xffffu);
        tr[0][(8 * rq + 2 * j + 1) * kMsS + s] = (unsigned short)(p[j] >> 16);
      }
      __syncthreads();
      stg16(st.xT0 + (size_t)(tl.a + trow) * kMsS + 8 * tq, *reinterpret_cast<const uint4 *>(&tr[0][trow * kMsS + 8 * tq]));
    }
    return;
  }

  // a1 (second half of Eq. 6): z = b + the column tiles' shares of W x, summed in a fixed order.  Rows beyond out_dim
  // are padding: their weights and biases are zero, so z = o = 0 there and the padded stores are unconditional.
  const int r = tl.a + 8 * rq;
  const size_t plane = (size_t)kMsS * st.out_pad;
  const bool fwd = tl.kind != 4, bwd = LEARN && tl.kind != 3;
  float z[8];
  if (fwd) {
    const float4 b0 = ldg_f4(st.b + r), b1 = ldg_f4(st.b + r + 4);
    z[0] = b0.x; z[1] = b0.y; z[2] = b0.z; z[3] = b0.w; z[4] = b1.x; z[5] = b1.y; z[6] = b1.z; z[7] = b1.w;
    ms_add_planes<8>(st.zp, s, r, st.n_ct, plane, z);
    if (tl.kind == 3) {   // a layer that is not the last of its stage: delta needs this tick's z later in the tick (Eq. 9)
      stg_f4(st.zbuf + (size_t)s * st.out_pad + r, make_float4(z[0], z[1], z[2], z[3]));
      stg_f4(st.zbuf + (size_t)s * st.out_pad + r + 4, make_float4(z[4], z[5], z[6], z[7]));
    }
  } else {
    const float4 z0 = ldg_f4(st.zbuf + (size_t)s * st.out_pad + r), z1 = ldg_f4(st.zbuf + (size_t)s * st.out_pad + r + 4);
    z[0] = z0.x; z[1] = z0.y; z[2] = z0.z; z[3] = z0.w; z[4] = z1.x; z[5] = z1.y; z[6] = z1.z; z[7] = z1.w;
  }
  float o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = act_fwd(st.act, z[j]);
  if (fwd && st.skip_in) {
    // the skipped tensor is added after the activation
    const float4 s0 = ldg_f4(st.skip_in + (size_t)s * st.out_pad + r), s1 = ldg_f4(st.skip_in + (size_t)s * st.out_pad + r + 4);
    o[0] += s0.x; o[1] += s0.y; o[2] += s0.z; o[3] += s0.w; o[4] += s1.x; o[5] += s1.y; o[6] += s1.z; o[7] += s1.w;
  }
  if (fwd && st.skip_out) {
    stg_f4(st.skip_out + (size_t)s * st.out_pad + r, make_float4(o[0], o[1], o[2], o[3]));
    stg_f4(st.skip_out + (size_t)s * st.out_pad + r + 4, make_float4(o[4], o[5], o[6], o[7]));
  }
  if (st.is_last) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (r + j < st.out_dim) stg_f(a.out + (size_t)s * st.out_dim + r + j, o[j]);
    if (LEARN) {   // the loss head (first work-groups of the matrix launch) reads the pre-activations of the stage
      stg_f4(st.zbuf + (size_t)s * st.out_pad + r, make_float4(z[0], z[1], z[2], z[3]));
      stg_f4(st.zbuf + (size_t)s * st.out_pad + r + 4, make_float4(z[4], z[5], z[6], z[7]));
      if (net.loss == PT_LOSS_CE) {
        // this tile's share of the softmax statistics of stream s: its largest output and the sum of exp(output - largest)
        // over its rows (rows beyond out_dim are not outputs); the 8 lanes of a stream are neighbours
        float m = -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; ++j) m = r + j < st.out_dim ? fmaxf(m, o[j]) : m;
        m = fmaxf(m, __shfl_xor(m, 1, 64));
        m = fmaxf(m, __shfl_xor(m, 2, 64));
        m = fmaxf(m, __shfl_xor(m, 4, 64));
        float t = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) t += r + j < st.out_dim ? expf(o[j] - m) : 0.f;
        t += __shfl_xor(t, 1, 64);
        t += __shfl_xor(t, 2, 64);
        t += __shfl_xor(t, 4, 64);
        if (rq == 0) {
          float *hp = net.hstat + ((size_t)(tl.a / kMsVR) * kMsS + s) * 2;
          stg_f(hp, m);
          stg_f(hp + 1, t);
        }
      }
    }
    return;
  }
  unsigned int po[4] = {0u, 0u, 0u, 0u}, pd[4] = {0u, 0u, 0u, 0u};
  if (fwd) {
    stg_f4(st.out_cur + (size_t)s * st.out_pad + r, make_float4(o[0], o[1], o[2], o[3]));
    stg_f4(st.out_cur + (size_t)s * st.out_pad + r + 4, make_float4(o[4], o[5], o[6], o[7]));
#pragma unroll
    for (int j = 0; j < 4; ++j) po[j] = pack_bf16(o[2 * j], o[2 * j + 1]);
    stg16(st.xq_cur + (size_t)s * st.out_pad + r, make_uint4(po[0], po[1], po[2], po[3]));
  }
  if (bwd) {
    // a3, a4: g = the error published by the next stage one tick earlier, or by the layer behind in this stage in this
    // tick (sum of its row-tile planes, Eq. 11 / Eq. 5), delta = rnd(g * phi'(z)) with this tick's z (Eq. 9).
    // Padding rows have z = 0 and g = 0, hence delta = 0.
    float g[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    ms_add_planes<4>(st.gin_prev, s, r, st.n_gparts, plane, g);
    if (st.serr_in) {    // source of a skip: the delayed gradient of the target joins
      const float4 e0 = ldg_f4(st.serr_in + (size_t)s * st.out_pad + r), e1 = ldg_f4(st.serr_in + (size_t)s * st.out_pad + r + 4);
      g[0] += e0.x; g[1] += e0.y; g[2] += e0.z; g[3] += e0.w; g[4] += e1.x; g[5] += e1.y; g[6] += e1.z; g[7] += e1.w;
    }
    if (st.serr_out) {   // target of a skip: the gradient at its output goes back unchanged
      stg_f4(st.serr_out + (size_t)s * st.out_pad + r, make_float4(g[0], g[1], g[2], g[3]));
      stg_f4(st.serr_out + (size_t)s * st.out_pad + r + 4, make_float4(g[4], g[5], g[6], g[7]));
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) pd[j] = pack_bf16(g[2 * j] * act_der(st.act, z[2 * j]), g[2 * j + 1] * act_der(st.act, z[2 * j + 1]));
    ms_put_delta(st.dlt, s, r, pd);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    tr[0][(8 * rq + 2 * j) * kMsS + s] = (unsigned short)(po[j] & 0xffffu);
    tr[0][(8 * rq + 2 * j + 1) * kMsS + s] = (unsigned short)(po[j] >> 16);
    if (LEARN) {
      tr[1][(8 * rq + 2 * j) * kMsS + s] = (unsigned short)(pd[j] & 0xffffu);
      tr[1][(8 * rq + 2 * j + 1) * kMsS + s] = (unsigned short)(pd[j] >> 16);
    }
  }
  __syncthreads();
  const int row = tl.a + trow;
  if (fwd) stg16(st.xT_cur + (size_t)row * kMsS + 8 * tq, *reinterpret_cast<const uint4 *>(&tr[0][trow * kMsS + 8 * tq]));
  if (bwd) {
    const uint4 d = *reinterpret_cast<const uint4 *>(&tr[1][trow * kMsS + 8 * tq]);
    stg16(st.dltT + (size_t)row * kMsS + 8 * tq, d);
    // a6 for the bias: b <- b - eta / S * sum over the streams of the rounded delta (what every product sees)
    float dsum = bf16_lo(d.x) + bf16_hi(d.x) + bf16_lo(d.y) + bf16_hi(d.y) + bf16_lo(d.z) + bf16_hi(d.z) + bf16_lo(d.w) + bf16_hi(d.w);
    dsum += __shfl_xor(dsum, 1, 64);
    dsum += __shfl_xor(dsum, 2, 64);
    if (tq == 0) {
      float mq = net.adam ? ldg_f(st.mb + row) : 0.f, vq = net.adam ? ldg_f(st.vb + row) : 0.f;
      stg_f(st.b + row, ms_step(net, a, ldg_f(st.b + row), dsum, mq, vq));
      if (net.adam) {
        stg_f(st.mb + row, mq);
        stg_f(st.vb + row, vq);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// inference tick (Eq. 6 only): one launch, nothing is folded across the tick boundary because nothing is written to
// the weights.  Tile = 64 rows of one stage x all columns, wave w owns 16 rows; the weights go from HBM straight into
// operand registers, the bf16 stage input, shared by the four waves, is staged through LDS one block of 512 columns at
// a time.  (Reading the shared operand from L2 in every wave instead was measured 2.7x slower.)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ms_infer_kernel(MsNet net, MsTick a) {
  constexpr int NB = kMsRW / 16;   // 16-row blocks per wave
  __shared__ __attribute__((aligned(16))) unsigned short xs[2][kMsS * kMsXPitch];
  const MsTileRec *rec = net.tiles_i + blockIdx.x;
  const MsTile tl = rec->t;
  const MsView st = ms_view(&rec->s, a.cur, a.cur ^ 1, a.tick);
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, li = lane & 15, g = lane >> 4;
  const bf16_t *xq = st.is_first ? nullptr : st.xq_fwd;   // what the stage in front published one tick earlier
  const int r0 = tl.a + kMsRW * wv;                    // out_pad is a multiple of the tile: always in range
  // W[r0 + 16 b + li][col + 32 u + 8 g .. + 7] is one 16-byte piece per lane, 1 KiB per wave (see ms_woff)
  const size_t cstride = (size_t)(st.out_pad >> 5) * kMsBlk;
  const bf16_t *wlane = st.W + lane * 8;
  f32x4_t acc[NB][2];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int h = 0; h < 2; ++h) acc[b][h] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // All tiles of a launch are resident together.  Walking the column blocks in the same order everywhere (sweep)
  // was measured 13 % faster in forward-only ticks than starting every tile at a different block.
  const int n_chunks = (st.in_pad + kMsKC - 1) / kMsKC;
  const int c_first = 0;
  auto chunk_at = [&](int ci) { return ((ci + c_first) % n_chunks) * kMsKC; };

  // X blocks are double buffered: block ci+1 is fetched into registers while block ci is multiplied, then
  // written to the other LDS buffer; one work-group barrier per block
  uint4 xr[8];
  // every load below is unconditional (addresses are clamped, out-of-range values are zeroed afterwards):
  // a branch around each load would make the compiler wait for one load before it issues the next
  auto fetch_x = [&](int kc) {
    const int kn = min(kMsKC, st.in_pad - kc);
    if (xq) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int i = tid + 256 * q, s = i / (kMsKC / 8), k8 = min((i % (kMsKC / 8)) * 8, kn - 8);
        xr[q] = ldg16(xq + (size_t)s * st.in_pad + kc + k8);
      }
    } else {
      // first stage: the caller's fp32 sample is rounded on the way in
      if ((st.in_dim & 3) == 0) {
        float4 v[8][2];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int i = tid + 256 * q, s = i / (kMsKC / 8), k = kc + (i % (kMsKC / 8)) * 8;
          const float *xp = a.x + (size_t)s * st.in_dim;
          v[q][0] = ldg_f4(xp + min(k, st.in_dim - 4));
          v[q][1] = ldg_f4(xp + min(k + 4, st.in_dim - 4));
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int i = tid + 256 * q, k = kc + (i % (kMsKC / 8)) * 8;
          const bool lo = k < st.in_dim, hi = k + 4 < st.in_dim;   // in_dim is a multiple of 4: whole quads
          xr[q] = make_uint4(lo ? pack_bf16(v[q][0].x, v[q][0].y) : 0u, lo ? pack_bf16(v[q][0].z, v[q][0].w) : 0u,
                             hi ? pack_bf16(v[q][1].x, v[q][1].y) : 0u, hi ? pack_bf16(v[q][1].z, v[q][1].w) : 0u);
        }
      } else {
        float v[8][8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int i = tid + 256 * q, s = i / (kMsKC / 8), k8 = (i % (kMsKC / 8)) * 8;
          const float *xp = a.x + (size_t)s * st.in_dim;
#pragma unroll
          for (int e = 0; e < 8; ++e) v[q][e] = ldg_f(xp + min(kc + k8 + e, st.in_dim - 1));
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int i = tid + 256 * q, k8 = (i % (kMsKC / 8)) * 8;
#pragma unroll
          for (int e = 0; e < 8; ++e) v[q][e] = kc + k8 + e < st.in_dim ? v[q][e] : 0.f;
          xr[q] = make_uint4(pack_bf16(v[q][0], v[q][1]), pack_bf16(v[q][2], v[q][3]), pack_bf16(v[q][4], v[q][5]),
                             pack_bf16(v[q][6], v[q][7]));
        }
      }
    }
  };
  auto put_x = [&](unsigned short *buf) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int i = tid + 256 * q, s = i / (kMsKC / 8), k8 = (i % (kMsKC / 8)) * 8;
      *reinterpret_cast<uint4 *>(&buf[s * kMsXPitch + k8]) = xr[q];
    }
  };
  // weights: two register sets, the next 256 columns are requested before the current 256 are multiplied
  auto wload = [&](uint4 (&w)[NB][8], int col) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int rr = r0 + 16 * b;
        w[b][u] = ldg16(wlane + (size_t)(col / kMsTC) * cstride + (size_t)(rr >> 5) * kMsBlk + (((col % kMsTC) >> 5) + u) * 1024 + ((rr >> 4) & 1) * 512);
      }
  };
  auto wmul = [&](const uint4 (&w)[NB][8], const unsigned short *xb, int kb) {
    // all sixteen operand reads of the step are issued before the first product: one LDS latency per step
    // instead of one per product
    uint4 bq[2][8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      bq[0][u] = *reinterpret_cast<const uint4 *>(&xb[li * kMsXPitch + kb + 32 * u + g * 8]);
      bq[1][u] = *reinterpret_cast<const uint4 *>(&xb[(16 + li) * kMsXPitch + kb + 32 * u + g * 8]);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        acc[b][0] = mfma16(w[b][u], bq[0][u], acc[b][0]);
        acc[b][1] = mfma16(w[b][u], bq[1][u], acc[b][1]);
      }
  };
  uint4 wa[NB][8], wb[NB][8];
  wload(wa, chunk_at(0));
  fetch_x(chunk_at(0));
  put_x(xs[0]);
  __syncthreads();
  for (int ci = 0; ci < n_chunks; ++ci) {
    const int kc = chunk_at(ci);                        // in_pad is a multiple of 512: every block is two steps
    const unsigned short *xb = xs[ci & 1];
    const bool more = ci + 1 < n_chunks;
    if (more) fetch_x(chunk_at(ci + 1));
    wload(wb, kc + 256);
    // keep the requests ahead of the products: left alone, the scheduler sinks each load next to its first use
    __builtin_amdgcn_sched_barrier(0);
    wmul(wa, xb, 0);
    if (more) wload(wa, chunk_at(ci + 1));
    __builtin_amdgcn_sched_barrier(0);
    wmul(wb, xb, 256);
    if (more) {
      put_x(xs[(ci + 1) & 1]);   // the other buffer: nobody reads it during this block
      __syncthreads();
    }
  }
  // C layout: lane (li, g) holds rows r0 + 16 b + 4 g + j of stream s = 16 h + li.  Rows beyond out_dim are
  // padding: their weights and biases are zero, so z = o = 0 there and every store below is unconditional
  // (only the caller's unpadded output array needs a guard).
  float4 bias[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) bias[b] = ldg_f4(st.b + r0 + 16 * b + 4 * g);
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int rb = r0 + 16 * b + 4 * g;
    const float bb[4] = {bias[b].x, bias[b].y, bias[b].z, bias[b].w};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int s = 16 * h + li;
      float o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = act_fwd(st.act, acc[b][h][j] + bb[j]);
      if (st.skip_in) {
        const float4 sk = ldg_f4(st.skip_in + (size_t)s * st.out_pad + rb);
        o[0] += sk.x; o[1] += sk.y; o[2] += sk.z; o[3] += sk.w;
      }
      if (st.skip_out) stg_f4(st.skip_out + (size_t)s * st.out_pad + rb, make_float4(o[0], o[1], o[2], o[3]));
      if (st.is_last) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (rb + j < st.out_dim) stg_f(a.out + (size_t)s * st.out_dim + rb + j, o[j]);
      } else {
        stg_f4(st.out_cur + (size_t)s * st.out_pad + rb, make_float4(o[0], o[1], o[2], o[3]));
        // bf16 copies for the next stage's products: [S][out_pad] and transposed [out_pad][S]
        const unsigned int p01 = pack_bf16(o[0], o[1]), p23 = pack_bf16(o[2], o[3]);
        stg8(st.xq_cur + (size_t)s * st.out_pad + rb, make_uint2(p01, p23));
        bf16_t *t = st.xT_cur + (size_t)rb * kMsS + s;
        stg_u16(t, p01 & 0xffffu);
        stg_u16(t + kMsS, p01 >> 16);
        stg_u16(t + 2 * kMsS, p23 & 0xffffu);
        stg_u16(t + 3 * kMsS, p23 >> 16);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// loss head of the last stage (a2, a4 and the bias part of a6): a tile is 64 rows x the 32 streams, thread (stream s,
// group of 8 rows) as in the vector kernel.  A softmax needs every output of its stream: the vector launch has left,
// per tile of 64 rows and per stream, the largest output and the sum of exp(output - largest); every head tile combines
// them in the same order, so all tiles work with the same statistics.  The head tiles are the first work-groups of the
// matrix launch; each counts itself in when its deltas are in memory, and the matrix tiles of the last stage start when
// all have done so.  (One work-group for the whole head took 25 us, with the last stage's tiles waiting behind it.)
// The activation is a template parameter: with a run-time switch inside the element loops every load sits in its
// own basic block and is waited for before the next one is issued.
// ------------------------------------------------------------------------------------------------
template <int ACT>
__device__ __forceinline__ void ms_head_tile(const MsNet &net, const MsTick &a, const MsTile &tl, const MsView &st, float *lds) {
  unsigned short *tr = reinterpret_cast<unsigned short *>(lds);   // bf16 [64 rows][32 streams]
  float *sloss = lds + kMsVR * kMsS / 2, *sred = sloss + kMsS;
  const int tid = threadIdx.x, s = tid >> 3, rq = tid & 7, trow = tid >> 2, tq = tid & 3;
  const bool ce = net.loss == PT_LOSS_CE, mse = net.loss == PT_LOSS_MSE;
  const float inv_n = 1.f / (float)net.out_dim;
  const int r = tl.a + 8 * rq;
  const float4 z0 = ldg_f4(st.zbuf + (size_t)s * st.out_pad + r), z1 = ldg_f4(st.zbuf + (size_t)s * st.out_pad + r + 4);
  const float z[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
  float gg[8], sq = 0.f, smax = 0.f, ssum = 1.f;
  int ys = 0;
  if (ce) {
    const int n_vt = st.out_pad / kMsVR;
    const float *hp = net.hstat + 2 * s;
    smax = -INFINITY;
    for (int t = 0; t < n_vt; ++t) smax = fmaxf(smax, ldg_f(hp + (size_t)t * 2 * kMsS));
    ssum = 0.f;
    for (int t = 0; t < n_vt; ++t) {
      const float mt = ldg_f(hp + (size_t)t * 2 * kMsS), et = ldg_f(hp + (size_t)t * 2 * kMsS + 1);
      ssum += et > 0.f ? et * expf(mt - smax) : 0.f;   // (a tile of padding rows only has no outputs)
    }
    ys = min(max(ldg_i(static_cast<const int *>(a.tgt) + s), 0), st.out_dim - 1);
    const float inv = 1.f / ssum;
#pragma unroll
    for (int j = 0; j < 8; ++j) gg[j] = a.learn ? expf(act_fwd(ACT, z[j]) - smax) * inv - (r + j == ys ? 1.f : 0.f) : 0.f;
  } else if (mse) {
    float y[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) y[j] = ldg_f(static_cast<const float *>(a.tgt) + (size_t)s * st.out_dim + min(r + j, st.out_dim - 1));
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float df = act_fwd(ACT, z[j]) - y[j];
      if (r + j < st.out_dim) sq = fmaf(df, df, sq);
      gg[j] = a.learn ? 2.f * df * inv_n : 0.f;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) gg[j] = 0.f;
  }
  // a4 for the last stage; the rounded delta is what every product (and the bias update) sees.  Rows beyond out_dim are
  // padding: their delta is zero
  unsigned int pd[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    pd[j] = pack_bf16(r + 2 * j < st.out_dim ? gg[2 * j] * act_der(ACT, z[2 * j]) : 0.f,
                      r + 2 * j + 1 < st.out_dim ? gg[2 * j + 1] * act_der(ACT, z[2 * j + 1]) : 0.f);
  ms_put_delta(st.dlt, s, r, pd);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    tr[(8 * rq + 2 * j) * kMsS + s] = (unsigned short)(pd[j] & 0xffffu);
    tr[(8 * rq + 2 * j + 1) * kMsS + s] = (unsigned short)(pd[j] >> 16);
  }
  if (ce && tl.a == 0 && rq == 0)
    sloss[s] = -(act_fwd(ACT, ldg_f(st.zbuf + (size_t)s * st.out_pad + ys)) - smax - logf(ssum));
  if (mse) {
    sq = wave_sum(sq);
    if ((tid & 63) == 0) sred[tid >> 6] = sq;
  }
  __syncthreads();
  const int row = tl.a + trow;
  const uint4 d = *reinterpret_cast<const uint4 *>(&tr[trow * kMsS + 8 * tq]);
  stg16(st.dltT + (size_t)row * kMsS + 8 * tq, d);
  float dsum = bf16_lo(d.x) + bf16_hi(d.x) + bf16_lo(d.y) + bf16_hi(d.y) + bf16_lo(d.z) + bf16_hi(d.z) + bf16_lo(d.w) + bf16_hi(d.w);
  dsum += __shfl_xor(dsum, 1, 64);
  dsum += __shfl_xor(dsum, 2, 64);
  if (tq == 0 && row < st.out_dim) {
    float mq = net.adam ? ldg_f(st.mb + row) : 0.f, vq = net.adam ? ldg_f(st.vb + row) : 0.f;
    stg_f(st.b + row, ms_step(net, a, ldg_f(st.b + row), dsum, mq, vq));
    if (net.adam) {
      stg_f(st.mb + row, mq);
      stg_f(st.vb + row, vq);
    }
  }
  if (ce && tl.a == 0 && tid == 0) {
    float L = 0.f;
    for (int q = 0; q < kMsS; ++q) L += sloss[q];
    a.loss1[0] = a.learn ? L * net.inv_s : 0.f;
  }
  if (mse && tid == 0) {
    float t = 0.f;
    for (int w = 0; w < kMsNWM; ++w) t += sred[w];
    __hip_atomic_store(net.hpart + tl.a / kMsVR, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // everything above is released to the rest of the device before this tile counts itself in
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const unsigned int before = __hip_atomic_fetch_add(net.head_flag, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (mse && before + 1u == a.seq) {
      // the last head tile of the tick adds the tiles' shares of the squared error in a fixed order
      float t = 0.f;
      for (int q = 0; q < st.out_pad / kMsVR; ++q) t += __hip_atomic_load(net.hpart + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      a.loss1[0] = a.learn ? t * inv_n * net.inv_s : 0.f;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// matrix kernel: tile = a block of rows (the stage's tile height) x kMsTC columns of one stage; the four waves share the rows and take 128
// columns each, so a wave keeps its share of E = W^T delta for its own columns to itself (64 VGPRs), while the four
// shares of the coming tick's Z for a block of 32 rows meet in LDS (one work-group barrier per block).
// MODE 0: a learning tick (E, update, forward of the coming tick); MODE 1: forward only.
// ------------------------------------------------------------------------------------------------

// what a wave holds of one block of 32 rows: its 32 x 128 weights and, for a learning tick, the deltas of those rows
// in the two operand layouts.  Everything is requested one block ahead, the deltas together with the weights: the
// memory counter of this chip retires in order, so a load that is issued after the prefetch and awaited before the
// arithmetic would make the arithmetic wait for the prefetch as well.
struct MsBlock {
  uint4 w[kMsSB][2];   // W[r0 + 16 b + li][c0 + 32 sb + 8 g .. + 7]
  uint4 de[2];     // delta as B operand of E (contraction over the 32 rows): rows r0 + 16 b + 4 g + j at stream 16 h + li
  uint4 du[2];     // delta^T as B operand of the update (contraction over the 32 streams): row r0 + 16 b + li, streams 8 g ..
};

template <int MODE, int OPT, bool HAS_E, bool FWD>
__device__ __forceinline__ void ms_mat_tile(const MsNet &net, const MsTick &a, const MsTile &tl, const MsView &st,
                                            float (&zred)[2][kMsNWM][1024]) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, li = lane & 15, g = lane >> 4;
  const int row_lo = tl.a * st.tr, row_hi = min(row_lo + st.tr, st.out_pad);   // multiples of 64 (sizes are padded)
  const int c0 = tl.b * kMsTC + 32 * kMsSB * wv;                                      // this wave's 128 columns
  // this lane's 16 bytes of W[r0 + 16 b + li][c0 + 32 sb + 8 g .. + 7] sit at wbase + (r0 / 32) * kMsBlk + (2 sb + b) * 512
  const size_t wbase = (size_t)tl.b * (st.out_pad >> 5) * kMsBlk + wv * (kMsSB * 1024) + lane * 8;

  // selectors that move a 16 x 32 register block into C layout (multiplication by a 0/1 matrix is exact)
  uint4 isel[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    unsigned int w[4] = {0u, 0u, 0u, 0u};
    const int m = c * 16 + li - g * 8;                 // element of this lane's 8 that must be 1.0
    if (m >= 0 && m < 8) w[m >> 1] = (m & 1) ? 0x3f800000u : 0x00003f80u;
    isel[c] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  // update operand A = rnd(X)[k(slot)][s]: slot = l % 16 = 4 q + jj  ->  k = c0 + 32 sb + 8 q + 4 e + jj
  uint4 xop[kMsSB][2];
  // forward operand B = rnd(X_next)[k][s]: lane (stream 16 h + li) holds k = c0 + 32 sb + 8 g .. + 7
  uint4 xf[kMsSB][2];
#pragma unroll
  for (int sb = 0; sb < kMsSB; ++sb)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      if (MODE == 0) {
        const int k = c0 + 32 * sb + 8 * (li >> 2) + 4 * e + (li & 3);
        xop[sb][e] = ldg16(st.xT_prev + (size_t)k * kMsS + g * 8);
      }
      if (FWD) xf[sb][e] = ldg16(st.xq_fwd + (size_t)(16 * e + li) * st.in_pad + c0 + 32 * sb + g * 8);
    }
  f32x4_t eacc[kMsSB][2][2];
#pragma unroll
  for (int sb = 0; sb < kMsSB; ++sb)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int h = 0; h < 2; ++h) eacc[sb][c][h] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const float scale = net.lr_over_s;
  auto load_block = [&](MsBlock &k, int r0) {
#pragma unroll
    for (int sb = 0; sb < kMsSB; ++sb)
#pragma unroll
      for (int b = 0; b < 2; ++b)
        k.w[sb][b] = ldg16(st.W + wbase + (size_t)(r0 >> 5) * kMsBlk + (2 * sb + b) * 512);
    if (MODE == 0) {
#pragma unroll
      for (int h = 0; h < 2; ++h) k.de[h] = ldg16(st.dlt + ((size_t)((r0 >> 5) * 2 + h) * 64 + lane) * 8);
#pragma unroll
      for (int b = 0; b < 2; ++b) k.du[b] = ldg16(st.dltT + (size_t)(r0 + 16 * b + li) * kMsS + g * 8);
    }
  };
  auto process_block = [&](MsBlock &k, int r0, int slot) {
    f32x4_t facc[2][2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int h = 0; h < 2; ++h) facc[b][h] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (MODE == 0 && OPT == 0) {
      // Plain SGD.  A wave is alone on its SIMD, so whatever waits for a result of the matrix pipe waits in full: the
      // products whose results the vector pipe works on are issued a whole phase ahead of that work, and each phase
      // pairs products with vector work that does not depend on them.
      const f32x4_t z4 = {0.f, 0.f, 0.f, 0.f};
      f32x4_t t[kMsSB][2][2], u[kMsSB][2][2];
      // phase 1: the block turned into the other operand layout, W[r0 + 16 q + 4 g + j][c0 + 32 sb + 16 c + li] in t[sb][c][q]
      if (HAS_E) {
#pragma unroll
        for (int sb = 0; sb < kMsSB; ++sb)
#pragma unroll
          for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int q = 0; q < 2; ++q) t[sb][c][q] = mfma16(k.w[sb][q], isel[c], z4);
      }
      __builtin_amdgcn_sched_barrier(0);
      // phase 2: the update products delta rnd(X)^T (they come out as lane (row li, k = 8 g + 4 e + j), the layout of the
      // loaded weights), while the vector pipe rounds the turned block
      uint4 wt[kMsSB][2];
#pragma unroll
      for (int sb = 0; sb < kMsSB; ++sb)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
          for (int e = 0; e < 2; ++e) u[sb][b][e] = mfma16(xop[sb][e], k.du[b], z4);
          if (HAS_E)
            wt[sb][b] = make_uint4(pack_bf16(t[sb][b][0][0], t[sb][b][0][1]), pack_bf16(t[sb][b][0][2], t[sb][b][0][3]),
                                   pack_bf16(t[sb][b][1][0], t[sb][b][1][1]), pack_bf16(t[sb][b][1][2], t[sb][b][1][3]));
        }
      if (HAS_E) {
#pragma unroll
        for (int i = 0; i < 4 * kMsSB; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one product,
          __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);   // then vector work under it
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      // phase 3: a6, W <- rnd(W - eta/S * delta rnd(X)^T), on the vector pipe; under it a5, E[k][s] += sum_r W[r][k]
      // delta[r][s] with the rows as loaded, and a1 of the coming tick (first half of Eq. 6) with the rows as stored
#pragma unroll
      for (int sb = 0; sb < kMsSB; ++sb)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const uint4 w = k.w[sb][b];
          const f32x4_t u0 = u[sb][b][0], u1 = u[sb][b][1];
          uint4 o;
          o.x = pack_bf16(bf16_lo(w.x) - scale * u0[0], bf16_hi(w.x) - scale * u0[1]);
          o.y = pack_bf16(bf16_lo(w.y) - scale * u0[2], bf16_hi(w.y) - scale * u0[3]);
          o.z = pack_bf16(bf16_lo(w.z) - scale * u1[0], bf16_hi(w.z) - scale * u1[1]);
          o.w = pack_bf16(bf16_lo(w.w) - scale * u1[2], bf16_hi(w.w) - scale * u1[3]);
          stg16(st.W + wbase + (size_t)(r0 >> 5) * kMsBlk + (2 * sb + b) * 512, o);
          if (HAS_E) {
#pragma unroll
            for (int h = 0; h < 2; ++h) eacc[sb][b][h] = mfma16(wt[sb][b], k.de[h], eacc[sb][b][h]);
          }
          if (FWD) {
#pragma unroll
            for (int h = 0; h < 2; ++h) facc[b][h] = mfma16(o, xf[sb][h], facc[b][h]);
          }
        }
      {
        constexpr int n_mfma = 2 * kMsSB * ((HAS_E ? 2 : 0) + (FWD ? 2 : 0));
#pragma unroll
        for (int i = 0; i < n_mfma; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x002, (HAS_E && FWD) ? 7 : 14, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    } else if (MODE == 0) {
      // Adam: the moments of 32 columns (both 16-row halves) travel one column group ahead of the arithmetic
      float4 mv[OPT == 1 ? 2 : 1][2][4];
      auto load_mv = [&](int buf, int sb) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const size_t off = wbase + (size_t)(r0 >> 5) * kMsBlk + (2 * sb + b) * 512;
          mv[buf][b][0] = ldg_f4(st.mW + off); mv[buf][b][1] = ldg_f4(st.mW + off + 4);
          mv[buf][b][2] = ldg_f4(st.vW + off); mv[buf][b][3] = ldg_f4(st.vW + off + 4);
        }
      };
      if (OPT == 1) load_mv(0, 0);
#pragma unroll
      for (int sb = 0; sb < kMsSB; ++sb) {
        if (OPT == 1 && sb + 1 < kMsSB) load_mv((sb + 1) & 1, sb + 1);
        if (HAS_E) {
          // a5: E[k][s] += sum_r W[r][k] delta[r][s] with the rows as loaded (not yet updated)
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            const f32x4_t z4 = {0.f, 0.f, 0.f, 0.f};
            const f32x4_t t0 = mfma16(k.w[sb][0], isel[c], z4);   // W[r0 + 4 g + j][c0 + 32 sb + 16 c + li]
            const f32x4_t t1 = mfma16(k.w[sb][1], isel[c], z4);   // rows + 16
            const uint4 wt = make_uint4(pack_bf16(t0[0], t0[1]), pack_bf16(t0[2], t0[3]),
                                        pack_bf16(t1[0], t1[1]), pack_bf16(t1[2], t1[3]));
#pragma unroll
            for (int h = 0; h < 2; ++h) eacc[sb][c][h] = mfma16(wt, k.de[h], eacc[sb][c][h]);
          }
        }
        // a6: W <- rnd(W - eta/S * delta rnd(X)^T); the product comes out as lane (row li, k = 8 g + 4 e + j)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const f32x4_t z4 = {0.f, 0.f, 0.f, 0.f};
          const uint4 w = k.w[sb][b];
          const f32x4_t u0 = mfma16(xop[sb][0], k.du[b], z4);
          const f32x4_t u1 = mfma16(xop[sb][1], k.du[b], z4);
          const size_t off = wbase + (size_t)(r0 >> 5) * kMsBlk + (2 * sb + b) * 512;
          uint4 o;
          if (OPT == 1) {
            // Adam: the moments of the lane's 8 weights, fp32, in and out
            const float4 m0 = mv[sb & 1][b][0], m1 = mv[sb & 1][b][1], v0 = mv[sb & 1][b][2], v1 = mv[sb & 1][b][3];
            float wq[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y), bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
            const float gq[8] = {u0[0], u0[1], u0[2], u0[3], u1[0], u1[1], u1[2], u1[3]};
            float mq[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w}, vq[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) wq[e] = ms_step(net, a, wq[e], gq[e], mq[e], vq[e]);
            stg_f4(st.mW + off, make_float4(mq[0], mq[1], mq[2], mq[3]));
            stg_f4(st.mW + off + 4, make_float4(mq[4], mq[5], mq[6], mq[7]));
            stg_f4(st.vW + off, make_float4(vq[0], vq[1], vq[2], vq[3]));
            stg_f4(st.vW + off + 4, make_float4(vq[4], vq[5], vq[6], vq[7]));
            o = make_uint4(pack_bf16(wq[0], wq[1]), pack_bf16(wq[2], wq[3]), pack_bf16(wq[4], wq[5]), pack_bf16(wq[6], wq[7]));
          } else {
            o.x = pack_bf16(bf16_lo(w.x) - scale * u0[0], bf16_hi(w.x) - scale * u0[1]);
            o.y = pack_bf16(bf16_lo(w.y) - scale * u0[2], bf16_hi(w.y) - scale * u0[3]);
            o.z = pack_bf16(bf16_lo(w.z) - scale * u1[0], bf16_hi(w.z) - scale * u1[1]);
            o.w = pack_bf16(bf16_lo(w.w) - scale * u1[2], bf16_hi(w.w) - scale * u1[3]);
          }
          stg16(st.W + off, o);
          // a1 of the coming tick (first half of Eq. 6) with the weights as just stored
          if (FWD) {
#pragma unroll
            for (int h = 0; h < 2; ++h) facc[b][h] = mfma16(o, xf[sb][h], facc[b][h]);
          }
        }
      }
    } else {
#pragma unroll
      for (int sb = 0; sb < kMsSB; ++sb)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int h = 0; h < 2; ++h) facc[b][h] = mfma16(k.w[sb][b], xf[sb][h], facc[b][h]);
    }
    if (!FWD) return;
    // the four waves' shares of Z for these 32 rows meet in LDS and are added in a fixed order.  Two slots: the
    // barrier of block i + 1 stands between the reads of block i and the writes of block i + 2.
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int h = 0; h < 2; ++h)
        *reinterpret_cast<f32x4_t *>(&zred[slot][wv][(b * 2 + h) * 256 + lane * 4]) = facc[b][h];
    // A plain work-group barrier also waits for every global access in flight, i.e. for this block's weight stores and
    // for the next block's prefetch: only the LDS writes have to be complete here.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (kMsNWM == 4 || tid < 256) {
      f32x4_t t = *reinterpret_cast<const f32x4_t *>(&zred[slot][0][tid * 4]);
#pragma unroll
      for (int w = 1; w < kMsNWM; ++w) t += *reinterpret_cast<const f32x4_t *>(&zred[slot][w][tid * 4]);
      // position tid = (b, h, lane'): rows r0 + 16 b + 4 g' + j of stream 16 h + li'
      // which in the planes' order is simply the tid-th 16-byte piece of the block's 4 KiB
      float *dst = st.zp + (size_t)tl.b * kMsS * st.out_pad + ((size_t)(r0 >> 5) * 256 + tid) * 4;
      stg_f4(dst, make_float4(t[0], t[1], t[2], t[3]));
    }
  };
  {
    // A ring of kMsRing register sets: block i + kMsRing - 1 is requested before block i is worked on.  A wave is alone on
    // its SIMD, so nothing else covers the time its requests are under way.  The loop has no data-dependent branch (a
    // tile is a whole number of rings; requests beyond the last block are clamped onto it and never used): where paths
    // with different numbers of requests in flight meet, the compiler has to wait for all of them, and the prefetch
    // would no longer run ahead of the arithmetic.
    constexpr int NR = (MODE == 0 && OPT == 1) ? 2 : kMsRing;   // (with Adam the moments take the registers)
    MsBlock kq[NR];
    // Odd ticks walk the tile's rows from the bottom up: what a tick wrote last is what the next tick reads first, while
    // it is still in the memory-side cache.
    const int n_blk = (row_hi - row_lo) >> 5;
    const bool rev = (a.cur & 1) != 0;
    auto row_of = [&](int i) { return rev ? row_hi - 32 - 32 * i : row_lo + 32 * i; };
#pragma unroll
    for (int u = 0; u < NR - 1; ++u) load_block(kq[u], row_of(u));
    for (int i = 0; i < n_blk; i += NR) {
#pragma unroll
      for (int u = 0; u < NR; ++u) {
        // (the scheduling barriers keep the requests where they are written: left alone, the scheduler sinks every
        // load next to its first use, i.e. behind the arithmetic it is meant to overlap)
        load_block(kq[(u + NR - 1) % NR], row_of(min(i + u + NR - 1, n_blk - 1)));
        __builtin_amdgcn_sched_barrier(0);
        process_block(kq[u], row_of(i + u), u & 1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  if (!HAS_E) return;
  // this wave's columns of error plane tl.a: lane (li, g) holds E[k = c0 + 32 sb + 16 c + 4 g + j][s = 16 h + li]
  float *plane = st.eout_cur + (size_t)tl.a * kMsS * st.in_pad;
#pragma unroll
  for (int sb = 0; sb < kMsSB; ++sb)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        float *dst = plane + ((size_t)(((c0 + 32 * sb + 16 * c) >> 4) * 2 + h) * 64 + lane) * 4;
        stg_f4(dst, make_float4(eacc[sb][c][h][0], eacc[sb][c][h][1], eacc[sb][c][h][2], eacc[sb][c][h][3]));
      }
}

template <int MODE, int OPT>
__global__ __launch_bounds__(64 * kMsNWM) void ms_mat_kernel(MsNet net, MsTick a) {
  __shared__ __attribute__((aligned(16))) float zred[2][kMsNWM][1024];
  const MsTileRec *rec = (MODE == 0 ? net.tiles_m : net.tiles_f) + blockIdx.x;
  const MsTile tl = rec->t;
  const MsView st = ms_view(&rec->s, a.cur, a.fhalf);
  const int tid = threadIdx.x;
  if (MODE == 0 && tl.kind == 2) {
    // a2 for the last stage: 64 of its rows
    float *hs = &zred[0][0][0];
    switch (st.act) {
      case PT_RELU: ms_head_tile<PT_RELU>(net, a, tl, st, hs); break;
      case PT_GELU: ms_head_tile<PT_GELU>(net, a, tl, st, hs); break;
      default: ms_head_tile<PT_ID>(net, a, tl, st, hs); break;
    }
    return;
  }
  if (MODE == 0 && st.is_last) {
    // delta of the last stage comes from the head tiles above.  They have the lowest indices of the launch, so they are
    // running or done by the time this one starts; the wait is bounded all the same, and when it runs out the
    // error flag is raised and the tile leaves the weights alone.
    __shared__ int s_ok;
    if (tid == 0) {
      long long spins = 0;
      int ok = 1;
      while ((int)(__hip_atomic_load(net.head_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - a.seq) < 0) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > net.spin_limit) {
          __hip_atomic_store(net.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ok = 0;
          break;
        }
      }
      s_ok = ok;
    }
    __syncthreads();
    if (!s_ok) return;
    // No cache invalidation is needed here (and a device-wide one would throw away the other tiles' operands):
    // caches start a launch empty, and nobody reads the last stage's delta in this launch before the flag is up,
    // so no cache on the device can hold a line of it from before the loss head's release.
  }
  // A layer folds the coming tick's forward product into this launch when it is the first of its stage: its input of the
  // coming tick is what the stage in front has published in this tick, or the caller's next sample (not there at the last
  // tick of a call).  The very first layer publishes no error.
  const bool fold = st.fold && (!st.is_first || a.x_next);
  if (MODE == 1) {
    ms_mat_tile<1, 0, false, true>(net, a, tl, st, zred);
  } else if (!st.is_first) {
    if (fold) ms_mat_tile<0, OPT, true, true>(net, a, tl, st, zred);
    else ms_mat_tile<0, OPT, true, false>(net, a, tl, st, zred);
  } else {
    if (fold) ms_mat_tile<0, OPT, false, true>(net, a, tl, st, zred);
    else ms_mat_tile<0, OPT, false, false>(net, a, tl, st, zred);
  }
}
