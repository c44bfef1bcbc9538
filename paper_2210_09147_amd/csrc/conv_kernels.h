// Convolutional pipeline: stages of conv3x3 (stride 1, pad 1, 64 output channels) + activation, closed by a
// global-average-pool + dense head.  One stream, fp32.  Every stage product is a dense contraction and runs
// on the matrix cores as an implicit GEMM with v_mfma_f32_32x32x2f32.  Included by partime.hip only.
//
// One tick = four launches over all stages when every stage is one layer (steps a0..a7 of the method, per stage);
// with several conv layers per stage (Eq. 3-5) the forward and the backward-data launches are repeated once per
// layer position, the forward ones front to back, the backward ones back to front:
//   cv_conv_kernel<FWD>  z = conv(in, W) + b, o = phi(z) (Eq. 6); delta = g * phi'(z) with g the error the
//                        next stage published one tick earlier (Eq. 11); per-tile bias-gradient partials;
//                        plus the channel means of the last conv stage's published output (pooling of the head)
//   cv_conv_kernel<BWD>  err = conv(delta, W flipped and transposed) = (dz/din)^T delta with the old W (Eq. 11);
//                        plus the head stage (dense, loss, its own update)
//   cv_wgrad_kernel      dW partials: delta correlated with the stage input over a band of rows (Eq. 9)
//   cv_update_kernel     W <- W - eta * sum of partials (or the Adam step on it), in all weight layouts; same for b
//
// Matrix-core layout (32x32x2, D = A * B + C, lane l): A holds A[l % 32][l / 32]; B holds B[l / 32][l % 32];
// C register r holds C[8 (r / 4) + 4 (l / 32) + r % 4][l % 32].

#pragma once

typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kCvCo = 64;       // channels per block: a conv tile computes 64 output channels, wider layers take several tiles
constexpr int kCvMaxC = 256;    // most channels of a conv layer
constexpr int kCvPx = 256;      // pixels per conv tile (whole rows)
constexpr int kCvCiCh = 8;      // input channels staged at a time in the conv kernel
constexpr int kCvNQ = 6;        // 16-byte pieces one thread stages per block of channels, at most
constexpr int kCvWgCi = 16;     // input channels per wave of the weight-gradient kernel
constexpr int kCvWgRows = 4;    // rows per weight-gradient tile
constexpr int kCvWgXC = 64;     // columns a weight-gradient wave stages at a time

struct CvStage {
  float *Wg;               // [co_pad][c_in * 9]   k = ci * 9 + ky * 3 + kx
  float *WT;               // [co_pad / 64][c_in rounded up to even][9][64]   WT[co / 64][ci * 9 + tap][co % 64] = Wg[co][ci * 9 + tap]
  float *WBT;              // [ci_pad / 64][co_pad * 9][64]   WBT[ci / 64][co * 9 + 8 - tap][ci % 64] = Wg[co][ci * 9 + tap] (taps flipped)
  float *b;                // [co_pad]
  float *mW, *vW, *mb, *vb;   // Adam moments in the order of Wg and b (NULL under plain SGD)
  int c_in, c_out, H, W, act;   // real channel counts; buffers and weight layouts are padded to multiples of 64 ...
  int ci_pad, co_pad;           // ... c_in and c_out rounded up, the padding is zero everywhere and stays so
  const float *in_act[2];  // [c_in][H][W] published by the previous stage (NULL: the caller's frame)
  float *out_act[2];       // [64][H][W]
  const float *gin[2];     // error published by the next conv stage [64][H][W] (NULL if the head follows)
  const float *ge[2];      // error published by the head: one value per channel (already divided by H * W)
  float *eout[2];          // [c_in][H][W] (NULL for the first stage)
  float *delta;            // [64][H][W]; for a layer that is not the last of its stage it holds z between the layer's
                           // forward pass and the backward pass of the layer behind it, which turns it into delta
  float *dwp;              // [n_wt][64][c_in * 9]
  float *dbp;              // [n_ft][64]
  int n_ft, n_wt;
  int fuse_delta;          // 1: last layer of its stage, the error it needs is one tick old: delta in the forward epilogue
  float *pred_delta;       // not the first of its stage: the layer in front of it (its z, then its delta) ...
  float *pred_dbp;         // ... and that layer's bias-gradient partials; NULL: publish the input-error (eout)
  int pred_act;
  // Residual connections (Sec. V-C): the target layer adds the source's output of d ticks ago (d = stage boundaries
  // crossed) after its own activation, and hands the gradient at its output back to the source over the same delay.
  // Both travel through rings of d + 1 frames [co_pad][H][W], slot = tick mod (d + 1); the rings belong to the target.
  const float *skip_in;    // this layer is a target: ring of the skipped map ...
  float *serr_out;         // ... and ring its output-gradient is written to
  int skip_n, skip_d;      // slots, delay
  float *skip_out;         // this layer is a source: ring its output is also written to ...
  const float *serr_in;    // ... and ring the gradient comes back over
  int src_n, src_d;
};

struct CvHead {
  float *W, *b;            // [out][c], [out]
  float *mW, *vW, *mb, *vb;   // Adam moments (NULL under plain SGD)
  int c, out, hw;
  const float *in_act[2];  // last conv stage's published output [c][hw]
  float *gapv;             // [c] channel means of this tick's input
  float *ge[2];            // [c] published error
};

struct CvTile {
  int stage, a, b, kind;   // conv: a = first row, b = block of 64 output channels.  kind 1 (FWD launch): pooling of channel a.
                           // kind 2 (BWD launch): the head.  wgrad: a = row band, b = block of 64 input channels,
                           // kind = block of 64 output channels
};

struct CvNet {
  const CvStage *stages;
  const CvTile *tiles_f, *tiles_b, *tiles_w;
  CvHead head;
  int n_conv, loss, adam;
  float lr, beta1, beta2, eps;
};

struct CvTick {
  const float *x;
  const void *tgt;
  float *out;
  float *loss1;
  int cur, learn;
  int tick;                 // tick number modulo a common multiple of all ring lengths (slots of the residual rings)
  float adam_c1, adam_c2;   // lr / (1 - beta1^n), 1 / sqrt(1 - beta2^n)
};

enum { CV_FWD = 0, CV_BWD = 1 };

// one step of the update rule on one parameter: plain SGD, or Adam with its moments read and written in place
__device__ __forceinline__ float cv_step(const CvNet &net, float adam_c1, float adam_c2, float w, float g, float *m, float *v, size_t i) {
  if (!net.adam) return w - net.lr * g;
  const float mn = fmaf(net.beta1, ldg_f(m + i), (1.f - net.beta1) * g);
  const float vn = fmaf(net.beta2, ldg_f(v + i), (1.f - net.beta2) * g * g);
  stg_f(m + i, mn);
  stg_f(v + i, vn);
  return w - adam_c1 * mn / (sqrtf(vn) * adam_c2 + net.eps);
}

__device__ __forceinline__ f32x16_t mfma32(float a, float b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// ------------------------------------------------------------------------------------------------
// conv as implicit GEMM: out[64][tile of 256 pixels] = Wmat[64][c * 9] * patches[c * 9][256]
// four waves: wave w takes output channels 32 (w & 1) .. +32 and the four 32-pixel blocks 4 (w >> 1) .. +3
// ------------------------------------------------------------------------------------------------
// RES: some layer of the pipeline has a residual connection.  A template parameter because the ring handling in the
// epilogues costs every tile registers and instructions (250 instead of 182 registers in the forward kernel; the
// 150-layer workload ran 7 % slower for it) that a pipeline without residual connections need not pay.
template <int MODE, bool LEARN, int LW, bool RES>
__global__ __launch_bounds__(256, 2) void cv_conv_kernel(CvNet net, CvTick a) {
  // (aligned: behind a static LDS variable of the kernel the array would otherwise start at an odd word, and every 16-byte
  // access to it would be a misaligned one: the 8 x 4096 fp32 workload ran 8 % slower that way)
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const CvTile tl = MODE == CV_FWD ? net.tiles_f[blockIdx.x] : net.tiles_b[blockIdx.x];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, prev = a.cur ^ 1;

  if (MODE == CV_FWD && tl.kind == 1) {
    // pooling for the head: mean of channel tl.a of what the last conv stage published one tick earlier
    const CvHead hd = net.head;
    const float *src = (prev ? hd.in_act[1] : hd.in_act[0]) + (size_t)tl.a * hd.hw;
    // (eight requests at a time, at clamped addresses: one request per trip of a loop with a run-time bound is one memory
    // round trip after the other)
    float s = 0.f;
    for (int i0 = tid * 4; i0 < hd.hw; i0 += 8 * 1024) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = ldg_f4(src + min(i0 + u * 1024, hd.hw - 4));
#pragma unroll
      for (int u = 0; u < 8; ++u) s += i0 + u * 1024 < hd.hw ? (v[u].x + v[u].y) + (v[u].z + v[u].w) : 0.f;
    }
    s = block_sum<4>(s, lds);
    if (tid == 0) stg_f(hd.gapv + tl.a, s / (float)hd.hw);
    return;
  }
  if (MODE == CV_BWD && tl.kind == 2) {
    // the head stage: z = W mean + b, loss, delta, published error (with the old W), update
    const CvHead hd = net.head;
    float *v = lds, *z = lds + 1024, *dl = lds + 2048, *sm = lds + 3072;
    for (int i = tid; i < hd.c; i += 256) v[i] = ldg_f(hd.gapv + i);
    __syncthreads();
    for (int j = tid; j < hd.out; j += 256) {
      float acc = ldg_f(hd.b + j);
      for (int c = 0; c < hd.c; ++c) acc = fmaf(ldg_f(hd.W + (size_t)j * hd.c + c), v[c], acc);
      z[j] = acc;
      stg_f(a.out + j, acc);
    }
    __syncthreads();
    if (!LEARN) return;
    if (net.loss == PT_LOSS_CE) {
      float m = -INFINITY;
      for (int j = tid; j < hd.out; j += 256) m = fmaxf(m, z[j]);
      m = block_max<4>(m, sm);
      float s = 0.f;
      for (int j = tid; j < hd.out; j += 256) s += expf(z[j] - m);
      s = block_sum<4>(s, sm + 8);
      const int y = min(max(ldg_i(a.tgt), 0), hd.out - 1);
      for (int j = tid; j < hd.out; j += 256) dl[j] = a.learn ? expf(z[j] - m) / s - (j == y ? 1.f : 0.f) : 0.f;
      if (tid == 0) stg_f(a.loss1, a.learn ? -(z[y] - m - logf(s)) : 0.f);
    } else {
      float s = 0.f;
      for (int j = tid; j < hd.out; j += 256) {
        const float d = z[j] - ldg_f(static_cast<const float *>(a.tgt) + j);
        s = fmaf(d, d, s);
        dl[j] = a.learn ? 2.f * d / (float)hd.out : 0.f;
      }
      s = block_sum<4>(s, sm);
      if (tid == 0) stg_f(a.loss1, a.learn ? s / (float)hd.out : 0.f);
    }
    __syncthreads();
    float *ge = a.cur ? hd.ge[1] : hd.ge[0];
    for (int c = tid; c < hd.c; c += 256) {
      float e = 0.f;
      for (int j = 0; j < hd.out; ++j) e = fmaf(ldg_f(hd.W + (size_t)j * hd.c + c), dl[j], e);
      stg_f(ge + c, e / (float)hd.hw);
    }
    __syncthreads();   // every read of the old W is done
    for (int i = tid; i < hd.out * hd.c; i += 256) {
      const int j = i / hd.c, c = i % hd.c;
      stg_f(hd.W + i, cv_step(net, a.adam_c1, a.adam_c2, ldg_f(hd.W + i), dl[j] * v[c], hd.mW, hd.vW, i));
    }
    for (int j = tid; j < hd.out; j += 256)
      stg_f(hd.b + j, cv_step(net, a.adam_c1, a.adam_c2, ldg_f(hd.b + j), dl[j], hd.mb, hd.vb, j));
    return;
  }

  // everything the tile needs from the stage record, read once into registers.  The frame width is a template
  // parameter: every LDS offset below is then an immediate, and one address register serves all operand reads.
  constexpr int W = 1 << LW, TR = kCvPx >> LW, PWp = W + 8, PR = TR + 2, W4 = W >> 2;
  constexpr int kTotal4 = kCvCiCh * PR * W4, NQ = (kTotal4 + 255) / 256;   // 16-byte pieces per block of channels
  constexpr int kChunkElems = kCvCiCh * PR * PWp;
  const CvStage *sp = net.stages + tl.stage;
  const int H = sp->H, act = sp->act, c_in = sp->c_in, c_out = sp->c_out;
  const int ch0 = tl.b * kCvCo;                               // first output channel of this tile
  constexpr int ldw = kCvCo;                                  // row pitch of the tap-major weights of one channel block
  const int ldb = MODE == CV_FWD ? sp->co_pad : sp->ci_pad;   // row pitch of the bias-gradient partials
  const float *in_prev = prev ? sp->in_act[1] : sp->in_act[0];
  const float *gin = a.cur ? sp->gin[0] : sp->gin[1];
  const float *ge = a.cur ? sp->ge[0] : sp->ge[1];
  float *outp = MODE == CV_FWD ? (a.cur ? sp->out_act[1] : sp->out_act[0]) : (a.cur ? sp->eout[1] : sp->eout[0]);
  float *delta = sp->delta, *dbp = sp->dbp;
  const float *bias = sp->b;
  const int fuse_delta = sp->fuse_delta, pred_act = sp->pred_act;
  float *pred_delta = sp->pred_delta, *pred_dbp = sp->pred_dbp;
  // residual rings, at the slots of this tick: the layer whose output (FWD) or output-gradient (FWD with the delta in
  // its epilogue; BWD: the layer in front, whose delta this launch forms) is in hand
  const float *skip_in = nullptr, *serr_in = nullptr;
  float *skip_out = nullptr, *serr_out = nullptr;
  if constexpr (RES) {
    const CvStage *rp = MODE == CV_FWD ? sp : sp - 1;
    if (MODE == CV_FWD || pred_delta) {
      const size_t frame = (size_t)rp->co_pad * H * sp->W;
      const int t = a.tick;
      if (rp->skip_in) {
        if (MODE == CV_FWD) skip_in = rp->skip_in + (size_t)((t + rp->skip_n - rp->skip_d) % rp->skip_n) * frame;
        if (LEARN) serr_out = rp->serr_out + (size_t)(t % rp->skip_n) * frame;
      }
      if (rp->skip_out) {
        if (MODE == CV_FWD) skip_out = rp->skip_out + (size_t)(t % rp->src_n) * frame;
        if (LEARN) serr_in = rp->serr_in + (size_t)((t + rp->src_n - rp->src_d) % rp->src_n) * frame;
      }
    }
  }
  // FWD: input channels are the stage's inputs; BWD: the "input" is delta (64 channels), the output has c_in channels
  const float *src = MODE == CV_FWD ? (in_prev ? in_prev : a.x) : delta;
  // tap-major weights of this tile's block of 64 output channels: [k][64], k = (input channel) * 9 + tap
  const float *wT = MODE == CV_FWD ? sp->WT + (size_t)tl.b * (((c_in + 1) & ~1) * 9 * kCvCo)
                                   : sp->WBT + (size_t)tl.b * (sp->co_pad * 9 * kCvCo);
  const int cin = MODE == CV_FWD ? c_in : c_out;            // delta is zero beyond the real output channels
  const int n_out = MODE == CV_FWD ? c_out : c_in;            // real output channels of the product
  const int HW = H * W, y0 = tl.a;
  const int n_units = (cin + 1) >> 1;                         // a pair of input channels = 9 products of depth 2
  const int n_chunks = (cin + kCvCiCh - 1) / kCvCiCh;
  float *pbuf0 = lds, *pbuf1 = lds + kChunkElems;             // [kCvCiCh][PR][PWp], pixel x of a row at index x + 4
  const int half = lane >> 5, cb = wv & 1, pg = wv >> 1;

  // staging plan of this thread: NQ pieces of 16 bytes per block of channels
  int goff[NQ], loff[NQ], cq[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int i = tid + 256 * q, seg = i / W4, col4 = i % W4, c = seg / PR, row = seg % PR, yy = y0 - 1 + row;
    const bool ok = i < kTotal4 && yy >= 0 && yy < H;
    goff[q] = ok ? c * HW + yy * W + col4 * 4 : 0;
    loff[q] = (c * PR + row) * PWp + 4 + col4 * 4;
    cq[q] = ok ? c : 1024;                                    // rows outside the frame are staged as zeros
  }
  float4 xr[NQ];
  // unconditional loads from clamped addresses, zeroed afterwards: no branch between the requests
  auto fetch = [&](int c0) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const bool use = c0 + cq[q] < cin;
      const float4 v = ldg_f4(src + (use ? (size_t)c0 * HW + goff[q] : 0));
      xr[q] = use ? v : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto put = [&](float *buf) {
#pragma unroll
    for (int q = 0; q < NQ; ++q)
      if (tid + 256 * q < kTotal4) *reinterpret_cast<float4 *>(buf + loff[q]) = xr[q];
  };
  // the zero border left and right of every staged row (both buffers are one run of rows)
  for (int r = tid; r < 2 * kCvCiCh * PR; r += 256) {
    lds[r * PWp + 3] = 0.f;
    lds[r * PWp + W + 4] = 0.f;
  }
  // operand address of this lane: pixel (pg * 4) * 32 + l % 32 of the tile; the upper half-wave works on the
  // second channel of each pair.  Tap j of pixel block q of pair u is then at a compile-time distance.
  const int p0 = pg * 128 + (lane & 31);
  const int lbase = (p0 / W) * PWp + (p0 % W) + half * (PR * PWp) + 3;
  f32x16_t acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;

  // weights go from memory (cache-resident, shared by all tiles) straight into operand registers, one pair of
  // channels ahead of the products
  float av[9], avn[9];
  auto load_a = [&](float (&dst)[9], int unit) {
    const float *wp = wT + (size_t)(2 * min(unit, n_units - 1) + half) * (9 * ldw) + cb * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < 9; ++j) dst[j] = ldg_f(wp + j * ldw);
  };
  fetch(0);
  load_a(av, 0);
  put(pbuf0);
  __syncthreads();
  for (int ch = 0; ch < n_chunks; ++ch) {
    const float *pb = ((ch & 1) ? pbuf1 : pbuf0) + lbase;
    const bool more = ch + 1 < n_chunks;
    if (more) fetch((ch + 1) * kCvCiCh);                     // in flight while this block is multiplied
    const int nu = min(kCvCiCh / 2, n_units - ch * (kCvCiCh / 2));
#pragma unroll
    for (int u = 0; u < kCvCiCh / 2; ++u) {
      if (u < nu) {
        load_a(avn, ch * (kCvCiCh / 2) + u + 1);
#pragma unroll
        for (int jh = 0; jh < 9; jh += 3) {
          float bv[3][4];
#pragma unroll
          for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int pq = q * 32;                          // pixel distance of block q inside the wave's 128
              bv[j][q] = pb[(2 * u * PR + (jh + j) / 3) * PWp + (jh + j) % 3 + (pq / W) * PWp + (pq % W)];
            }
#pragma unroll
          for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = mfma32(av[jh + j], bv[j][q], acc[q]);
        }
#pragma unroll
        for (int j = 0; j < 9; ++j) av[j] = avn[j];
      }
    }
    if (more) {
      put((ch & 1) ? pbuf0 : pbuf1);                         // the other buffer: nobody reads it during this block
      __syncthreads();
    }
  }

  // epilogue: register r of lane l is output channel 32 cb + 8 (r / 4) + 4 (l / 32) + r % 4, pixel block column l % 32
  float dsum[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) dsum[r] = 0.f;
  float bz[16];
  if (MODE == CV_FWD) {
#pragma unroll
    for (int r = 0; r < 16; ++r) bz[r] = ldg_f(bias + ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3));
  }
  const bool to_pred = MODE == CV_BWD && pred_delta != nullptr;
  // FULL: all 64 channels of the block are real, no per-channel checks (they differ between the half-waves, so each
  // one is a divergent branch that also keeps the loads and stores of a pixel block from being issued together)
  auto epilogue = [&](auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int p = y0 * W + (pg * 4 + q) * 32 + (lane & 31);
      if (MODE == CV_FWD) {
        float gv[16];
        if (LEARN && fuse_delta) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int co = ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            const int cc = FULL ? co : min(co, n_out - 1);       // padding channels: clamped load, never stored
            gv[r] = gin ? ldg_f(gin + (size_t)cc * HW + p) : ldg_f(ge + cc);
          }
          if (serr_in) {      // the gradient that comes back over a residual connection starting at this output
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int co = ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
              gv[r] += ldg_f(serr_in + (size_t)(FULL ? co : min(co, n_out - 1)) * HW + p);
            }
          }
          if (serr_out) {     // o = phi(z) + skipped map: the gradient at o goes to the skipped map unchanged
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int co = ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
              if (FULL || co < n_out) stg_f(serr_out + (size_t)co * HW + p, gv[r]);
            }
          }
        }
        float sk[16];
        if (skip_in) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int co = ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            sk[r] = ldg_f(skip_in + (size_t)(FULL ? co : min(co, n_out - 1)) * HW + p);
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int co = ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          if (!FULL && co >= n_out) continue;                    // padding channels are zero everywhere and stay so
          const float z = acc[q][r] + bz[r];
          const float o = skip_in ? act_fwd(act, z) + sk[r] : act_fwd(act, z);
          stg_f(outp + (size_t)co * HW + p, o);
          if (skip_out) stg_f(skip_out + (size_t)co * HW + p, o);
          if (LEARN) {
            if (fuse_delta) {
              const float d = gv[r] * act_der(act, z);
              stg_f(delta + (size_t)co * HW + p, d);
              dsum[r] += d;
            } else {
              stg_f(delta + (size_t)co * HW + p, z);             // kept for the backward pass of the layer behind
            }
          }
        }
      } else if (to_pred) {
        // exact back-propagation inside a stage (Eq. 5): the input-error of this layer times phi'(z) of the layer
        // in front is that layer's delta; its z waits in its delta buffer
        float zv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int co = ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          zv[r] = ldg_f(pred_delta + (size_t)(FULL ? co : min(co, n_out - 1)) * HW + p);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int co = ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          if (!FULL && co >= n_out) continue;
          float gq = acc[q][r];                                  // gradient at the output of the layer in front
          if (serr_in) gq += ldg_f(serr_in + (size_t)co * HW + p);
          if (serr_out) stg_f(serr_out + (size_t)co * HW + p, gq);
          const float d = gq * act_der(pred_act, zv[r]);
          stg_f(pred_delta + (size_t)co * HW + p, d);
          dsum[r] += d;
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int co = ch0 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          if (FULL || co < n_out) stg_f(outp + (size_t)co * HW + p, acc[q][r]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);   // one pixel block at a time: the loads of all four at once need too many registers
    }
  };
  if (ch0 + kCvCo <= n_out) epilogue(std::true_type{});
  else epilogue(std::false_type{});
  if ((MODE == CV_FWD && LEARN && fuse_delta) || to_pred) {
    // bias-gradient partial of this tile: sum of delta over its 256 pixels, per channel
    float *dbo = MODE == CV_FWD ? dbp : pred_dbp;
    __syncthreads();
    float *red = lds;   // [2 pixel groups][64]
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float s = dsum[r];
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);   // over the 32 lanes that share the channel
      if ((lane & 31) == 0) red[pg * 64 + cb * 32 + (r >> 2) * 8 + half * 4 + (r & 3)] = s;
    }
    __syncthreads();
    if (tid < 64) stg_f(dbo + (size_t)(y0 / TR) * ldb + ch0 + tid, red[tid] + red[64 + tid]);
  }
}

// ------------------------------------------------------------------------------------------------
// weight gradient (Eq. 9 for a conv stage): dW[64][c_in * 9] partial over a band of rows, as
// delta[64][pixels] * patches[pixels][c_in * 9] with v_mfma_f32_16x16x4f32 (A holds A[l % 16][l / 16], B holds
// B[l / 16][l % 16], C register j holds C[4 (l / 16) + j][l % 16]).
// Eight independent waves per tile: wave = (block of 16 input channels, half of the output channels).  A wave
// keeps its 32 x 144 sums in registers, reads delta straight from memory (each lane 16 bytes of its own output
// channel: the four pixels are fed to four consecutive products) and stages its 16 input channels, three rows as
// a ring, in its private part of LDS: no work-group barrier anywhere.
// XC = columns staged at a time (the frame width if that is smaller).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ f32x4_t mfma16f(float a, float b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

template <int XC>
__global__ __launch_bounds__(512) void cv_wgrad_kernel(CvNet net, CvTick a) {
  // (aligned: behind a static LDS variable of the kernel the array would otherwise start at an odd word, and every 16-byte
  // access to it would be a misaligned one: the 8 x 4096 fp32 workload ran 8 % slower that way)
  extern __shared__ __attribute__((aligned(16))) float lds[];
  constexpr int kPitch = XC + 12, XC4 = XC / 4;             // pixel x of a staged row at index x - xc0 + 4
  constexpr int kSlot = kCvWgCi * kPitch, NQ = (kCvWgCi * XC4 + 63) / 64;
  const CvTile tl = net.tiles_w[blockIdx.x];
  const CvStage *sp = net.stages + tl.stage;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, li = lane & 15, g = lane >> 4, prev = a.cur ^ 1;
  const int H = sp->H, W = sp->W, HW = H * W, c_in = sp->c_in, ktot = c_in * 9;
  const float *in_prev = prev ? sp->in_act[1] : sp->in_act[0];
  const float *src = in_prev ? in_prev : a.x;
  const float *delta = sp->delta;
  float *dwp = sp->dwp;
  const int cbk = wv & 3, mh = wv >> 2, ci0 = tl.b * kCvCo + cbk * kCvWgCi, co0 = tl.kind * kCvCo + mh * 32;
  const int nc = min(kCvWgCi, c_in - ci0);
  if (nc <= 0 || co0 >= sp->c_out) return;                   // no barrier below: a wave without channels just leaves
  const int yb = tl.a * kCvWgRows, ye = min(yb + kCvWgRows, H);
  float *ring = lds + wv * (3 * kSlot);                      // [slot][channel][kPitch]

  // column nb * 16 + li of the product is (channel, tap) = (k / 9, k % 9) of this wave's channel block
  int cst[9];
  unsigned kyp = 0;
#pragma unroll
  for (int nb = 0; nb < 9; ++nb) {
    const int k = nb * 16 + li, cil = k / 9, tap = k - 9 * cil, ky = tap / 3, kx = tap - 3 * ky;
    cst[nb] = cil * kPitch + 3 + kx + 4 * g;
    kyp |= (unsigned)ky << (2 * nb);
  }
  f32x4_t acc[2][9];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int nb = 0; nb < 9; ++nb) acc[mb][nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // staging of one image row of the 16 channels: 16-byte pieces for the inside, one scalar per channel and side
  float4 pre[NQ];
  float preh;
  const int cih = (lane >> 1) & 15, hside = lane & 1;
  auto fetch_row = [&](int r, int xc0) {
    const bool rok = r >= 0 && r < H;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int idx = lane + 64 * q, ci = idx / XC4, col4 = idx % XC4;
      const bool use = rok && ci < nc;
      const float4 v = ldg_f4(src + (use ? (size_t)(ci0 + ci) * HW + r * W + xc0 + col4 * 4 : 0));
      pre[q] = use ? v : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const int x = hside ? xc0 + XC : xc0 - 1;
    const bool use = rok && cih < nc && x >= 0 && x < W;
    const float v = ldg_f(src + (use ? (size_t)(ci0 + cih) * HW + r * W + x : 0));
    preh = use ? v : 0.f;
  };
  auto put_row = [&](int slot) {
    float *rp = ring + slot * kSlot;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int idx = lane + 64 * q, ci = idx / XC4, col4 = idx % XC4;
      if (ci < kCvWgCi) *reinterpret_cast<float4 *>(rp + ci * kPitch + 4 + col4 * 4) = pre[q];
    }
    if (lane < 32) rp[cih * kPitch + (hside ? 4 + XC : 3)] = preh;
  };

  for (int xc0 = 0; xc0 < W; xc0 += XC) {
    for (int r = yb - 1; r <= yb + 1; ++r) {
      fetch_row(r, xc0);
      put_row((r + 3) % 3);
    }
    for (int y = yb; y < ye; ++y) {
      const bool more = y + 1 < ye;
      if (more) fetch_row(y + 2, xc0);                       // in flight while row y is multiplied
      const int s0 = ((y + 2) % 3) * kSlot, s1 = (y % 3) * kSlot, s2 = ((y + 1) % 3) * kSlot;   // rows y - 1, y, y + 1
      const float *rp[9];
#pragma unroll
      for (int nb = 0; nb < 9; ++nb) {
        const unsigned ky = (kyp >> (2 * nb)) & 3u;
        rp[nb] = ring + cst[nb] + (ky == 0 ? s0 : ky == 1 ? s1 : s2);
      }
      const float *dp = delta + (size_t)(co0 + li) * HW + y * W + xc0 + 4 * g;
      float4 a4[2], a4n[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) a4[mb] = ldg_f4(dp + (size_t)mb * 16 * HW);
#pragma unroll
      for (int m = 0; m < XC; m += 16) {
        if (m + 16 < XC) {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb) a4n[mb] = ldg_f4(dp + (size_t)mb * 16 * HW + m + 16);
        }
#pragma unroll
        for (int step = 0; step < 4; ++step) {
          float b[9];
#pragma unroll
          for (int nb = 0; nb < 9; ++nb) b[nb] = rp[nb][m + step];
#pragma unroll
          for (int mb = 0; mb < 2; ++mb) {
            const float av = step == 0 ? a4[mb].x : step == 1 ? a4[mb].y : step == 2 ? a4[mb].z : a4[mb].w;
#pragma unroll
            for (int nb = 0; nb < 9; ++nb) acc[mb][nb] = mfma16f(av, b[nb], acc[mb][nb]);
          }
        }
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) a4[mb] = a4n[mb];
      }
      if (more) put_row((y + 2) % 3);                        // over row y - 1, which nobody needs any more
    }
  }

  float *dst = dwp + (size_t)tl.a * sp->co_pad * ktot + (size_t)co0 * ktot + ci0 * 9;
#pragma unroll
  for (int nb = 0; nb < 9; ++nb) {
    const int kc = nb * 16 + li;
    if (kc < nc * 9) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) stg_f(dst + (size_t)(mb * 16 + 4 * g + j) * ktot + kc, acc[mb][nb][j]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// update: one thread per weight (and per bias) of every conv stage; keeps the three weight layouts in step
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cv_update_kernel(CvNet net, int total, float adam_c1, float adam_c2) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  for (int h = 0; h < net.n_conv; ++h) {
    const CvStage *sp = net.stages + h;
    const int ktot = sp->c_in * 9, cop = sp->co_pad, nw = cop * ktot;
    if (i < nw + cop) {
      if (i < nw) {
        // partials of sixteen bands are requested together (clamped, then masked): one memory latency per sixteen
        float g = 0.f;
        const int n_wt = sp->n_wt;
        const float *dp = sp->dwp + i;
        for (int p = 0; p < n_wt; p += 16) {
          float v[16];
#pragma unroll
          for (int u = 0; u < 16; ++u) v[u] = ldg_f(dp + (size_t)min(p + u, n_wt - 1) * nw);
#pragma unroll
          for (int u = 0; u < 16; ++u) g += p + u < n_wt ? v[u] : 0.f;
        }
        const float w = cv_step(net, adam_c1, adam_c2, ldg_f(sp->Wg + i), g, sp->mW, sp->vW, i);
        stg_f(sp->Wg + i, w);
        const int co = i / ktot, k = i % ktot, ci = k / 9, tap = k % 9;
        stg_f(sp->WT + ((size_t)(co / kCvCo) * (((sp->c_in + 1) & ~1) * 9) + k) * kCvCo + co % kCvCo, w);
        stg_f(sp->WBT + ((size_t)(ci / kCvCo) * (cop * 9) + co * 9 + (8 - tap)) * kCvCo + ci % kCvCo, w);
      } else {
        const int co = i - nw;
        // (requested sixteen at a time like the weight partials: one request per trip would be n_ft memory round trips
        // in a row, and these few threads set the length of the launch)
        float g = 0.f;
        const int n_ft = sp->n_ft;
        const float *dp = sp->dbp + co;
        for (int p = 0; p < n_ft; p += 16) {
          float v[16];
#pragma unroll
          for (int u = 0; u < 16; ++u) v[u] = ldg_f(dp + (size_t)min(p + u, n_ft - 1) * cop);
#pragma unroll
          for (int u = 0; u < 16; ++u) g += p + u < n_ft ? v[u] : 0.f;
        }
        stg_f(sp->b + co, cv_step(net, adam_c1, adam_c2, ldg_f(sp->b + co), g, sp->mb, sp->vb, co));
      }
      return;
    }
    i -= nw + cop;
  }
}
