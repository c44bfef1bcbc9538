/*
 * CPU oracle for pipelined online learning over a stream (PARTIME).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * method computes, written from the paper: Sec. III (Eq. 1-11) and Algorithm 1.
 * It shares no code, header, table or helper with the HIP library, and nothing
 * in the product path may include, link or call it.
 *
 * What one tick does (Algorithm 1; Eq. 6, Eq. 9, Eq. 11), for every stage h:
 *   - the stage input is x(t) for the first stage, otherwise what stage h-1
 *     wrote during the previous tick (the "stable" area of Algorithm 1);
 *   - the stage runs its layers forward with its current weights (Eq. 6);
 *   - the last stage emits the network output and the loss gradient
 *     g_D = dL/do (text under Eq. 10); any other stage publishes its output for
 *     the next tick and takes as g_h the input-gradient that stage h+1 produced
 *     during the previous tick (Algorithm 1 "copy gradients from the next
 *     stage"; Eq. 11);
 *   - the stage back-propagates g_h through its own layers at this tick's
 *     input and weights (Eq. 5, Eq. 9), publishes its input-gradient (computed
 *     with the weights as they were before this tick's update) and then
 *     updates its weights at once (Algorithm 1, last two steps).
 * No stage reads anything another stage writes during the same tick, so the
 * order in which stages are visited inside a tick cannot matter; the caller
 * may pass any order to prove it.
 *
 * Readings where the paper is silent (each one is listed in the design notes):
 *   - buffers start at zero and the loss gradient is held at zero until a
 *     real sample and its target have both reached the last stage
 *     (tick < max(D-1, k));
 *   - the target consumed at tick t is the one supplied at tick t-k;
 *   - MSE = mean_i (o_i-y_i)^2, CE = -log softmax(o)[y]; mean over streams;
 *   - GELU is the exact erf form; ReLU'(0) = 0.
 *
 * Arithmetic: weights and the inter-tick vectors are stored as fp32 (or as
 * fp32 values rounded to bf16, round-to-nearest-even); everything inside a
 * tick is fp64.  Optionally (the multi-stream bf16 configuration, whose stage
 * products are bf16 x bf16 matrix contractions) whatever enters a product -
 * a layer's input and a layer's delta - is first rounded to bf16.  Parity unpinned: the choice, for the Jacobian of stage h+1 in
 * Eq. 11, of stage h+1's own input of the previous tick (what Algorithm 1 can
 * compute locally) over the literal evaluation point printed in Eq. 11.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { K_DENSE = 0, K_CONV3 = 1, K_GAPDENSE = 2 };
enum { A_ID = 0, A_RELU = 1, A_GELU = 2 };
enum { L_NONE = 0, L_MSE = 1, L_CE = 2 };

typedef struct {
  int kind, act, in_dim, out_dim, c_in, c_out, hh, ww;
  long in_size, out_size, n_w, n_b;
  float *W, *b;     /* stored values (already in storage precision)       */
  double *dW, *db;  /* gradient of the last tick, mean over streams        */
  float *mW, *vW, *mb, *vb; /* Adam moments (fp32 storage), NULL under plain SGD */
  /* skip connection (Sec. V-C): the output of layer skip_src (-1: none) is added to this layer's output.  Between
   * stages it travels like everything else, one stage per tick, through identity lanes; so does its gradient. */
  int skip_src, skip_dst;   /* skip_dst: the layer that takes this layer's output as its skip (-1: none)          */
  double *o;                /* [S][out_size] output of this tick (after the skip was added)                       */
  double *gskip;            /* [S][out_size] gradient that came back over a skip inside the stage, this tick      */
  float **lane_a[2];        /* owned by the target layer: lane_a[half][stage], value leaving `stage` forward      */
  float **lane_e[2];        /* owned by the target layer: lane_e[half][stage], gradient leaving `stage` backward  */
  double *u;        /* [S][in_size]  layer input of this tick              */
  double *z;        /* [S][out_size] pre-activation of this tick           */
} layer_t;

typedef struct {
  int n_layers, depth, S, w_bf16, loss, k;
  int op_bf16;                 /* round the operands of every product (layer inputs, deltas) to bf16 */
  double lr;
  int adam;                    /* 0: plain SGD, 1: Adam (Sec. V-D trains with it) */
  double beta1, beta2, eps;
  layer_t *layers;
  int *first, *count;          /* stage -> first layer, layer count        */
  int *stage_of;               /* layer -> stage                            */
  float **act[2];              /* act[half][stage]  [S][stage out size]    */
  float **err[2];              /* err[half][stage]  [S][stage in size]     */
  long tick;
  double kink_margin;          /* diagnostic only: smallest |z| at which a ReLU derivative was taken with g != 0 */
  /* test diagnostic, no part of the method (see oracle_set_kink_band) */
  double band_eps;             /* half-width of the band around z = 0, relative to sum |w u| + |b|; 0 = no band  */
  int band_side;               /* 0: ReLU'(z) = [z > 0] everywhere; +1 / -1: inside the band the derivative is 1 / 0 */
  long n_events, cap_events;   /* ReLU units found inside the band with a non-zero error signal                  */
  long *events;                /* triples (tick, layer, stream * out_size + unit), the first cap_events of them  */
  long tgt_elems;              /* elements of one tick's target            */
  unsigned char *tgt_hist;     /* last k targets, oldest first             */
  double *g, *g2;              /* scratch [S][max size]                    */
  long max_size;
} net_t;

/* ---- storage rounding --------------------------------------------------- */

/* fp32 -> bf16 -> fp32, round to nearest, ties to even (IEEE 754 rule applied
 * to the upper 16 bits).  NaN keeps a quiet payload. */
float oracle_round_bf16(float v) {
  uint32_t u;
  memcpy(&u, &v, 4);
  if ((u & 0x7f800000u) == 0x7f800000u && (u & 0x007fffffu)) {
    u = (u | 0x00400000u) & 0xffff0000u;
  } else {
    uint32_t lower = u & 0xffffu, keep = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (keep & 1u))) keep += 1u;
    u = keep << 16;
  }
  memcpy(&v, &u, 4);
  return v;
}

/* operand rounding of the multi-stream bf16 configuration: what enters a matrix product is bf16 */
static double opr(const net_t *n, double v) { return n->op_bf16 ? (double)oracle_round_bf16((float)v) : v; }

static float store_w(const net_t *n, double v) {
  float f = (float)v;
  return n->w_bf16 ? oracle_round_bf16(f) : f;
}

/* ---- activations --------------------------------------------------------- */

static double phi(int act, double z) {
  if (act == A_RELU) return z > 0.0 ? z : 0.0;
  if (act == A_GELU) return 0.5 * z * (1.0 + erf(z * 0.70710678118654752440));
  return z;
}
static double dphi(int act, double z) {
  if (act == A_RELU) return z > 0.0 ? 1.0 : 0.0;
  if (act == A_GELU) {
    double cdf = 0.5 * (1.0 + erf(z * 0.70710678118654752440));
    double pdf = exp(-0.5 * z * z) * 0.3989422804014326779; /* 1/sqrt(2 pi) */
    return cdf + z * pdf;
  }
  return 1.0;
}


/* ---- one layer: forward, input-gradient, weight-gradient ---------------- */

static void layer_forward(const layer_t *l, const double *u, double *z) {
  if (l->kind == K_DENSE) {
#pragma omp parallel for schedule(static)
    for (long r = 0; r < l->out_dim; ++r) {
      const float *w = l->W + r * (long)l->in_dim;
      double acc = 0.0;
      for (long c = 0; c < l->in_dim; ++c) acc += (double)w[c] * u[c];
      z[r] = acc + (double)l->b[r];
    }
  } else if (l->kind == K_CONV3) {
    const int H = l->hh, Wd = l->ww;
#pragma omp parallel for schedule(static)
    for (int co = 0; co < l->c_out; ++co)
      for (int y = 0; y < H; ++y)
        for (int x = 0; x < Wd; ++x) {
          double acc = 0.0;
          for (int ci = 0; ci < l->c_in; ++ci)
            for (int ky = 0; ky < 3; ++ky)
              for (int kx = 0; kx < 3; ++kx) {
                int yy = y + ky - 1, xx = x + kx - 1;
                if (yy < 0 || yy >= H || xx < 0 || xx >= Wd) continue;
                acc += (double)l->W[((co * (long)l->c_in + ci) * 3 + ky) * 3 + kx] *
                       u[(ci * (long)H + yy) * Wd + xx];
              }
          z[(co * (long)H + y) * Wd + x] = acc + (double)l->b[co];
        }
  } else { /* global average pool over H x W, then dense c_in -> out_dim */
    const long HW = (long)l->hh * l->ww;
    for (long r = 0; r < l->out_dim; ++r) {
      double acc = 0.0;
      for (int c = 0; c < l->c_in; ++c) {
        double m = 0.0;
        for (long p = 0; p < HW; ++p) m += u[c * HW + p];
        acc += (double)l->W[r * (long)l->c_in + c] * (m / (double)HW);
      }
      z[r] = acc + (double)l->b[r];
    }
  }
}

/* gin = (d z / d u)^T delta, with the layer's current (not yet updated) W */
static void layer_input_grad(const layer_t *l, const double *delta, double *gin) {
  if (l->kind == K_DENSE) {
    const long N = l->in_dim;
#pragma omp parallel for schedule(static)
    for (long c0 = 0; c0 < N; c0 += 256) {
      long c1 = c0 + 256 < N ? c0 + 256 : N;
      for (long c = c0; c < c1; ++c) gin[c] = 0.0;
      for (long r = 0; r < l->out_dim; ++r) {
        const float *w = l->W + r * N;
        const double d = delta[r];
        for (long c = c0; c < c1; ++c) gin[c] += d * (double)w[c];
      }
    }
  } else if (l->kind == K_CONV3) {
    const int H = l->hh, Wd = l->ww;
#pragma omp parallel for schedule(static)
    for (int ci = 0; ci < l->c_in; ++ci)
      for (int yy = 0; yy < H; ++yy)
        for (int xx = 0; xx < Wd; ++xx) {
          double acc = 0.0;
          for (int co = 0; co < l->c_out; ++co)
            for (int ky = 0; ky < 3; ++ky)
              for (int kx = 0; kx < 3; ++kx) {
                int y = yy - ky + 1, x = xx - kx + 1; /* z[y][x] touched u[yy][xx] */
                if (y < 0 || y >= H || x < 0 || x >= Wd) continue;
                acc += (double)l->W[((co * (long)l->c_in + ci) * 3 + ky) * 3 + kx] *
                       delta[(co * (long)H + y) * Wd + x];
              }
          gin[(ci * (long)H + yy) * Wd + xx] = acc;
        }
  } else {
    const long HW = (long)l->hh * l->ww;
    for (int c = 0; c < l->c_in; ++c) {
      double acc = 0.0;
      for (long r = 0; r < l->out_dim; ++r)
        acc += delta[r] * (double)l->W[r * (long)l->c_in + c];
      for (long p = 0; p < HW; ++p) gin[c * HW + p] = acc / (double)HW;
    }
  }
}

/* dW += scale * (d z / d W)^T delta ; db += scale * delta-sum */
static void layer_weight_grad(const layer_t *l, const double *u, const double *delta,
                              double scale, double *dW, double *db) {
  if (l->kind == K_DENSE) {
#pragma omp parallel for schedule(static)
    for (long r = 0; r < l->out_dim; ++r) {
      double *g = dW + r * (long)l->in_dim;
      const double d = scale * delta[r];
      for (long c = 0; c < l->in_dim; ++c) g[c] += d * u[c];
      db[r] += d;
    }
  } else if (l->kind == K_CONV3) {
    const int H = l->hh, Wd = l->ww;
#pragma omp parallel for schedule(static)
    for (int co = 0; co < l->c_out; ++co) {
      for (int ci = 0; ci < l->c_in; ++ci)
        for (int ky = 0; ky < 3; ++ky)
          for (int kx = 0; kx < 3; ++kx) {
            double acc = 0.0;
            for (int y = 0; y < H; ++y)
              for (int x = 0; x < Wd; ++x) {
                int yy = y + ky - 1, xx = x + kx - 1;
                if (yy < 0 || yy >= H || xx < 0 || xx >= Wd) continue;
                acc += delta[(co * (long)H + y) * Wd + x] * u[(ci * (long)H + yy) * Wd + xx];
              }
            dW[((co * (long)l->c_in + ci) * 3 + ky) * 3 + kx] += scale * acc;
          }
      double s = 0.0;
      for (long p = 0; p < (long)H * Wd; ++p) s += delta[co * (long)H * Wd + p];
      db[co] += scale * s;
    }
  } else {
    const long HW = (long)l->hh * l->ww;
    for (long r = 0; r < l->out_dim; ++r) {
      for (int c = 0; c < l->c_in; ++c) {
        double m = 0.0;
        for (long p = 0; p < HW; ++p) m += u[c * HW + p];
        dW[r * (long)l->c_in + c] += scale * delta[r] * (m / (double)HW);
      }
      db[r] += scale * delta[r];
    }
  }
}

/* ---- test band around z = 0 (see oracle_set_kink_band): how large the terms of one unit's sum are ---------- */

/* sum_i |w_i u_i| + |b| of output unit r (for stream input u): the scale the rounding error of any way of summing
 * z_r = sum_i w_i u_i + b is proportional to */
static double unit_abs_sum(const layer_t *l, const double *u, long r) {
  double acc = 0.0;
  if (l->kind == K_DENSE) {
    const float *w = l->W + r * (long)l->in_dim;
    for (long c = 0; c < l->in_dim; ++c) acc += fabs((double)w[c] * u[c]);
    return acc + fabs((double)l->b[r]);
  }
  if (l->kind == K_CONV3) {
    const int H = l->hh, Wd = l->ww;
    const int co = (int)(r / ((long)H * Wd)), y = (int)((r / Wd) % H), x = (int)(r % Wd);
    for (int ci = 0; ci < l->c_in; ++ci)
      for (int ky = 0; ky < 3; ++ky)
        for (int kx = 0; kx < 3; ++kx) {
          int yy = y + ky - 1, xx = x + kx - 1;
          if (yy < 0 || yy >= H || xx < 0 || xx >= Wd) continue;
          acc += fabs((double)l->W[((co * (long)l->c_in + ci) * 3 + ky) * 3 + kx] * u[(ci * (long)H + yy) * Wd + xx]);
        }
    return acc + fabs((double)l->b[co]);
  }
  const long HW = (long)l->hh * l->ww;
  for (int c = 0; c < l->c_in; ++c) {
    double m = 0.0;
    for (long p = 0; p < HW; ++p) m += u[c * HW + p];
    acc += fabs((double)l->W[r * (long)l->c_in + c] * (m / (double)HW));
  }
  return acc + fabs((double)l->b[r]);
}

/* an upper bound of unit_abs_sum over all units of the layer (cheap: used to skip the units far from 0) */
static double layer_abs_bound(const layer_t *l, const double *u) {
  double mw = 0.0, mb = 0.0, su = 0.0, mu = 0.0;
  for (long i = 0; i < l->n_w; ++i) { double a = fabs((double)l->W[i]); if (a > mw) mw = a; }
  for (long i = 0; i < l->n_b; ++i) { double a = fabs((double)l->b[i]); if (a > mb) mb = a; }
  for (long i = 0; i < l->in_size; ++i) { double a = fabs(u[i]); su += a; if (a > mu) mu = a; }
  if (l->kind == K_DENSE) return mw * su + mb;
  if (l->kind == K_CONV3) return mw * 9.0 * l->c_in * mu + mb;
  return mw * l->c_in * mu + mb;
}

/* ---- loss heads (text under Eq. 10: g_D = dL/do at this tick's output) -- */

static double loss_and_grad(const net_t *n, const double *o, const void *target, long s,
                            long N, double *g) {
  if (n->loss == L_MSE) {
    const float *y = (const float *)target + s * N;
    double acc = 0.0;
    for (long i = 0; i < N; ++i) {
      double d = o[i] - (double)y[i];
      acc += d * d;
      g[i] = 2.0 * d / (double)N;
    }
    return acc / (double)N;
  }
  /* cross-entropy of softmax(o) against class id y */
  const int y = ((const int32_t *)target)[s];
  double m = o[0];
  for (long i = 1; i < N; ++i) m = o[i] > m ? o[i] : m;
  double sum = 0.0;
  for (long i = 0; i < N; ++i) sum += exp(o[i] - m);
  for (long i = 0; i < N; ++i) g[i] = exp(o[i] - m) / sum - (i == y ? 1.0 : 0.0);
  return -(o[y] - m - log(sum));
}

/* ---- construction -------------------------------------------------------- */

static long stage_in(const net_t *n, int h) { return n->layers[n->first[h]].in_size; }
static long stage_out(const net_t *n, int h) {
  return n->layers[n->first[h] + n->count[h] - 1].out_size;
}

/* desc: 9 ints per layer: kind, act, in_dim, out_dim, c_in, c_out, h, w, skip_src */
void *oracle_create(int n_layers, const int *desc, int depth, const int *balance, int S,
                    int w_bf16, int loss, float lr, int k) {
  net_t *n = (net_t *)calloc(1, sizeof(net_t));
  if (!n) return NULL;
  n->kink_margin = 1e300;
  n->n_layers = n_layers; n->depth = depth; n->S = S; n->w_bf16 = w_bf16;
  n->loss = loss; n->lr = (double)lr; n->k = k;
  n->layers = (layer_t *)calloc(n_layers, sizeof(layer_t));
  long mx = 0;
  for (int i = 0; i < n_layers; ++i) {
    layer_t *l = &n->layers[i];
    const int *d = desc + 9 * i;
    l->kind = d[0]; l->act = d[1]; l->in_dim = d[2]; l->out_dim = d[3];
    l->c_in = d[4]; l->c_out = d[5]; l->hh = d[6]; l->ww = d[7]; l->skip_src = d[8]; l->skip_dst = -1;
    if (l->kind == K_DENSE) {
      l->in_size = l->in_dim; l->out_size = l->out_dim;
      l->n_w = (long)l->in_dim * l->out_dim; l->n_b = l->out_dim;
    } else if (l->kind == K_CONV3) {
      l->in_size = (long)l->c_in * l->hh * l->ww; l->out_size = (long)l->c_out * l->hh * l->ww;
      l->n_w = (long)l->c_out * l->c_in * 9; l->n_b = l->c_out;
    } else {
      l->in_size = (long)l->c_in * l->hh * l->ww; l->out_size = l->out_dim;
      l->n_w = (long)l->out_dim * l->c_in; l->n_b = l->out_dim;
    }
    l->W = (float *)calloc(l->n_w, sizeof(float));
    l->b = (float *)calloc(l->n_b, sizeof(float));
    l->dW = (double *)calloc(l->n_w, sizeof(double));
    l->db = (double *)calloc(l->n_b, sizeof(double));
    l->u = (double *)calloc((long)S * l->in_size, sizeof(double));
    l->z = (double *)calloc((long)S * l->out_size, sizeof(double));
    l->o = (double *)calloc((long)S * l->out_size, sizeof(double));
    l->gskip = (double *)calloc((long)S * l->out_size, sizeof(double));
    if (l->in_size > mx) mx = l->in_size;
    if (l->out_size > mx) mx = l->out_size;
  }
  n->max_size = mx;
  n->g = (double *)calloc((long)S * mx, sizeof(double));
  n->g2 = (double *)calloc((long)S * mx, sizeof(double));
  n->first = (int *)calloc(depth, sizeof(int));
  n->count = (int *)calloc(depth, sizeof(int));
  int at = 0;
  for (int h = 0; h < depth; ++h) { n->first[h] = at; n->count[h] = balance[h]; at += balance[h]; }
  for (int p = 0; p < 2; ++p) {
    n->act[p] = (float **)calloc(depth, sizeof(float *));
    n->err[p] = (float **)calloc(depth, sizeof(float *));
    for (int h = 0; h < depth; ++h) {
      n->act[p][h] = (float *)calloc((long)S * stage_out(n, h), sizeof(float));
      n->err[p][h] = (float *)calloc((long)S * stage_in(n, h), sizeof(float));
    }
  }
  /* identity lanes of the skips that cross stage boundaries */
  n->stage_of = (int *)calloc(n_layers, sizeof(int));
  for (int h = 0; h < depth; ++h)
    for (int j = 0; j < n->count[h]; ++j) n->stage_of[n->first[h] + j] = h;
  for (int i = 0; i < n_layers; ++i) {
    layer_t *l = &n->layers[i];
    if (l->skip_src < 0) continue;
    n->layers[l->skip_src].skip_dst = i;
    for (int p = 0; p < 2; ++p) {
      l->lane_a[p] = (float **)calloc(depth, sizeof(float *));
      l->lane_e[p] = (float **)calloc(depth, sizeof(float *));
      for (int h = 0; h < depth; ++h) {
        l->lane_a[p][h] = (float *)calloc((long)S * l->out_size, sizeof(float));
        l->lane_e[p][h] = (float *)calloc((long)S * l->out_size, sizeof(float));
      }
    }
  }
  long N = stage_out(n, depth - 1);
  n->tgt_elems = loss == L_MSE ? (long)S * N : (long)S; /* 4-byte elements either way */
  n->tgt_hist = (unsigned char *)calloc((size_t)(k > 0 ? k : 1) * n->tgt_elems, 4);
  return n;
}

void oracle_destroy(void *p) {
  net_t *n = (net_t *)p;
  for (int i = 0; i < n->n_layers; ++i) {
    layer_t *l = &n->layers[i];
    free(l->W); free(l->b); free(l->dW); free(l->db); free(l->u); free(l->z);
    free(l->mW); free(l->vW); free(l->mb); free(l->vb); free(l->o); free(l->gskip);
    for (int q = 0; q < 2 && l->skip_src >= 0; ++q) {
      for (int h = 0; h < n->depth; ++h) { free(l->lane_a[q][h]); free(l->lane_e[q][h]); }
      free(l->lane_a[q]); free(l->lane_e[q]);
    }
  }
  for (int q = 0; q < 2; ++q) {
    for (int h = 0; h < n->depth; ++h) { free(n->act[q][h]); free(n->err[q][h]); }
    free(n->act[q]); free(n->err[q]);
  }
  free(n->stage_of);
  free(n->layers); free(n->first); free(n->count); free(n->g); free(n->g2); free(n->tgt_hist);
  free(n->events);
  free(n);
}

static void *dup_mem(const void *src, size_t bytes) {
  if (!src) return NULL;
  void *d = malloc(bytes ? bytes : 1);
  memcpy(d, src, bytes);
  return d;
}

/* Deep copy of a pipeline with everything it carries between ticks (weights, moments, both halves of every buffer
 * and lane, target history, tick, switches); the gradients of the last tick are not carried over.  For the tests:
 * several continuations of one state. */
void *oracle_clone(const void *p) {
  const net_t *n = (const net_t *)p;
  net_t *c = (net_t *)malloc(sizeof(net_t));
  *c = *n;
  const int D = n->depth, S = n->S;
  c->layers = (layer_t *)dup_mem(n->layers, (size_t)n->n_layers * sizeof(layer_t));
  c->first = (int *)dup_mem(n->first, (size_t)D * sizeof(int));
  c->count = (int *)dup_mem(n->count, (size_t)D * sizeof(int));
  c->stage_of = (int *)dup_mem(n->stage_of, (size_t)n->n_layers * sizeof(int));
  c->g = (double *)calloc((size_t)S * n->max_size, sizeof(double));
  c->g2 = (double *)calloc((size_t)S * n->max_size, sizeof(double));
  c->tgt_hist = (unsigned char *)dup_mem(n->tgt_hist, (size_t)(n->k > 0 ? n->k : 1) * n->tgt_elems * 4);
  c->events = (long *)dup_mem(n->events, (size_t)n->cap_events * 3 * sizeof(long));
  for (int q = 0; q < 2; ++q) {
    c->act[q] = (float **)calloc(D, sizeof(float *));
    c->err[q] = (float **)calloc(D, sizeof(float *));
    for (int h = 0; h < D; ++h) {
      c->act[q][h] = (float *)dup_mem(n->act[q][h], (size_t)S * stage_out(n, h) * sizeof(float));
      c->err[q][h] = (float *)dup_mem(n->err[q][h], (size_t)S * stage_in(n, h) * sizeof(float));
    }
  }
  for (int i = 0; i < n->n_layers; ++i) {
    const layer_t *l = &n->layers[i];
    layer_t *d = &c->layers[i];
    const size_t so = (size_t)S * l->out_size;
    d->W = (float *)dup_mem(l->W, l->n_w * sizeof(float));
    d->b = (float *)dup_mem(l->b, l->n_b * sizeof(float));
    /* scratch of a tick (rebuilt by every tick before it is read): fresh, not copied */
    d->dW = (double *)calloc(l->n_w, sizeof(double));
    d->db = (double *)calloc(l->n_b, sizeof(double));
    d->mW = (float *)dup_mem(l->mW, l->n_w * sizeof(float));
    d->vW = (float *)dup_mem(l->vW, l->n_w * sizeof(float));
    d->mb = (float *)dup_mem(l->mb, l->n_b * sizeof(float));
    d->vb = (float *)dup_mem(l->vb, l->n_b * sizeof(float));
    d->u = (double *)calloc((size_t)S * l->in_size, sizeof(double));
    d->z = (double *)calloc(so, sizeof(double));
    d->o = (double *)calloc(so, sizeof(double));
    d->gskip = (double *)calloc(so, sizeof(double));
    for (int q = 0; q < 2 && l->skip_src >= 0; ++q) {
      d->lane_a[q] = (float **)calloc(D, sizeof(float *));
      d->lane_e[q] = (float **)calloc(D, sizeof(float *));
      for (int h = 0; h < D; ++h) {
        d->lane_a[q][h] = (float *)dup_mem(l->lane_a[q][h], so * sizeof(float));
        d->lane_e[q][h] = (float *)dup_mem(l->lane_e[q][h], so * sizeof(float));
      }
    }
  }
  return c;
}

void oracle_set_weights(void *p, int layer, const float *W, const float *b) {
  net_t *n = (net_t *)p;
  layer_t *l = &n->layers[layer];
  for (long i = 0; i < l->n_w; ++i) l->W[i] = store_w(n, (double)W[i]);
  for (long i = 0; i < l->n_b; ++i) l->b[i] = b[i];
}
void oracle_get_weights(void *p, int layer, float *W, float *b) {
  layer_t *l = &((net_t *)p)->layers[layer];
  memcpy(W, l->W, l->n_w * sizeof(float));
  memcpy(b, l->b, l->n_b * sizeof(float));
}
void oracle_get_grads(void *p, int layer, double *dW, double *db) {
  layer_t *l = &((net_t *)p)->layers[layer];
  memcpy(dW, l->dW, l->n_w * sizeof(double));
  memcpy(db, l->db, l->n_b * sizeof(double));
}
/* which: 0 = activation buffer of a stage, 1 = error buffer of a stage */
void oracle_get_buffer(void *p, int which, int stage, int half, float *dst) {
  net_t *n = (net_t *)p;
  long sz = (long)n->S * (which == 0 ? stage_out(n, stage) : stage_in(n, stage));
  memcpy(dst, which == 0 ? n->act[half][stage] : n->err[half][stage], sz * sizeof(float));
}
void oracle_set_buffer(void *p, int which, int stage, int half, const float *src) {
  net_t *n = (net_t *)p;
  long sz = (long)n->S * (which == 0 ? stage_out(n, stage) : stage_in(n, stage));
  memcpy(which == 0 ? n->act[half][stage] : n->err[half][stage], src, sz * sizeof(float));
}
/* Test access to the delay lines of the skip that ends in layer `layer`: kind 0 = the skipped tensor, 1 = the gradient
 * on its way back; age 0 = the entry written during the last tick, age d - 1 (d = stage boundaries crossed) the one
 * the coming tick consumes.  set != 0 writes, else reads; [S][out_size].  Returns 0, or -1 if there is no such entry. */
int oracle_lane(void *p, int layer, int kind, int age, float *buf, int set) {
  net_t *n = (net_t *)p;
  if (layer < 0 || layer >= n->n_layers || n->layers[layer].skip_src < 0) return -1;
  layer_t *l = &n->layers[layer];
  const int hs = n->stage_of[l->skip_src], ht = n->stage_of[layer];
  if (age < 0 || age >= ht - hs) return -1;
  const int half = (int)((n->tick + 1) & 1);   /* the half the last tick wrote */
  float *lane = kind == 0 ? l->lane_a[half][hs + age] : l->lane_e[half][ht - age];
  const size_t bytes = (size_t)n->S * l->out_size * sizeof(float);
  if (set) memcpy(lane, buf, bytes);
  else memcpy(buf, lane, bytes);
  return 0;
}
/* the targets of the last k ticks, oldest first (k x one tick's targets, 4-byte elements) */
void oracle_get_history(void *p, void *dst) {
  net_t *n = (net_t *)p;
  if (n->k > 0) memcpy(dst, n->tgt_hist, (size_t)n->k * n->tgt_elems * 4);
}
void oracle_set_history(void *p, const void *src) {
  net_t *n = (net_t *)p;
  if (n->k > 0) memcpy(n->tgt_hist, src, (size_t)n->k * n->tgt_elems * 4);
}
long oracle_get_tick(void *p) { return ((net_t *)p)->tick; }
void oracle_set_tick(void *p, long t) { ((net_t *)p)->tick = t; }
void oracle_set_lr(void *p, float lr) { ((net_t *)p)->lr = (double)lr; }
void oracle_set_operand_rounding(void *p, int on) { ((net_t *)p)->op_bf16 = on; }
/* Switch the update rule to Adam (Kingma & Ba, with bias correction; every tick is one optimiser step of every
 * stage, counted from the first tick after creation or reset).  Moments start at zero. */
void oracle_set_adam(void *p, double beta1, double beta2, double eps) {
  net_t *n = (net_t *)p;
  n->adam = 1; n->beta1 = beta1; n->beta2 = beta2; n->eps = eps;
  for (int i = 0; i < n->n_layers; ++i) {
    layer_t *l = &n->layers[i];
    if (!l->mW) {
      l->mW = (float *)calloc(l->n_w, sizeof(float)); l->vW = (float *)calloc(l->n_w, sizeof(float));
      l->mb = (float *)calloc(l->n_b, sizeof(float)); l->vb = (float *)calloc(l->n_b, sizeof(float));
    }
  }
}
void oracle_get_moments(void *p, int layer, float *mW, float *vW, float *mb, float *vb) {
  layer_t *l = &((net_t *)p)->layers[layer];
  memcpy(mW, l->mW, l->n_w * sizeof(float)); memcpy(vW, l->vW, l->n_w * sizeof(float));
  memcpy(mb, l->mb, l->n_b * sizeof(float)); memcpy(vb, l->vb, l->n_b * sizeof(float));
}
void oracle_set_moments(void *p, int layer, const float *mW, const float *vW, const float *mb, const float *vb) {
  layer_t *l = &((net_t *)p)->layers[layer];
  memcpy(l->mW, mW, l->n_w * sizeof(float)); memcpy(l->vW, vW, l->n_w * sizeof(float));
  memcpy(l->mb, mb, l->n_b * sizeof(float)); memcpy(l->vb, vb, l->n_b * sizeof(float));
}
/* Diagnostic for the parity tests, no part of the method: the smallest |z| at which the derivative of a ReLU
 * entered a non-zero delta since the last call (a huge value if none).  The derivative jumps at z = 0 (Eq. 9
 * evaluates it at this tick's z), so an implementation that sums z in another order or precision can land on the
 * other side when |z| is within its rounding error; a run whose margin is that small has no element-wise answer. */
double oracle_take_kink_margin(void *p) {
  net_t *n = (net_t *)p;
  double m = n->kink_margin;
  n->kink_margin = 1e300;
  return m;
}
/* Test diagnostic, no part of the method.  Eq. 9 takes the derivative at this tick's z, and ReLU' jumps at 0: an
 * implementation that sums z = sum_i w_i u_i + b in fp32, or in another order, can land on the other side of 0 when
 * |z| is within its rounding error, and then takes the other one-sided derivative; both are derivatives of the
 * function it evaluated.  The rounding error of a sum is proportional to the size of its terms, so the band is
 * relative: with eps > 0 every ReLU unit with |z| < eps * (sum_i |w_i u_i| + |b|) and a non-zero error signal is
 * recorded (tick, layer, stream * out_size + unit).  side = 0 leaves the arithmetic alone (ReLU'(z) = [z > 0]);
 * side = +1 / -1 takes 1 / 0 as the derivative of the recorded units, so that a test can tell which results depend
 * on those units at all. */
void oracle_set_kink_band(void *p, double eps, int side, long cap) {
  net_t *n = (net_t *)p;
  n->band_eps = eps; n->band_side = side;
  free(n->events);
  n->cap_events = cap > 0 ? cap : 0;
  n->events = (long *)calloc((size_t)(n->cap_events ? n->cap_events : 1) * 3, sizeof(long));
  n->n_events = 0;
}
/* number of recorded units since the last call; the first min(count, cap) triples are copied to buf */
long oracle_take_kink_events(void *p, long *buf) {
  net_t *n = (net_t *)p;
  const long cnt = n->n_events, m = cnt < n->cap_events ? cnt : n->cap_events;
  if (buf && m > 0) memcpy(buf, n->events, (size_t)m * 3 * sizeof(long));
  n->n_events = 0;
  return cnt;
}

void oracle_reset(void *p) {
  net_t *n = (net_t *)p;
  n->n_events = 0;
  for (int q = 0; q < 2; ++q)
    for (int h = 0; h < n->depth; ++h) {
      memset(n->act[q][h], 0, (size_t)n->S * stage_out(n, h) * sizeof(float));
      memset(n->err[q][h], 0, (size_t)n->S * stage_in(n, h) * sizeof(float));
    }
  memset(n->tgt_hist, 0, (size_t)(n->k > 0 ? n->k : 1) * n->tgt_elems * 4);
  n->tick = 0;
  n->kink_margin = 1e300;
  for (int i = 0; i < n->n_layers; ++i) {
    layer_t *l = &n->layers[i];
    for (int q = 0; q < 2 && l->skip_src >= 0; ++q)
      for (int h = 0; h < n->depth; ++h) {
        memset(l->lane_a[q][h], 0, (size_t)n->S * l->out_size * sizeof(float));
        memset(l->lane_e[q][h], 0, (size_t)n->S * l->out_size * sizeof(float));
      }
  }
  for (int i = 0; i < n->n_layers && n->adam; ++i) {
    layer_t *l = &n->layers[i];
    memset(l->mW, 0, l->n_w * sizeof(float)); memset(l->vW, 0, l->n_w * sizeof(float));
    memset(l->mb, 0, l->n_b * sizeof(float)); memset(l->vb, 0, l->n_b * sizeof(float));
  }
}

/* ---- one stage of one tick ---------------------------------------------- */

static void stage_tick(net_t *n, int h, const float *x_t, const void *target_used, int learn,
                       float *out_t, double *loss_acc) {
  const int D = n->depth, S = n->S;
  const int cur = (int)(n->tick & 1), prev = 1 - cur;
  const int f = n->first[h], c = n->count[h];
  const long nin = stage_in(n, h), nout = stage_out(n, h);

  /* Algorithm 1, first step: the stage input */
  layer_t *l0 = &n->layers[f];
  for (long i = 0; i < (long)S * nin; ++i)
    l0->u[i] = opr(n, h == 0 ? (double)x_t[i] : (double)n->act[prev][h - 1][i]);

  /* forward through the stage's layers (Eq. 6) */
  for (int j = 0; j < c; ++j) {
    layer_t *l = &n->layers[f + j];
    for (int s = 0; s < S; ++s) layer_forward(l, l->u + s * l->in_size, l->z + s * l->out_size);
    for (long i = 0; i < (long)S * l->out_size; ++i) l->o[i] = phi(l->act, l->z[i]);
    if (l->skip_src >= 0) {
      /* the skipped tensor: from the same stage directly, else what the lane delivered for this tick */
      const int hs = n->stage_of[l->skip_src];
      for (long i = 0; i < (long)S * l->out_size; ++i)
        l->o[i] += hs == h ? n->layers[l->skip_src].o[i] : (double)l->lane_a[prev][h - 1][i];
    }
    double *o = j + 1 < c ? n->layers[f + j + 1].u : n->g2;
    for (long i = 0; i < (long)S * l->out_size; ++i) o[i] = j + 1 < c ? opr(n, l->o[i]) : l->o[i];
  }
  /* identity lanes: a skip that starts in this stage enters its lane, one that passes through moves on by one stage */
  for (int i = 0; i < n->n_layers; ++i) {
    layer_t *t = &n->layers[i];
    if (t->skip_src < 0) continue;
    const int hs = n->stage_of[t->skip_src], ht = n->stage_of[i];
    const long sz = (long)S * t->out_size;
    if (hs == h && ht > h)
      for (long q = 0; q < sz; ++q) t->lane_a[cur][h][q] = (float)n->layers[t->skip_src].o[q];
    else if (hs < h && h < ht)
      memcpy(t->lane_a[cur][h], t->lane_a[prev][h - 1], sz * sizeof(float));
  }
  layer_t *ll = &n->layers[f + c - 1];
  double *o = n->g2; /* [S][nout] stage output, fp64 */

  if (h == D - 1) {
    for (long i = 0; i < (long)S * nout; ++i) out_t[i] = (float)o[i];
  } else {
    for (long i = 0; i < (long)S * nout; ++i) n->act[cur][h][i] = (float)o[i];
  }
  if (!learn) return;

  /* g_h of this tick */
  double *g = n->g;
  if (h == D - 1) {
    const long fill = (D - 1 > n->k ? D - 1 : n->k);
    if (n->tick >= fill) {
      double acc = 0.0;
      for (int s = 0; s < S; ++s) acc += loss_and_grad(n, o + s * nout, target_used, s, nout, g + s * nout);
      *loss_acc = acc / (double)S;
    } else {
      for (long i = 0; i < (long)S * nout; ++i) g[i] = 0.0;
      *loss_acc = 0.0;
    }
  } else {
    for (long i = 0; i < (long)S * nout; ++i) g[i] = (double)n->err[prev][h + 1][i];
  }

  /* backward inside the stage (Eq. 5), weight gradients at this tick's input and
   * weights (Eq. 9); the input-gradient uses the not-yet-updated weights */
  for (int j = c - 1; j >= 0; --j) {
    layer_t *l = &n->layers[f + j];
    memset(l->dW, 0, l->n_w * sizeof(double));
    memset(l->db, 0, l->n_b * sizeof(double));
    const long osz = (long)S * l->out_size;
    if (l->skip_dst >= 0) {
      /* this layer's output also fed a skip: its gradient comes back over the lane (one stage per tick), or
       * directly if the skip ended inside this stage */
      layer_t *t = &n->layers[l->skip_dst];
      const int ht = n->stage_of[l->skip_dst];
      for (long i = 0; i < osz; ++i) g[i] += ht == h ? l->gskip[i] : (double)t->lane_e[prev][h + 1][i];
    }
    if (l->skip_src >= 0) {
      /* o = phi(z) + skipped tensor: the gradient at o goes to the skipped tensor unchanged */
      const int hs = n->stage_of[l->skip_src];
      if (hs == h) memcpy(n->layers[l->skip_src].gskip, g, osz * sizeof(double));
      else
        for (long i = 0; i < osz; ++i) l->lane_e[cur][h][i] = (float)g[i];
    }
    double *delta = n->g2; /* o is no longer needed */
    for (long i = 0; i < (long)S * l->out_size; ++i) delta[i] = opr(n, g[i] * dphi(l->act, l->z[i]));
    if (l->act == A_RELU)
      for (int s = 0; s < S; ++s) {
        const double *us = l->u + s * l->in_size;
        const double bound = n->band_eps > 0.0 ? n->band_eps * layer_abs_bound(l, us) : 0.0;
        for (long q = 0; q < l->out_size; ++q) {
          const long i = s * l->out_size + q;
          if (g[i] == 0.0) continue;
          const double az = fabs(l->z[i]);
          if (az < n->kink_margin) n->kink_margin = az;
          /* test band (see oracle_set_kink_band): |z| below band_eps times the size of the unit's terms */
          if (az < bound && az < n->band_eps * unit_abs_sum(l, us, q)) {
            if (n->n_events < n->cap_events) {
              long *e = n->events + 3 * n->n_events;
              e[0] = n->tick; e[1] = f + j; e[2] = i;
            }
            n->n_events += 1;
            if (n->band_side != 0) delta[i] = opr(n, n->band_side > 0 ? g[i] : 0.0);
          }
        }
      }
    for (int s = 0; s < S; ++s)
      layer_weight_grad(l, l->u + s * l->in_size, delta + s * l->out_size, 1.0 / (double)S, l->dW, l->db);
    if (j > 0 || h > 0)
      for (int s = 0; s < S; ++s)
        layer_input_grad(l, delta + s * l->out_size, g + s * l->in_size);
  }
  (void)ll;
  if (h > 0)
    for (long i = 0; i < (long)S * nin; ++i) n->err[cur][h][i] = (float)g[i];
  /* gradient lanes that pass through this stage move on by one stage */
  for (int i = 0; i < n->n_layers; ++i) {
    layer_t *t = &n->layers[i];
    if (t->skip_src < 0) continue;
    const int hs = n->stage_of[t->skip_src], ht = n->stage_of[i];
    if (hs < h && h < ht) memcpy(t->lane_e[cur][h], t->lane_e[prev][h + 1], (size_t)S * t->out_size * sizeof(float));
  }

  /* immediate update (Algorithm 1, last step) */
  for (int j = 0; j < c; ++j) {
    layer_t *l = &n->layers[f + j];
    if (!n->adam) {
#pragma omp parallel for schedule(static)
      for (long i = 0; i < l->n_w; ++i) l->W[i] = store_w(n, (double)l->W[i] - n->lr * l->dW[i]);
      for (long i = 0; i < l->n_b; ++i) l->b[i] = (float)((double)l->b[i] - n->lr * l->db[i]);
    } else {
      /* Adam: m <- b1 m + (1 - b1) g, v <- b2 v + (1 - b2) g^2, w <- w - lr (m / (1 - b1^n)) / (sqrt(v / (1 - b2^n)) + eps),
       * n = number of this optimiser step; the moments are stored in fp32 */
      const double nstep = (double)(n->tick + 1);
      const double c1 = 1.0 - pow(n->beta1, nstep), c2 = 1.0 - pow(n->beta2, nstep);
#pragma omp parallel for schedule(static)
      for (long i = 0; i < l->n_w; ++i) {
        const double g = l->dW[i];
        const double m = n->beta1 * (double)l->mW[i] + (1.0 - n->beta1) * g;
        const double v = n->beta2 * (double)l->vW[i] + (1.0 - n->beta2) * g * g;
        l->mW[i] = (float)m; l->vW[i] = (float)v;
        l->W[i] = store_w(n, (double)l->W[i] - n->lr * (m / c1) / (sqrt(v / c2) + n->eps));
      }
      for (long i = 0; i < l->n_b; ++i) {
        const double g = l->db[i];
        const double m = n->beta1 * (double)l->mb[i] + (1.0 - n->beta1) * g;
        const double v = n->beta2 * (double)l->vb[i] + (1.0 - n->beta2) * g * g;
        l->mb[i] = (float)m; l->vb[i] = (float)v;
        l->b[i] = (float)((double)l->b[i] - n->lr * (m / c1) / (sqrt(v / c2) + n->eps));
      }
    }
  }
}

/* ---- public tick loops --------------------------------------------------- */

/* x: [n_ticks][S][in]; target: [n_ticks][S][out] fp32 (MSE) or [n_ticks][S] int32 (CE);
 * out: [n_ticks][S][out]; loss: [n_ticks]; order: NULL or a permutation of 0..D-1. */
void oracle_step(void *p, const float *x, const void *target, int n_ticks, float *out,
                 float *loss, const int *order) {
  net_t *n = (net_t *)p;
  const int D = n->depth;
  const long nin = (long)n->S * stage_in(n, 0), nout = (long)n->S * stage_out(n, D - 1);
  const size_t tb = (size_t)n->tgt_elems * 4;
  for (int i = 0; i < n_ticks; ++i) {
    const unsigned char *tgt_now = (const unsigned char *)target + (size_t)i * tb;
    /* target supplied k ticks ago: oldest entry of the history when k > 0 */
    const void *used = n->k > 0 ? (const void *)n->tgt_hist : (const void *)tgt_now;
    double la = 0.0;
    for (int q = 0; q < D; ++q) {
      int h = order ? order[q] : q;
      stage_tick(n, h, x + (size_t)i * nin, used, 1, out + (size_t)i * nout, &la);
    }
    loss[i] = (float)la;
    if (n->k > 0) {
      memmove(n->tgt_hist, n->tgt_hist + tb, (size_t)(n->k - 1) * tb);
      memcpy(n->tgt_hist + (size_t)(n->k - 1) * tb, tgt_now, tb);
    }
    n->tick += 1;
  }
}

void oracle_infer(void *p, const float *x, int n_ticks, float *out) {
  net_t *n = (net_t *)p;
  const int D = n->depth;
  const long nin = (long)n->S * stage_in(n, 0), nout = (long)n->S * stage_out(n, D - 1);
  for (int i = 0; i < n_ticks; ++i) {
    double la;
    for (int h = 0; h < D; ++h)
      stage_tick(n, h, x + (size_t)i * nin, NULL, 0, out + (size_t)i * nout, &la);
    n->tick += 1;
  }
}
