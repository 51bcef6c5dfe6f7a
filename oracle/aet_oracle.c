/*
 * CPU oracle for the AET-SGD client/round/server loop.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar implementation of what the GPU library computes, written from
 * the paper (arXiv 2112.13935) and sharing no code with the GPU path.  Only the tests,
 * the smoke check and the benchmark's "cpu_baseline" leg may load it; no product code
 * may call into it.
 *
 * What follows what:
 *   - the SGD recursion w <- w - eta * grad f(w; xi)                  : eq. (3)
 *   - clients run local recursions on their own data, send the sum of
 *     gradients U of the round, a server aggregates and rebroadcasts   : Introduction,
 *                                                                        client-server paragraph
 *   - the local round: h = 0, U = 0; while h < s_{i,c}: sample xi
 *     uniformly from D_c; g = grad f(w_c, xi); w_c -= eta_i g;
 *     U += g; h += 1; then send (c, U_i, i)                            : Algorithm 2, MainComputeNode
 *   - a received (v, U, k) is applied as w -= eta_k * U, H_v += 1      : Algorithm 2, Receive
 *   - peer-to-peer form: every node keeps its own model, sends
 *     (c, U_i, i) to its neighbours only and applies what they send    : Algorithm 2 as printed;
 *                                                                        Section 2.2.1 (undirected
 *                                                                        topology, neighbour lists given)
 *   - the delay checkpoint max_e (i - H_e) > d                         : Algorithm 2, Synchronize
 *   - Setup: each of the s_i recursions of global round i is assigned
 *     to node c with probability p_c; s_{i,c} counts node c's share    : Algorithm 1
 *   - round lengths s_i = a*i^p + b with p = 1; step size
 *     eta0 / (1 + beta * t^power), constant inside a round             : Section 3.1, Experiments
 *                                                                        ("Objective function"), Table 5
 *
 * Readings taken where the paper is silent:
 * thresholds are per client and count samples; a mini-batch step uses the mean of the
 * per-sample gradients; sampling is i.i.d. with replacement from a counter hash
 * (SplitMix64, Steele/Lea/Flood 2014); clients adopt the global model only at the start
 * of a round; time advances in integer ticks, a round of a client with compute factor f
 * occupies f ticks and a straggler's message is delayed by a hashed number of ticks.
 *
 * Precision: compile with -DREAL=double (the reference) or -DREAL=float (conditioning
 * twin).  No blocking, fusion or reordering beyond the definitions.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL double
#endif
typedef REAL real;

#define ORC_CONV 0
#define ORC_POOL 1
#define ORC_DENSE 2
#define ORC_MAX_LAYERS 16

typedef struct { int32_t type, cout, k, pad, relu; } orc_layer;
typedef struct {
    int32_t in_c, in_h, in_w, n_layers, batch;
    orc_layer layers[ORC_MAX_LAYERS];
} orc_model;

/* resolved layer geometry */
typedef struct {
    int type, relu, k, pad;
    int ic, ih, iw, oc, oh, ow;
    int64_t w_off, b_off, in_size, out_size;
} lay_t;

typedef struct {
    int32_t c, k;
    double eta;
    int64_t arrival;
    real *U;
} msg_t;

typedef struct {
    int64_t s, m, q0, t0, start_tick, arrival;
    double eta, loss;
    int64_t kink_events;     /* near-kink decisions met in the round (kink analysis on) */
    double *kink_allow;      /* per parameter tensor: sum of the jumps those would cause */
} rinfo_t;

typedef struct orc_ctx {
    orc_model model;
    int L;
    lay_t lay[ORC_MAX_LAYERS];
    int64_t P;
    int n;
    const float **X;
    const int32_t **y;
    int64_t *N;
    real *Wg, *W;
    int64_t *i_c, *t_c, *q_c, *free_at, *H;
    int setup;               /* 1: round lengths from the coin flips of Algorithm 1 */
    uint64_t setup_seed;
    uint64_t *cumw;          /* cumulative node weights, cumw[c] = w_0 + ... + w_c */
    int p2p;                 /* 1: peer-to-peer form on the topology below */
    int32_t *nbr_off, *nbr;  /* neighbour lists, CSR: nbr[nbr_off[c] .. nbr_off[c+1]) ascending */
    int64_t tick;
    uint64_t seed;
    msg_t *queue; int n_queue, cap_queue;
    rinfo_t **rinfo; int *n_rinfo, *cap_rinfo;
    int64_t *ev_tick; int32_t *ev_c, *ev_k; int64_t n_ev, cap_ev;
    double kink_eps;         /* > 0: kink analysis with this relative margin */
    int n_tensors;           /* parameter tensors: weights and bias of every conv / dense layer */
    char err[256];
} orc_ctx;

/* ------------------------------------------------------------------------------------
 * Counter hash.  SplitMix64 (Steele, Lea, Flood, "Fast splittable pseudorandom number
 * generators", OOPSLA 2014; constants of the public-domain reference generator):
 * output number k (from 0) of a generator seeded with s is mix(s + (k+1)*GAMMA).
 * ---------------------------------------------------------------------------------- */
static const uint64_t GAMMA = 0x9E3779B97F4A7C15ULL;

static uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
uint64_t orc_draw(uint64_t seed, uint64_t k) { return mix64(seed + (k + 1) * GAMMA); }

#define TAG_SAMPLE 0
#define TAG_NET 1
#define TAG_SETUP 2
/* one stream per (seed, purpose, client); element `ctr` of that stream */
uint64_t orc_stream(uint64_t seed, uint64_t tag, uint64_t c, uint64_t ctr) {
    return orc_draw(orc_draw(orc_draw(seed, tag), c), ctr);
}
/* map the top 32 bits of a hash onto [0, range) by multiply-shift */
static uint32_t to_range(uint64_t h, uint64_t range) {
    return (uint32_t)(((h >> 32) * range) >> 32);
}
/* Algorithm 2, sampling step of MainComputeNode: index of the q-th sample that
 * client c draws, uniform on [0, n_samples), with replacement. */
int32_t orc_sample_index(uint64_t seed, int32_t c, int64_t q, int64_t n_samples) {
    return (int32_t)to_range(orc_stream(seed, TAG_SAMPLE, (uint64_t)c, (uint64_t)q),
                             (uint64_t)n_samples);
}
/* extra ticks a straggler's round-k message spends in the network */
int32_t orc_net_delay(uint64_t dseed, int32_t c, int32_t k, int32_t dmin, int32_t dmax) {
    return dmin + (int32_t)to_range(orc_stream(dseed, TAG_NET, (uint64_t)c, (uint64_t)k),
                                    (uint64_t)(dmax - dmin + 1));
}

/* Section 3.1 / Table 5: s_i = a*i + b (the p = 1 case the paper uses) */
int64_t orc_threshold(int64_t a, int64_t b, int64_t i) { return a * i + b; }

/* Section 3.1: K = sum_{j=0..T} s_j.  Number of non-empty rounds, taken in order from
 * round 0, until at least K recursions have been done (0 if K <= 0; -1 if never). */
int64_t orc_rounds_needed(int64_t a, int64_t b, int64_t K) {
    int64_t done = 0, rounds = 0;
    if (K <= 0) return 0;
    if (a <= 0 && b <= 0) return -1;
    for (int64_t i = 0; done < K; ++i) {
        int64_t s = orc_threshold(a, b, i);
        if (s > 0) { done += s; rounds += 1; }
    }
    return rounds;
}

/* Experiments, "Objective function": eta0 / (1 + beta * t^power); the paper uses
 * power = 1/2, t = recursions done so far; constant within a round (Section 3.1). */
double orc_eta(double eta0, double beta, double power, int64_t t) {
    return eta0 / (1.0 + beta * pow((double)t, power));
}

/* ------------------------------------------------------------------------------------
 * Model geometry
 * ---------------------------------------------------------------------------------- */
static int resolve(const orc_model *m, lay_t *lay, int64_t *P) {
    int c = m->in_c, h = m->in_h, w = m->in_w;
    int64_t off = 0;
    if (m->n_layers < 1 || m->n_layers > ORC_MAX_LAYERS || m->batch < 1) return -1;
    for (int l = 0; l < m->n_layers; ++l) {
        const orc_layer *q = &m->layers[l];
        lay_t *o = &lay[l];
        memset(o, 0, sizeof *o);
        o->type = q->type; o->relu = q->relu; o->k = q->k; o->pad = q->pad;
        o->ic = c; o->ih = h; o->iw = w;
        o->in_size = (int64_t)c * h * w;
        if (q->type == ORC_CONV) {
            if (q->k < 1 || q->pad < 0 || q->cout < 1) return -1;
            o->oc = q->cout; o->oh = h + 2 * q->pad - q->k + 1; o->ow = w + 2 * q->pad - q->k + 1;
            if (o->oh < 1 || o->ow < 1) return -1;
            o->w_off = off; off += (int64_t)q->cout * c * q->k * q->k;
            o->b_off = off; off += q->cout;
        } else if (q->type == ORC_POOL) {
            if ((h & 1) || (w & 1)) return -1;
            o->oc = c; o->oh = h / 2; o->ow = w / 2;
        } else if (q->type == ORC_DENSE) {
            if (q->cout < 1) return -1;
            o->oc = q->cout; o->oh = 1; o->ow = 1;
            o->w_off = off; off += (int64_t)q->cout * o->in_size;
            o->b_off = off; off += q->cout;
        } else return -1;
        o->out_size = (int64_t)o->oc * o->oh * o->ow;
        c = o->oc; h = o->oh; w = o->ow;
    }
    if (m->layers[m->n_layers - 1].type != ORC_DENSE || m->layers[m->n_layers - 1].relu) return -1;
    *P = off;
    return 0;
}

int64_t orc_n_params(const orc_model *m) {
    lay_t lay[ORC_MAX_LAYERS]; int64_t P;
    return resolve(m, lay, &P) ? -1 : P;
}

/* per-thread scratch for one sample's forward/backward pass */
typedef struct {
    real *act[ORC_MAX_LAYERS + 1];   /* act[0] = input, act[l+1] = output of layer l */
    real *del[ORC_MAX_LAYERS + 1];   /* d loss / d act[l] */
    int32_t *amax[ORC_MAX_LAYERS];   /* pool: flat input index of each output's maximum */
} scratch_t;

static int scratch_alloc(const lay_t *lay, int L, scratch_t *s) {
    memset(s, 0, sizeof *s);
    s->act[0] = (real *)malloc(sizeof(real) * lay[0].in_size);
    s->del[0] = (real *)malloc(sizeof(real) * lay[0].in_size);
    if (!s->act[0] || !s->del[0]) return -1;
    for (int l = 0; l < L; ++l) {
        s->act[l + 1] = (real *)malloc(sizeof(real) * lay[l].out_size);
        s->del[l + 1] = (real *)malloc(sizeof(real) * lay[l].out_size);
        if (!s->act[l + 1] || !s->del[l + 1]) return -1;
        if (lay[l].type == ORC_POOL) {
            s->amax[l] = (int32_t *)malloc(sizeof(int32_t) * lay[l].out_size);
            if (!s->amax[l]) return -1;
        }
    }
    return 0;
}
static void scratch_free(int L, scratch_t *s) {
    for (int l = 0; l <= L; ++l) { free(s->act[l]); free(s->del[l]); }
    for (int l = 0; l < L; ++l) free(s->amax[l]);
}

/* ------------------------------------------------------------------------------------
 * f(w; xi) = cross-entropy of softmax(net(x)) against the label, and its gradient.
 * Adds grad f(w; x, y) into g (g is NOT cleared) and returns the loss.  g == NULL:
 * loss only.  Plain definitions: direct convolution, 2x2/stride-2 max pooling with the
 * first maximum in row-major window order winning, ReLU' = 1[z > 0].
 * ---------------------------------------------------------------------------------- */
static real sample_loss_grad(const lay_t *lay, int L, const real *w, const float *x, int32_t label,
                             real *g, scratch_t *s) {
    for (int64_t i = 0; i < lay[0].in_size; ++i) s->act[0][i] = (real)x[i];
    /* forward */
    for (int l = 0; l < L; ++l) {
        const lay_t *q = &lay[l];
        const real *in = s->act[l];
        real *out = s->act[l + 1];
        if (q->type == ORC_CONV) {
            const real *W = w + q->w_off, *b = w + q->b_off;
            for (int co = 0; co < q->oc; ++co)
                for (int oy = 0; oy < q->oh; ++oy)
                    for (int ox = 0; ox < q->ow; ++ox) {
                        real acc = b[co];
                        for (int ci = 0; ci < q->ic; ++ci)
                            for (int ky = 0; ky < q->k; ++ky) {
                                int iy = oy + ky - q->pad;
                                if (iy < 0 || iy >= q->ih) continue;
                                for (int kx = 0; kx < q->k; ++kx) {
                                    int ix = ox + kx - q->pad;
                                    if (ix < 0 || ix >= q->iw) continue;
                                    acc += W[(((int64_t)co * q->ic + ci) * q->k + ky) * q->k + kx] *
                                           in[((int64_t)ci * q->ih + iy) * q->iw + ix];
                                }
                            }
                        if (q->relu && !(acc > 0)) acc = 0;
                        out[((int64_t)co * q->oh + oy) * q->ow + ox] = acc;
                    }
        } else if (q->type == ORC_POOL) {
            for (int c = 0; c < q->oc; ++c)
                for (int oy = 0; oy < q->oh; ++oy)
                    for (int ox = 0; ox < q->ow; ++ox) {
                        int64_t best = ((int64_t)c * q->ih + 2 * oy) * q->iw + 2 * ox;
                        for (int dy = 0; dy < 2; ++dy)
                            for (int dx = 0; dx < 2; ++dx) {
                                int64_t j = ((int64_t)c * q->ih + 2 * oy + dy) * q->iw + 2 * ox + dx;
                                if (in[j] > in[best]) best = j;
                            }
                        int64_t o = ((int64_t)c * q->oh + oy) * q->ow + ox;
                        out[o] = in[best];
                        s->amax[l][o] = (int32_t)best;
                    }
        } else {
            const real *W = w + q->w_off, *b = w + q->b_off;
            for (int o = 0; o < q->oc; ++o) {
                real acc = b[o];
                for (int64_t k = 0; k < q->in_size; ++k) acc += W[(int64_t)o * q->in_size + k] * in[k];
                if (q->relu && !(acc > 0)) acc = 0;
                out[o] = acc;
            }
        }
    }
    /* softmax cross-entropy on the logits, with the maximum subtracted */
    const int C = lay[L - 1].oc;
    const real *z = s->act[L];
    real zmax = z[0];
    for (int j = 1; j < C; ++j) if (z[j] > zmax) zmax = z[j];
    real sum = 0;
    for (int j = 0; j < C; ++j) sum += (real)exp((double)(z[j] - zmax));
    real lse = zmax + (real)log((double)sum);
    real loss = lse - z[label];
    if (!g) return loss;
    for (int j = 0; j < C; ++j) s->del[L][j] = (real)exp((double)(z[j] - lse)) - (j == label ? 1 : 0);
    /* backward */
    for (int l = L - 1; l >= 0; --l) {
        const lay_t *q = &lay[l];
        const real *in = s->act[l], *out = s->act[l + 1];
        real *dout = s->del[l + 1], *din = s->del[l];
        const int need_din = (l > 0);
        if (need_din) for (int64_t i = 0; i < q->in_size; ++i) din[i] = 0;
        if (q->type == ORC_CONV) {
            const real *W = w + q->w_off;
            real *gW = g + q->w_off, *gb = g + q->b_off;
            for (int co = 0; co < q->oc; ++co)
                for (int oy = 0; oy < q->oh; ++oy)
                    for (int ox = 0; ox < q->ow; ++ox) {
                        int64_t o = ((int64_t)co * q->oh + oy) * q->ow + ox;
                        real d = dout[o];
                        if (q->relu && !(out[o] > 0)) d = 0;
                        gb[co] += d;
                        for (int ci = 0; ci < q->ic; ++ci)
                            for (int ky = 0; ky < q->k; ++ky) {
                                int iy = oy + ky - q->pad;
                                if (iy < 0 || iy >= q->ih) continue;
                                for (int kx = 0; kx < q->k; ++kx) {
                                    int ix = ox + kx - q->pad;
                                    if (ix < 0 || ix >= q->iw) continue;
                                    int64_t wi = (((int64_t)co * q->ic + ci) * q->k + ky) * q->k + kx;
                                    int64_t ii = ((int64_t)ci * q->ih + iy) * q->iw + ix;
                                    gW[wi] += d * in[ii];
                                    if (need_din) din[ii] += d * W[wi];
                                }
                            }
                    }
        } else if (q->type == ORC_POOL) {
            if (need_din)
                for (int64_t o = 0; o < q->out_size; ++o) din[s->amax[l][o]] += dout[o];
        } else {
            const real *W = w + q->w_off;
            real *gW = g + q->w_off, *gb = g + q->b_off;
            for (int o = 0; o < q->oc; ++o) {
                real d = dout[o];
                if (q->relu && !(out[o] > 0)) d = 0;
                gb[o] += d;
                for (int64_t k = 0; k < q->in_size; ++k) {
                    gW[(int64_t)o * q->in_size + k] += d * in[k];
                    if (need_din) din[k] += d * W[(int64_t)o * q->in_size + k];
                }
            }
        }
    }
    return loss;
}

/* Mean loss and mean gradient of a mini-batch of B samples (rows of X, labels y).
 * g (P entries) is overwritten; g may be NULL for the loss alone.  Returns < 0 on a bad
 * model.  Exposed so that the tests can difference the loss numerically. */
double orc_batch_loss_grad(const orc_model *m, const real *w, const float *X, const int32_t *y,
                           int32_t B, real *g) {
    lay_t lay[ORC_MAX_LAYERS]; int64_t P; scratch_t s;
    if (resolve(m, lay, &P)) return -1.0;
    if (scratch_alloc(lay, m->n_layers, &s)) { scratch_free(m->n_layers, &s); return -2.0; }
    if (g) for (int64_t p = 0; p < P; ++p) g[p] = 0;
    real loss = 0;
    for (int j = 0; j < B; ++j)
        loss += sample_loss_grad(lay, m->n_layers, w, X + (int64_t)j * lay[0].in_size, y[j], g, &s);
    if (g) for (int64_t p = 0; p < P; ++p) g[p] /= (real)B;
    scratch_free(m->n_layers, &s);
    return (double)(loss / (real)B);
}

/* ------------------------------------------------------------------------------------
 * Kinks (bookkeeping for the parity tolerance; not part of what the method computes).
 *
 * f(w; xi) is piecewise smooth in w: grad f jumps where the pre-activation of a ReLU unit
 * crosses zero and where the two largest entries of a pooling window cross.  Another
 * implementation of the same recursion (another precision, another summation order) can
 * land on the other side of such a point; from there on its w and U differ from this
 * oracle's by the jump, whatever the quality of its arithmetic.  For one sample whose
 * forward and backward pass has just run (the scratch still holds activations and deltas)
 * the functions below find the decisions that lie within a relative margin eps of
 * flipping,
 *     ReLU unit:    |z| < eps * (|b| + sum |w| |x|)              (z its pre-activation)
 *     pool window:  best - second < eps * max(scale of the two)  (scale as above, of the
 *                   units that produced the two entries; only windows with best > 0)
 * and, for each, the change of the sample's gradient if that one decision flipped:
 *     ReLU unit:    the unit's incoming delta, taken as a one-hot delta at its layer and
 *                   carried down through the layers below with their decisions as they are;
 *     pool window:  that delta moved from the winning entry to the runner-up.
 * Per parameter tensor the largest entry of each such change is added up (kink_t.allow).
 * ---------------------------------------------------------------------------------- */
typedef struct {
    double eps;
    int64_t events;
    double *allow;                      /* per parameter tensor, in layer order: W then b */
    real *jump;                         /* P entries, zero between events */
    real *kd[ORC_MAX_LAYERS + 1];       /* delta of the flipped decision at every level */
    real *scale[ORC_MAX_LAYERS];        /* |b| + sum |w||x| of every conv / dense output */
    /* optional list of the events themselves (tests): layer, output index, whole jump */
    int64_t rec_cap, rec_P;
    int32_t *rec_layer; int64_t *rec_unit; real *rec_jump;
} kink_t;

static int kink_alloc(const lay_t *lay, int L, int64_t P, int n_tensors, double eps, kink_t *k) {
    memset(k, 0, sizeof *k);
    k->eps = eps;
    k->allow = (double *)calloc(n_tensors > 0 ? n_tensors : 1, sizeof(double));
    k->jump = (real *)calloc(P, sizeof(real));
    if (!k->allow || !k->jump) return -1;
    k->kd[0] = (real *)calloc(lay[0].in_size, sizeof(real));
    if (!k->kd[0]) return -1;
    for (int l = 0; l < L; ++l) {
        k->kd[l + 1] = (real *)calloc(lay[l].out_size, sizeof(real));
        if (!k->kd[l + 1]) return -1;
        if (lay[l].type != ORC_POOL) {
            k->scale[l] = (real *)calloc(lay[l].out_size, sizeof(real));
            if (!k->scale[l]) return -1;
        }
    }
    return 0;
}
static void kink_free(int L, kink_t *k) {
    free(k->allow); free(k->jump);
    for (int l = 0; l <= L; ++l) free(k->kd[l]);
    for (int l = 0; l < L; ++l) free(k->scale[l]);
}

/* pre-activation z and its magnitude scale |b| + sum |w||x| of output o of a conv / dense layer */
static void preactivation(const lay_t *q, const real *w, const real *in, int64_t o, real *z, real *sc) {
    const real *W = w + q->w_off, *b = w + q->b_off;
    real acc, mag;
    if (q->type == ORC_DENSE) {
        acc = b[o]; mag = (real)fabs((double)b[o]);
        for (int64_t k = 0; k < q->in_size; ++k) {
            const real t = W[o * q->in_size + k] * in[k];
            acc += t; mag += (real)fabs((double)t);
        }
    } else {
        const int co = (int)(o / ((int64_t)q->oh * q->ow));
        const int oy = (int)((o / q->ow) % q->oh), ox = (int)(o % q->ow);
        acc = b[co]; mag = (real)fabs((double)b[co]);
        for (int ci = 0; ci < q->ic; ++ci)
            for (int ky = 0; ky < q->k; ++ky) {
                const int iy = oy + ky - q->pad;
                if (iy < 0 || iy >= q->ih) continue;
                for (int kx = 0; kx < q->k; ++kx) {
                    const int ix = ox + kx - q->pad;
                    if (ix < 0 || ix >= q->iw) continue;
                    const real t = W[(((int64_t)co * q->ic + ci) * q->k + ky) * q->k + kx] *
                                   in[((int64_t)ci * q->ih + iy) * q->iw + ix];
                    acc += t; mag += (real)fabs((double)t);
                }
            }
    }
    *z = acc; *sc = mag;
}

/* The delta k->kd[top + 1] at the output of layer `top` (zero but for a few entries) carried
 * down to the input: adds the parameter gradients it causes into k->jump.  Layers below
 * `top` apply their ReLU decisions as the forward pass took them; layer `top` itself does
 * only when mask_top is set (a flipped unit's own delta passes by definition). */
static void carry_down(const lay_t *lay, int top, int mask_top, const real *w, const scratch_t *s, kink_t *k) {
    for (int l = top; l >= 0; --l) {
        const lay_t *q = &lay[l];
        const real *in = s->act[l], *out = s->act[l + 1];
        const real *dout = k->kd[l + 1];
        real *din = k->kd[l];
        const int masked = q->relu && (l < top || mask_top);
        for (int64_t i = 0; i < q->in_size; ++i) din[i] = 0;
        if (q->type == ORC_POOL) {
            for (int64_t o = 0; o < q->out_size; ++o)
                if (dout[o] != 0) din[s->amax[l][o]] += dout[o];
        } else if (q->type == ORC_DENSE) {
            const real *W = w + q->w_off;
            for (int o = 0; o < q->oc; ++o) {
                real d = dout[o];
                if (masked && !(out[o] > 0)) d = 0;
                if (d == 0) continue;
                k->jump[q->b_off + o] += d;
                for (int64_t j = 0; j < q->in_size; ++j) {
                    k->jump[q->w_off + (int64_t)o * q->in_size + j] += d * in[j];
                    din[j] += d * W[(int64_t)o * q->in_size + j];
                }
            }
        } else {
            const real *W = w + q->w_off;
            for (int co = 0; co < q->oc; ++co)
                for (int oy = 0; oy < q->oh; ++oy)
                    for (int ox = 0; ox < q->ow; ++ox) {
                        const int64_t o = ((int64_t)co * q->oh + oy) * q->ow + ox;
                        real d = dout[o];
                        if (masked && !(out[o] > 0)) d = 0;
                        if (d == 0) continue;
                        k->jump[q->b_off + co] += d;
                        for (int ci = 0; ci < q->ic; ++ci)
                            for (int ky = 0; ky < q->k; ++ky) {
                                const int iy = oy + ky - q->pad;
                                if (iy < 0 || iy >= q->ih) continue;
                                for (int kx = 0; kx < q->k; ++kx) {
                                    const int ix = ox + kx - q->pad;
                                    if (ix < 0 || ix >= q->iw) continue;
                                    const int64_t wi = (((int64_t)co * q->ic + ci) * q->k + ky) * q->k + kx;
                                    const int64_t ii = ((int64_t)ci * q->ih + iy) * q->iw + ix;
                                    k->jump[q->w_off + wi] += d * in[ii];
                                    din[ii] += d * W[wi];
                                }
                            }
                    }
        }
    }
}

/* after carry_down: per tensor, add the largest |entry| of the jump to the allowance and
 * clear the jump again (layers 0..top only were touched) */
static void book_jump(const lay_t *lay, int top, int ev_layer, int64_t ev_unit, kink_t *k) {
    int t = 0;
    if (k->events < k->rec_cap) {
        k->rec_layer[k->events] = ev_layer; k->rec_unit[k->events] = ev_unit;
        memcpy(k->rec_jump + k->events * k->rec_P, k->jump, sizeof(real) * k->rec_P);
    }
    for (int l = 0; l <= top; ++l) {
        const lay_t *q = &lay[l];
        if (q->type == ORC_POOL) continue;
        const int64_t nw = q->b_off - q->w_off, nb = q->oc;
        double mw = 0, mb = 0;
        for (int64_t j = 0; j < nw; ++j) {
            const double a = fabs((double)k->jump[q->w_off + j]);
            if (a > mw) mw = a;
            k->jump[q->w_off + j] = 0;
        }
        for (int64_t j = 0; j < nb; ++j) {
            const double a = fabs((double)k->jump[q->b_off + j]);
            if (a > mb) mb = a;
            k->jump[q->b_off + j] = 0;
        }
        k->allow[t] += mw; k->allow[t + 1] += mb;
        t += 2;
    }
    k->events += 1;
}

/* All near-kink decisions of the sample that sample_loss_grad has just processed with the
 * same w and scratch. */
static void sample_kinks(const lay_t *lay, int L, const real *w, const scratch_t *s, kink_t *k) {
    for (int l = 0; l < L; ++l) {
        const lay_t *q = &lay[l];
        if (q->type != ORC_POOL) {
            const int wanted = q->relu || (l + 1 < L && lay[l + 1].type == ORC_POOL);
            if (!wanted) continue;
            for (int64_t o = 0; o < q->out_size; ++o) {
                real z, sc;
                preactivation(q, w, s->act[l], o, &z, &sc);
                k->scale[l][o] = sc;
                if (!q->relu || !((real)fabs((double)z) < (real)k->eps * sc)) continue;
                const real d = s->del[l + 1][o];      /* what reaches the unit from above */
                for (int64_t j = 0; j < q->out_size; ++j) k->kd[l + 1][j] = 0;
                k->kd[l + 1][o] = d;
                if (d != 0) carry_down(lay, l, 0, w, s, k);
                book_jump(lay, l, l, o, k);
            }
        } else {
            if (l == 0 || lay[l - 1].type == ORC_POOL) continue;   /* no scale to measure the gap against */
            const real *in = s->act[l];
            for (int c = 0; c < q->oc; ++c)
                for (int oy = 0; oy < q->oh; ++oy)
                    for (int ox = 0; ox < q->ow; ++ox) {
                        const int64_t o = ((int64_t)c * q->oh + oy) * q->ow + ox;
                        const int64_t best = s->amax[l][o];
                        if (!(in[best] > 0)) continue;
                        int64_t second = -1;
                        for (int dy = 0; dy < 2; ++dy)
                            for (int dx = 0; dx < 2; ++dx) {
                                const int64_t j = ((int64_t)c * q->ih + 2 * oy + dy) * q->iw + 2 * ox + dx;
                                if (j != best && (second < 0 || in[j] > in[second])) second = j;
                            }
                        real sc = k->scale[l - 1][best];
                        if (k->scale[l - 1][second] > sc) sc = k->scale[l - 1][second];
                        if (!(in[best] - in[second] < (real)k->eps * sc)) continue;
                        const real d = s->del[l + 1][o];
                        /* the runner-up takes the delta, the winner loses it; the layer below
                         * applies its own ReLU decisions to both */
                        for (int64_t j = 0; j < q->in_size; ++j) k->kd[l][j] = 0;
                        k->kd[l][second] = d;
                        k->kd[l][best] = -d;
                        if (d != 0) carry_down(lay, l - 1, 1, w, s, k);
                        book_jump(lay, l - 1, l, o, k);
                    }
        }
    }
}

static int count_tensors(const lay_t *lay, int L) {
    int t = 0;
    for (int l = 0; l < L; ++l) if (lay[l].type != ORC_POOL) t += 2;
    return t;
}

/* The near-kink decisions of ONE sample at weights w, for the tests: up to cap events with
 * the layer they belong to, the output index of the unit / pool window, and the whole jump
 * of the sample's gradient (cap x P); allow: per parameter tensor, the sum over all events
 * of the largest |entry| of the jump.  Returns the number of events found (< 0: error). */
int64_t orc_sample_kinks(const orc_model *m, const real *w, const float *x, int32_t label, double eps,
                         int64_t cap, int32_t *ev_layer, int64_t *ev_unit, real *ev_jump, double *allow) {
    lay_t lay[ORC_MAX_LAYERS]; int64_t P; scratch_t s; kink_t k;
    if (resolve(m, lay, &P)) return -1;
    const int L = m->n_layers, nt = count_tensors(lay, L);
    real *g = (real *)calloc(P, sizeof(real));
    if (!g || scratch_alloc(lay, L, &s)) { free(g); return -2; }
    if (kink_alloc(lay, L, P, nt, eps, &k)) { free(g); scratch_free(L, &s); kink_free(L, &k); return -2; }
    k.rec_cap = cap; k.rec_P = P; k.rec_layer = ev_layer; k.rec_unit = ev_unit; k.rec_jump = ev_jump;
    sample_loss_grad(lay, L, w, x, label, g, &s);
    sample_kinks(lay, L, w, &s, &k);
    for (int t = 0; t < nt; ++t) allow[t] = k.allow[t];
    const int64_t n = k.events;
    free(g); scratch_free(L, &s); kink_free(L, &k);
    return n;
}

/* ------------------------------------------------------------------------------------
 * Context
 * ---------------------------------------------------------------------------------- */
void orc_destroy(orc_ctx *C) {
    if (!C) return;
    for (int i = 0; i < C->n_queue; ++i) free(C->queue[i].U);
    free(C->queue);
    if (C->rinfo) for (int c = 0; c < C->n; ++c) {
        for (int k = 0; k < C->n_rinfo[c]; ++k) free(C->rinfo[c][k].kink_allow);
        free(C->rinfo[c]);
    }
    free(C->rinfo); free(C->n_rinfo); free(C->cap_rinfo);
    free(C->ev_tick); free(C->ev_c); free(C->ev_k);
    free(C->X); free(C->y); free(C->N);
    free(C->Wg); free(C->W);
    free(C->i_c); free(C->t_c); free(C->q_c); free(C->free_at); free(C->H);
    free(C->nbr_off); free(C->nbr); free(C->cumw);
    free(C);
}

/* Setup: every client starts from the same global model w0 (Algorithm 1, first line).
 * X[c] is client c's data set D_c, n_samples[c] rows of in_size floats; y[c] the labels.
 * The arrays are borrowed, not copied. */
orc_ctx *orc_create(const orc_model *m, int32_t n_clients, const float *const *X,
                    const int32_t *const *y, const int64_t *n_samples, const float *w0,
                    uint64_t seed) {
    orc_ctx *C = (orc_ctx *)calloc(1, sizeof *C);
    if (!C) return NULL;
    C->model = *m; C->L = m->n_layers; C->n = n_clients; C->seed = seed;
    if (n_clients < 1 || resolve(m, C->lay, &C->P)) { free(C); return NULL; }
    C->n_tensors = count_tensors(C->lay, C->L);
    C->X = (const float **)malloc(sizeof(float *) * n_clients);
    C->y = (const int32_t **)malloc(sizeof(int32_t *) * n_clients);
    C->N = (int64_t *)malloc(sizeof(int64_t) * n_clients);
    C->Wg = (real *)malloc(sizeof(real) * C->P);
    C->W = (real *)malloc(sizeof(real) * C->P * n_clients);
    C->i_c = (int64_t *)calloc(n_clients, sizeof(int64_t));
    C->t_c = (int64_t *)calloc(n_clients, sizeof(int64_t));
    C->q_c = (int64_t *)calloc(n_clients, sizeof(int64_t));
    C->free_at = (int64_t *)calloc(n_clients, sizeof(int64_t));
    C->H = (int64_t *)calloc(n_clients, sizeof(int64_t));
    C->rinfo = (rinfo_t **)calloc(n_clients, sizeof(rinfo_t *));
    C->n_rinfo = (int *)calloc(n_clients, sizeof(int));
    C->cap_rinfo = (int *)calloc(n_clients, sizeof(int));
    for (int c = 0; c < n_clients; ++c) {
        if (n_samples[c] < 1) { orc_destroy(C); return NULL; }
        C->X[c] = X[c]; C->y[c] = y[c]; C->N[c] = n_samples[c];
    }
    for (int64_t p = 0; p < C->P; ++p) C->Wg[p] = (real)w0[p];
    for (int c = 0; c < n_clients; ++c)
        for (int64_t p = 0; p < C->P; ++p) C->W[(int64_t)c * C->P + p] = C->Wg[p];
    return C;
}

static int fail(orc_ctx *C, const char *msg) { snprintf(C->err, sizeof C->err, "%s", msg); return -1; }
const char *orc_last_error(const orc_ctx *C) { return C->err; }

/* Algorithm 1 (Setup): recursion t of global round i belongs to node a(i,t) = c with
 * probability p_c = weight_c / sum of weights.  The draw is element t of the hash stream of
 * (seed, round i), mapped to [0, sum of weights) by multiply-shift; c is the node whose
 * cumulative-weight interval holds it.  Integer arithmetic only. */
int32_t orc_setup_owner(uint64_t seed, const uint64_t *cumw, int32_t n, int64_t i, int64_t t) {
    const uint64_t r = to_range(orc_stream(seed, TAG_SETUP, (uint64_t)i, (uint64_t)t), cumw[n - 1]);
    int32_t c = 0;
    while (r >= cumw[c]) ++c;
    return c;
}

/* From now on the threshold a*i + b is the GLOBAL sequence s_i (samples over all nodes) and
 * node c's round i has s_{i,c} = batch * |{ t < s_i / batch : a(i,t) = c }| samples: the
 * unit that is handed out is one recursion (one mini-batch).  weights: n non-negative
 * integers, their sum in [1, 2^32). */
int orc_set_setup(orc_ctx *C, const uint32_t *weights, uint64_t seed) {
    uint64_t sum = 0;
    for (int c = 0; c < C->n; ++c) sum += weights[c];
    if (sum < 1 || sum >= (1ULL << 32)) return fail(C, "sum of the weights must be in [1, 2^32)");
    for (int c = 0; c < C->n; ++c) if (C->i_c[c] != 0) return fail(C, "Setup comes before the first round");
    free(C->cumw);
    C->cumw = (uint64_t *)malloc(sizeof(uint64_t) * C->n);
    sum = 0;
    for (int c = 0; c < C->n; ++c) { sum += weights[c]; C->cumw[c] = sum; }
    C->setup = 1; C->setup_seed = seed;
    return 0;
}

/* s_{i,c}: the node's round length in samples (-1: s_i is not a multiple of the batch) */
static int64_t round_length(const orc_ctx *C, int c, int64_t i, int64_t a, int64_t b) {
    const int64_t s = orc_threshold(a, b, i);
    const int B = C->model.batch;
    if (s % B) return -1;
    if (!C->setup) return s;
    int64_t mine = 0;
    for (int64_t t = 0; t < s / B; ++t)
        if (orc_setup_owner(C->setup_seed, C->cumw, C->n, i, t) == c) mine += 1;
    return mine * B;
}

/* Switch to the peer-to-peer form of Algorithm 2 on an undirected topology (Section 2.2.1:
 * the neighbour list of every node is given).  nbr_off has n+1 entries; the neighbours of c
 * are nbr[nbr_off[c] .. nbr_off[c+1]), strictly ascending, never c itself, and v is listed
 * for c exactly when c is listed for v.  Only before the first round.  From then on every
 * node keeps its own model from round to round (no global model is adopted), a message
 * goes to the sender's neighbours, and the delay checkpoint looks at neighbours only. */
int orc_set_topology(orc_ctx *C, const int32_t *nbr_off, const int32_t *nbr) {
    if (C->tick != 0 || C->n_queue != 0) return fail(C, "topology must be set before the first round");
    for (int c = 0; c < C->n; ++c) if (C->i_c[c] != 0) return fail(C, "topology must be set before the first round");
    if (nbr_off[0] != 0) return fail(C, "nbr_off[0] must be 0");
    for (int c = 0; c < C->n; ++c) {
        if (nbr_off[c + 1] < nbr_off[c]) return fail(C, "nbr_off must not decrease");
        for (int32_t j = nbr_off[c]; j < nbr_off[c + 1]; ++j) {
            const int32_t v = nbr[j];
            if (v < 0 || v >= C->n || v == c) return fail(C, "neighbour out of range or self loop");
            if (j > nbr_off[c] && nbr[j - 1] >= v) return fail(C, "neighbour lists must be strictly ascending");
            int back = 0;
            for (int32_t q = nbr_off[v]; q < nbr_off[v + 1]; ++q) if (nbr[q] == c) back = 1;
            if (!back) return fail(C, "topology is not undirected");
        }
    }
    free(C->nbr_off); free(C->nbr);
    const int32_t E = nbr_off[C->n];
    C->nbr_off = (int32_t *)malloc(sizeof(int32_t) * (C->n + 1));
    C->nbr = (int32_t *)malloc(sizeof(int32_t) * (E > 0 ? E : 1));
    memcpy(C->nbr_off, nbr_off, sizeof(int32_t) * (C->n + 1));
    if (E > 0) memcpy(C->nbr, nbr, sizeof(int32_t) * E);
    C->p2p = 1;
    return 0;
}

/* One tick of local rounds (Algorithm 2, MainComputeNode, one pass of the round loop for
 * every client that is free).  A client starts round i = i_c if it is idle, has rounds
 * left and passes the delay checkpoint; it adopts the global model (server form; in the
 * peer-to-peer form it goes on from its own model), runs m = s_i / B
 * mini-batch recursions with the round's step size, and posts (c, U_i, i).
 * Outputs: the clients that ran and their round numbers, ascending client order. */
int orc_run_round(orc_ctx *C, int64_t a, int64_t b, int32_t rounds, double eta0, double beta,
                  double power, const int32_t *compute_factor, const uint8_t *is_straggler,
                  int32_t delay_min, int32_t delay_max, uint64_t delay_seed, int32_t d_max,
                  int32_t *n_finished, int32_t *fin_client, int32_t *fin_round) {
    const int B = C->model.batch;
    if (a < 0 || b < 0 || rounds < 0) return fail(C, "threshold parameters must be non-negative");
    if (delay_min < 0 || delay_max < delay_min) return fail(C, "bad delay range");
    if (!(eta0 > 0) || beta < 0) return fail(C, "bad step size parameters");
    int *act = (int *)malloc(sizeof(int) * C->n);
    int na = 0;
    for (int c = 0; c < C->n; ++c) {
        if (C->free_at[c] > C->tick || C->i_c[c] >= rounds) continue;
        /* Synchronize: d_c = max over the map H of (i - H_e); wait while d_c > d.  The map
         * holds the other nodes (server form) or the node's neighbours (peer-to-peer form).
         * A message reaches all neighbours of its sender in the same tick, so every
         * neighbour's count of v's rounds is the one number H_v. */
        if (d_max >= 0) {
            int64_t dc = 0;
            if (C->p2p) {
                for (int32_t j = C->nbr_off[c]; j < C->nbr_off[c + 1]; ++j) {
                    const int e = C->nbr[j];
                    if (C->i_c[c] - C->H[e] > dc) dc = C->i_c[c] - C->H[e];
                }
            } else {
                for (int e = 0; e < C->n; ++e)
                    if (e != c && C->i_c[c] - C->H[e] > dc) dc = C->i_c[c] - C->H[e];
            }
            if (dc > d_max) continue;
        }
        if (round_length(C, c, C->i_c[c], a, b) < 0) {
            free(act);
            return fail(C, "round length is not a multiple of the mini-batch");
        }
        if (compute_factor && compute_factor[c] < 1) { free(act); return fail(C, "compute factor < 1"); }
        act[na++] = c;
    }
    int oom = 0;
    msg_t *out = (msg_t *)calloc(na > 0 ? na : 1, sizeof(msg_t));
    rinfo_t *ri = (rinfo_t *)calloc(na > 0 ? na : 1, sizeof(rinfo_t));
#pragma omp parallel for schedule(dynamic, 1)
    for (int ai = 0; ai < na; ++ai) {
        const int c = act[ai];
        const int64_t i = C->i_c[c];
        const int64_t s = round_length(C, c, i, a, b), m = s / B;
        const double eta_d = orc_eta(eta0, beta, power, C->t_c[c]);
        const real eta = (real)eta_d;
        real *Wc = C->W + (int64_t)c * C->P;
        real *U = (real *)calloc(C->P, sizeof(real));
        real *g = (real *)malloc(sizeof(real) * C->P);
        scratch_t sc;
        kink_t kk;
        const int kinks = C->kink_eps > 0;
        if (!U || !g || scratch_alloc(C->lay, C->L, &sc)) { oom = 1; free(U); free(g); continue; }
        if (kinks && kink_alloc(C->lay, C->L, C->P, C->n_tensors, C->kink_eps, &kk)) { oom = 1; free(U); free(g); continue; }
        if (!C->p2p)
            for (int64_t p = 0; p < C->P; ++p) Wc[p] = C->Wg[p];      /* adopt the broadcast */
        real loss_sum = 0;
        for (int64_t u = 0; u < m; ++u) {
            for (int64_t p = 0; p < C->P; ++p) g[p] = 0;
            real lstep = 0;
            for (int j = 0; j < B; ++j) {
                int32_t idx = orc_sample_index(C->seed, c, C->q_c[c] + u * B + j, C->N[c]);
                lstep += sample_loss_grad(C->lay, C->L, Wc, C->X[c] + (int64_t)idx * C->lay[0].in_size,
                                          C->y[c][idx], g, &sc);
                if (kinks) sample_kinks(C->lay, C->L, Wc, &sc, &kk);
            }
            for (int64_t p = 0; p < C->P; ++p) g[p] /= (real)B;
            for (int64_t p = 0; p < C->P; ++p) { Wc[p] -= eta * g[p]; U[p] += g[p]; }
            loss_sum += lstep / (real)B;
        }
        scratch_free(C->L, &sc);
        free(g);
        if (kinks) {
            /* a sample's gradient enters the recursion divided by the mini-batch size */
            ri[ai].kink_events = kk.events;
            ri[ai].kink_allow = kk.allow;
            for (int t = 0; t < C->n_tensors; ++t) ri[ai].kink_allow[t] /= (double)B;
            kk.allow = NULL;
            kink_free(C->L, &kk);
        }
        const int64_t f = compute_factor ? compute_factor[c] : 1;
        const int64_t delta = (is_straggler && is_straggler[c])
                                  ? orc_net_delay(delay_seed, c, (int32_t)i, delay_min, delay_max) : 0;
        out[ai].c = c; out[ai].k = (int32_t)i; out[ai].eta = eta_d; out[ai].U = U;
        out[ai].arrival = C->tick + f - 1 + delta;
        ri[ai].s = s; ri[ai].m = m; ri[ai].q0 = C->q_c[c]; ri[ai].t0 = C->t_c[c];
        ri[ai].start_tick = C->tick; ri[ai].arrival = out[ai].arrival; ri[ai].eta = eta_d;
        ri[ai].loss = m > 0 ? (double)(loss_sum / (real)m) : 0.0;
    }
    if (oom) {
        for (int ai = 0; ai < na; ++ai) free(out[ai].U);
        free(out); free(ri); free(act);
        return fail(C, "out of memory");
    }
    for (int ai = 0; ai < na; ++ai) {
        const int c = act[ai];
        const int64_t f = compute_factor ? compute_factor[c] : 1;
        if (C->n_queue == C->cap_queue) {
            C->cap_queue = C->cap_queue ? 2 * C->cap_queue : 64;
            C->queue = (msg_t *)realloc(C->queue, sizeof(msg_t) * C->cap_queue);
        }
        C->queue[C->n_queue++] = out[ai];
        if (C->n_rinfo[c] == C->cap_rinfo[c]) {
            C->cap_rinfo[c] = C->cap_rinfo[c] ? 2 * C->cap_rinfo[c] : 64;
            C->rinfo[c] = (rinfo_t *)realloc(C->rinfo[c], sizeof(rinfo_t) * C->cap_rinfo[c]);
        }
        C->rinfo[c][C->n_rinfo[c]++] = ri[ai];
        C->t_c[c] += ri[ai].m; C->q_c[c] += ri[ai].s; C->i_c[c] += 1; C->free_at[c] = C->tick + f;
        if (fin_client) fin_client[ai] = c;
        if (fin_round) fin_round[ai] = out[ai].k;
    }
    if (n_finished) *n_finished = na;
    free(out); free(ri); free(act);
    return 0;
}

/* The message with the smallest (round, client) among those arriving in this tick; -1: none */
static int next_arrival(const orc_ctx *C) {
    int best = -1;
    for (int j = 0; j < C->n_queue; ++j) {
        if (C->queue[j].arrival != C->tick) continue;
        if (best < 0 || C->queue[j].k < C->queue[best].k ||
            (C->queue[j].k == C->queue[best].k && C->queue[j].c < C->queue[best].c)) best = j;
    }
    return best;
}

static void log_event(orc_ctx *C, int32_t c, int32_t k) {
    if (C->n_ev == C->cap_ev) {
        C->cap_ev = C->cap_ev ? 2 * C->cap_ev : 256;
        C->ev_tick = (int64_t *)realloc(C->ev_tick, sizeof(int64_t) * C->cap_ev);
        C->ev_c = (int32_t *)realloc(C->ev_c, sizeof(int32_t) * C->cap_ev);
        C->ev_k = (int32_t *)realloc(C->ev_k, sizeof(int32_t) * C->cap_ev);
    }
    C->ev_tick[C->n_ev] = C->tick; C->ev_c[C->n_ev] = c; C->ev_k[C->n_ev] = k; C->n_ev++;
}

/* Server form of Receive: every message whose arrival tick is the current tick is
 * applied, in (round, client) ascending order, as Wg -= (agg_scale * eta_k) * U with the
 * SENDER's round step size, and H_c += 1.  Then the tick advances. */
int orc_server_aggregate(orc_ctx *C, double agg_scale, int32_t *n_applied, int32_t *app_client,
                         int32_t *app_round) {
    if (C->p2p) return fail(C, "peer-to-peer form: use orc_receive");
    int na = 0;
    for (;;) {
        const int best = next_arrival(C);
        if (best < 0) break;
        msg_t *q = &C->queue[best];
        const real scale = (real)(agg_scale * q->eta);
        for (int64_t p = 0; p < C->P; ++p) C->Wg[p] -= scale * q->U[p];
        C->H[q->c] += 1;
        log_event(C, q->c, q->k);
        if (app_client) app_client[na] = q->c;
        if (app_round) app_round[na] = q->k;
        na++;
        free(q->U);
        C->queue[best] = C->queue[--C->n_queue];
    }
    if (n_applied) *n_applied = na;
    C->tick += 1;
    return 0;
}

/* Receive as Algorithm 2 prints it: a message (v, U, k) arriving in this tick is applied
 * by every neighbour r of v to its own model, w_r -= (scale * eta_k) * U, with the step
 * size of the sender's round k (scale = 1 is the paper's rule), and H_v += 1.  Messages
 * are taken in (round, sender) ascending order, so each node applies its arrivals in
 * that order.  A node whose round occupies several ticks did its recursions in the
 * round's first tick; what arrives meanwhile lands on the model as that round left it.
 * Outputs: the messages delivered (sender, round).  Then the tick advances. */
int orc_receive(orc_ctx *C, double scale, int32_t *n_applied, int32_t *app_sender, int32_t *app_round) {
    if (!C->p2p) return fail(C, "no topology set: use orc_server_aggregate");
    int na = 0;
    for (;;) {
        const int best = next_arrival(C);
        if (best < 0) break;
        msg_t *q = &C->queue[best];
        const real sc = (real)(scale * q->eta);
        for (int32_t j = C->nbr_off[q->c]; j < C->nbr_off[q->c + 1]; ++j) {
            real *Wr = C->W + (int64_t)C->nbr[j] * C->P;
            for (int64_t p = 0; p < C->P; ++p) Wr[p] -= sc * q->U[p];
        }
        C->H[q->c] += 1;
        log_event(C, q->c, q->k);
        if (app_sender) app_sender[na] = q->c;
        if (app_round) app_round[na] = q->k;
        na++;
        free(q->U);
        C->queue[best] = C->queue[--C->n_queue];
    }
    if (n_applied) *n_applied = na;
    C->tick += 1;
    return 0;
}

int orc_all_done(const orc_ctx *C, int32_t rounds) {
    if (C->n_queue) return 0;
    for (int c = 0; c < C->n; ++c) if (C->i_c[c] < rounds) return 0;
    return 1;
}
int64_t orc_tick(const orc_ctx *C) { return C->tick; }
int64_t orc_queue_len(const orc_ctx *C) { return C->n_queue; }
int64_t orc_params(const orc_ctx *C) { return C->P; }

/* U of a message that is still in flight (posted, not yet applied) */
int orc_get_U(orc_ctx *C, int32_t c, int32_t k, real *dst) {
    for (int j = 0; j < C->n_queue; ++j)
        if (C->queue[j].c == c && C->queue[j].k == k) {
            memcpy(dst, C->queue[j].U, sizeof(real) * C->P);
            return 0;
        }
    return fail(C, "no such message in flight");
}
/* client < 0: the global model; else the client's local model as its last round left it */
int orc_get_weights(orc_ctx *C, int32_t c, real *dst) {
    if (c >= C->n) return fail(C, "client out of range");
    memcpy(dst, c < 0 ? C->Wg : C->W + (int64_t)c * C->P, sizeof(real) * C->P);
    return 0;
}
/* overwrite the global model (client < 0) or a client's local model: lets a test restart
 * both sides of a comparison from the same state */
int orc_set_weights(orc_ctx *C, int32_t c, const real *src) {
    if (c >= C->n) return fail(C, "client out of range");
    memcpy(c < 0 ? C->Wg : C->W + (int64_t)c * C->P, src, sizeof(real) * C->P);
    return 0;
}
/* bookkeeping of round k of client c: s, m, q0, t0, start tick, arrival tick; eta, loss */
int orc_get_round_info(orc_ctx *C, int32_t c, int32_t k, int64_t *ints6, double *dbl2) {
    if (c < 0 || c >= C->n || k < 0 || k >= C->n_rinfo[c]) return fail(C, "no such round");
    const rinfo_t *r = &C->rinfo[c][k];
    ints6[0] = r->s; ints6[1] = r->m; ints6[2] = r->q0; ints6[3] = r->t0;
    ints6[4] = r->start_tick; ints6[5] = r->arrival;
    dbl2[0] = r->eta; dbl2[1] = r->loss;
    return 0;
}
/* Kink analysis on (eps > 0) or off for the rounds that follow: see the section "Kinks". */
void orc_set_kink_eps(orc_ctx *C, double eps) { C->kink_eps = eps; }
int32_t orc_n_tensors(const orc_ctx *C) { return C->n_tensors; }
/* of round k of client c, run with the analysis on: the number of near-kink decisions and,
 * per parameter tensor (weights, bias of every conv / dense layer, in order), the sum of the
 * jumps of the mini-batch gradient they could cause (entries of g, i.e. already / B) */
int orc_get_round_kinks(orc_ctx *C, int32_t c, int32_t k, int64_t *events, double *allow) {
    if (c < 0 || c >= C->n || k < 0 || k >= C->n_rinfo[c]) return fail(C, "no such round");
    const rinfo_t *r = &C->rinfo[c][k];
    if (!r->kink_allow) return fail(C, "round ran without the kink analysis");
    *events = r->kink_events;
    for (int t = 0; t < C->n_tensors; ++t) allow[t] = r->kink_allow[t];
    return 0;
}
int64_t orc_event_count(const orc_ctx *C) { return C->n_ev; }
void orc_get_events(const orc_ctx *C, int64_t *tick, int32_t *c, int32_t *k) {
    for (int64_t j = 0; j < C->n_ev; ++j) { tick[j] = C->ev_tick[j]; c[j] = C->ev_c[j]; k[j] = C->ev_k[j]; }
}
int64_t orc_history(const orc_ctx *C, int32_t c) { return C->H[c]; }
int orc_real_bytes(void) { return (int)sizeof(real); }
