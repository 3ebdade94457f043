/*
 * snn_oracle.c -- plain, slow, single-purpose CPU reference for BPTT through a
 * multi-layer leaky-integrate-and-fire (LIF) spiking RNN under the four state
 * storage strategies of the paper (Fig. 1; Sections "Standard Checkpointing",
 * "Remote Checkpointing", "Double Checkpointing").
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the checker the GPU library is
 * compared against; it is never part of the product path and shares no code,
 * header, table or helper with it.  Only tests, the smoke check and the
 * CPU-baseline leg of the benchmark may call it.
 *
 * The paper defines the storage/recompute schedules and the memory and time
 * closed forms, but prints no neuron equations (Section "BPTT based SNN
 * training on the IPU" defers to its reference [Finkbeiner et al. 2023]).  The
 * model below is the one the benchmark configuration fixes:
 *
 *   layers l = 1..L, s^0_t = input spikes, v_0 = s_0 = u_0 = 0, t = 1..T
 *     I^l_t = sum_{j} s^{l-1}_t[j] * W_in^l[j,:]  +  sum_{j} s^l_{t-1}[j] * W_rec^l[j,:]
 *     v^l_t = (alpha * v^l_{t-1} - theta * s^l_{t-1}) + I^l_t
 *     s^l_t = H(v^l_t - theta)           (strict: fires iff v > theta)
 *     u_t   = beta * u_{t-1} + sum_j s^L_t[j] * W_out[j,:]
 *     ubar  = (1/T) sum_t u_t
 *     loss  = (1/B) sum_b [ logsumexp(ubar_b) - ubar_b[y_b] ]
 *
 *   backward, surrogate derivative sigma'(x) = 1 / (1 + k|x|)^2  (k = surr_beta):
 *     g        = (softmax(ubar) - onehot(y)) / (B*T)     (labelled class: - sum of the other classes' softmax)
 *     du_t     = beta * du_{t+1} + g
 *     dW_out[j,:]  += s^L_t[j] * du_t
 *     ds^l_t   = (l==L ? W_out du_t : W_in^{l+1} dv^{l+1}_t) + W_rec^l dv^l_{t+1} - theta * dv^l_{t+1}
 *     dv^l_t   = alpha * dv^l_{t+1} + sigma'(v^l_t - theta) * ds^l_t
 *     dW_in^l[j,:]  += s^{l-1}_t[j] * dv^l_t
 *     dW_rec^l[j,:] += s^l_{t-1}[j] * dv^l_t
 *   optional window w > 0 (not in the paper; the compact-support variant that makes the spike
 *   derivative sparse): sigma'(x) is replaced by 0 wherever |x| >= w.
 *
 * Every sum over presynaptic neurons runs over ascending j starting from 0 and
 * skips entries with s[j] == 0; the input sum and the recurrent sum are formed
 * separately and then added.  The file must be compiled with
 * -ffp-contract=off so that no multiply-add is fused.
 *
 * "smooth" mode replaces H by S(x) = x / (1 + k|x|), whose derivative is exactly
 * sigma'; the whole network is then differentiable and the backward pass can be
 * checked against finite differences.  The same code path serves both modes:
 * spikes are stored as REAL values (0/1 in Heaviside mode).
 *
 * "forced" mode takes the hidden spike trains as an input instead of
 * thresholding (this is exactly what a recompute pass does: Section "Standard
 * Checkpointing" and the Discussion say spikes of the full sequence are kept
 * and only the states are recomputed).
 *
 * "forced states" mode additionally takes the membrane potentials v_t as inputs
 * (full storage only).  It exists for one purpose: evaluating the backward pass
 * in double precision on the exact fp32 forward trajectory, which separates the
 * rounding error of a backward implementation from the (shared, bit-identical)
 * rounding of the fp32 forward states.
 *
 * Storage strategies (names as in the caption of Fig. 1):
 *   STANDARD  every state x_1..x_T is kept (eq. M_Base).
 *   CHUNK     x_c kept for c in {0,F,2F,..} < T in local memory, one chunk buffer
 *             of F states; each chunk is recomputed from its checkpoint then
 *             back-propagated (eq. M_Standard, T_Standard).
 *   REMOTE    the same checkpoints, every C steps, but kept in "remote" memory;
 *             one is loaded before each chunk is recomputed (eq. M_Remote).
 *   DOUBLE    coarse checkpoints every C steps in remote memory; for each coarse
 *             segment one is loaded, Re-Forward_1 rebuilds fine checkpoints every
 *             F steps, then Re-Forward_2 rebuilds each fine chunk which is then
 *             back-propagated (eq. M_Double, T_Double, N_c).
 *   HIER      Section "Hierarchical Checkpointing": checkpoints every F steps are
 *             moved to and from remote memory in batches of C = nb_local checkpoints
 *             (one transfer per batch); the last batch never leaves local memory
 *             (eq. M_Hier).  The paper's count of transfers is read from its prose:
 *             one write and one read per batch except the last, N_c = 2 (batches - 1).
 *
 * All work is organised per batch element (forward, recompute and the adjoint
 * recurrence are independent across the batch; only weight gradients and the
 * loss sum over it).  With nthreads > 1 batch elements are distributed over
 * OpenMP threads, each with private gradient accumulators that are reduced in
 * thread order.
 *
 * Compile twice: -DREAL=float -DSUFFIX=f32 and -DREAL=double -DSUFFIX=f64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef REAL
#define REAL double
#endif
#ifndef SUFFIX
#define SUFFIX f64
#endif
#define CAT_(a, b) a##_##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, SUFFIX)

enum { STRAT_STANDARD = 0, STRAT_CHUNK = 1, STRAT_REMOTE = 2, STRAT_DOUBLE = 3, STRAT_HIER = 4 };
enum { MODE_HEAVISIDE = 0, MODE_SMOOTH = 1 };

/* schedule event codes written to the optional event log (batch element 0 only) */
enum {
  EV_SAVE_LOCAL = 1,  /* a = checkpoint index c (state x_c kept in local memory)   */
  EV_SAVE_REMOTE = 2, /* a = c (state x_c written to remote memory)                */
  EV_LOAD_REMOTE = 3, /* a = c (state x_c read back from remote memory)            */
  EV_REFWD1 = 4,      /* recompute (a, b], keeping only fine checkpoints           */
  EV_KEEP_FINE = 5,   /* a = c (fine checkpoint x_c kept during Re-Forward_1)      */
  EV_REFWD2 = 6,      /* recompute (a, b] into the chunk buffer                    */
  EV_BACKWARD = 7,    /* back-propagate steps a, a-1, ..., b  (a >= b)             */
  EV_SAVE_BATCH = 8,  /* a = first checkpoint index c of a batch written to remote, b = count */
  EV_LOAD_BATCH = 9   /* a = first checkpoint index c of a batch read back, b = count        */
};

typedef struct {
  int32_t n_in, n_layers, n_out, T, B;
  const int32_t *n_hidden; /* [n_layers] */
  double alpha, beta, theta, surr_beta;
  int32_t mode;     /* MODE_HEAVISIDE / MODE_SMOOTH */
  int32_t forced;   /* 1: hidden spikes are inputs (spikes[] read, not written) */
  int32_t strategy; /* STRAT_* */
  int32_t C, F;     /* coarse (remote) and fine (local) checkpoint intervals */
  int32_t nthreads; /* OpenMP threads over the batch (1 = plain loop) */
  int32_t forced_states; /* 1: membrane potentials are inputs too (vtraj[] read, STANDARD only) */
  double surr_window;    /* w > 0: sigma'(x) = 0 wherever |x| >= w (Heaviside mode only); <= 0: no window */
} oracle_cfg;

typedef struct {
  int64_t fwd_steps;     /* membrane updates done in the forward pass, per batch element */
  int64_t refwd1_steps;  /* ... in Re-Forward_1 passes                                   */
  int64_t refwd2_steps;  /* ... in Re-Forward_2 / single recompute passes                */
  int64_t bwd_steps;     /* backward steps                                               */
  int64_t remote_writes; /* states written to remote memory                              */
  int64_t remote_reads;  /* states read from remote memory                               */
  int64_t local_slots;   /* states resident in local memory at the peak                  */
  int64_t remote_slots;  /* states resident in remote memory                             */
  int64_t n_events;      /* entries written to the event log                             */
  int32_t threads_used;
} oracle_stats;

/* ------------------------------------------------------------------------- */

typedef struct {
  const oracle_cfg *c;
  int L, SN;    /* layers, sum of hidden sizes */
  int *off;     /* [L+1] offset of layer l's neurons inside a state vector */
  const REAL *const *W_in, *const *W_rec;
  const REAL *W_out;
  REAL alpha, beta, theta, k;
  float win; /* surrogate window, <= 0 for none */
} net_t;

static int npre(const net_t *n, int l) { return l == 0 ? n->c->n_in : n->c->n_hidden[l - 1]; }

/* S(x) or H(x) */
static REAL spike_fn(const net_t *n, REAL x) {
  if (n->c->mode == MODE_SMOOTH) return x / ((REAL)1 + n->k * (REAL)fabs((double)x));
  return x > (REAL)0 ? (REAL)1 : (REAL)0;
}
static REAL surrogate(const net_t *n, REAL x) {
  /* The window test is a decision, so it is taken in single precision whatever REAL is: on an
   * fp32 trajectory x = v - theta rounds to the float the single-precision build compares. */
  if (n->win > 0.0f && !(fabsf((float)x) < n->win)) return (REAL)0;
  REAL d = (REAL)1 + n->k * (REAL)fabs((double)x);
  return (REAL)1 / (d * d);
}

/* pointer to spikes of layer l (0 = input) at step t (1..T) of batch element b;
 * step 0 is the all-zero initial condition and is never stored. */
typedef struct {
  const uint8_t *in;  /* [T][B][n_in] */
  REAL *const *hid;   /* hid[l-1] : [T][B][N_l] */
} spikes_t;

/* One membrane update of layer l (1-based) for one batch element:
 * v_out = (alpha * v_prev - theta * s_prev) + (I_in + I_rec), with the two
 * currents summed separately over ascending presynaptic index. */
static void lif_membrane_update(const net_t *n, const spikes_t *sp, int b, int t, int l,
                                const REAL *v_prev, REAL *v_out, REAL *I_in, REAL *I_rec) {
  const int B = n->c->B, N = n->c->n_hidden[l - 1], P = npre(n, l - 1);
  const REAL *Wi = n->W_in[l - 1], *Wr = n->W_rec[l - 1];
  for (int i = 0; i < N; ++i) { I_in[i] = (REAL)0; I_rec[i] = (REAL)0; }
  if (l == 1) {
    const uint8_t *s = sp->in + ((size_t)(t - 1) * B + b) * P;
    for (int j = 0; j < P; ++j)
      if (s[j])
        for (int i = 0; i < N; ++i) I_in[i] = I_in[i] + (REAL)s[j] * Wi[(size_t)j * N + i];
  } else {
    const REAL *s = sp->hid[l - 2] + ((size_t)(t - 1) * B + b) * P;
    for (int j = 0; j < P; ++j)
      if (s[j] != (REAL)0)
        for (int i = 0; i < N; ++i) I_in[i] = I_in[i] + s[j] * Wi[(size_t)j * N + i];
  }
  const REAL *sr = t >= 2 ? sp->hid[l - 1] + ((size_t)(t - 2) * B + b) * N : NULL;
  if (sr)
    for (int j = 0; j < N; ++j)
      if (sr[j] != (REAL)0)
        for (int i = 0; i < N; ++i) I_rec[i] = I_rec[i] + sr[j] * Wr[(size_t)j * N + i];
  for (int i = 0; i < N; ++i) {
    REAL a = n->alpha * v_prev[i];
    if (sr && sr[i] != (REAL)0) a = a - n->theta * sr[i];
    v_out[i] = a + (I_in[i] + I_rec[i]);
  }
}

/* x_{t-1} -> x_t for every layer.  generate != 0: spikes of step t are produced
 * by thresholding (the forward pass); otherwise they are read from storage (a
 * recompute pass, which skips spike generation). */
static void advance_state(const net_t *n, const spikes_t *sp, int b, int t, const REAL *x_prev,
                          REAL *x_out, REAL *scratch, int generate) {
  const int B = n->c->B;
  for (int l = 1; l <= n->L; ++l) {
    const int N = n->c->n_hidden[l - 1];
    lif_membrane_update(n, sp, b, t, l, x_prev + n->off[l - 1], x_out + n->off[l - 1], scratch,
                        scratch + N);
    if (generate) {
      REAL *s = sp->hid[l - 1] + ((size_t)(t - 1) * B + b) * N;
      for (int i = 0; i < N; ++i) s[i] = spike_fn(n, x_out[n->off[l - 1] + i] - n->theta);
    }
  }
}

typedef struct {
  REAL *dW_in[16], *dW_rec[16], *dW_out;
} grads_t;

/* adjoint state carried from step t+1 to step t */
typedef struct {
  REAL *dv_next; /* [SN] dv_{t+1}  */
  REAL *dv_cur;  /* [SN] dv_t      */
  REAL *du;      /* [n_out]        */
  REAL *ds;      /* scratch [max N] */
} adj_t;

/* One backward step at time t for batch element b, given the state x_t. */
static void backward_step(const net_t *n, const spikes_t *sp, int b, int t, const REAL *x_t,
                          const REAL *g, adj_t *a, grads_t *G) {
  const int B = n->c->B, L = n->L, O = n->c->n_out;
  /* readout adjoint and dW_out */
  for (int o = 0; o < O; ++o) a->du[o] = n->beta * a->du[o] + g[o];
  {
    const int N = n->c->n_hidden[L - 1];
    const REAL *s = sp->hid[L - 1] + ((size_t)(t - 1) * B + b) * N;
    for (int j = 0; j < N; ++j)
      if (s[j] != (REAL)0)
        for (int o = 0; o < O; ++o) G->dW_out[(size_t)j * O + o] += s[j] * a->du[o];
  }
  for (int l = L; l >= 1; --l) {
    const int N = n->c->n_hidden[l - 1], P = npre(n, l - 1);
    const REAL *dvn = a->dv_next + n->off[l - 1];
    REAL *dvc = a->dv_cur + n->off[l - 1];
    const REAL *Wr = n->W_rec[l - 1];
    for (int j = 0; j < N; ++j) {
      REAL up = (REAL)0, rec = (REAL)0;
      if (l == L) {
        for (int o = 0; o < O; ++o) up = up + n->W_out[(size_t)j * O + o] * a->du[o];
      } else {
        const int M = n->c->n_hidden[l];
        const REAL *Wn = n->W_in[l]; /* W_in^{l+1} : [N_l][N_{l+1}] */
        const REAL *dvu = a->dv_cur + n->off[l];
        for (int i = 0; i < M; ++i) up = up + Wn[(size_t)j * M + i] * dvu[i];
      }
      for (int i = 0; i < N; ++i) rec = rec + Wr[(size_t)j * N + i] * dvn[i];
      a->ds[j] = (up + rec) - n->theta * dvn[j];
    }
    for (int j = 0; j < N; ++j)
      dvc[j] = n->alpha * dvn[j] + surrogate(n, x_t[n->off[l - 1] + j] - n->theta) * a->ds[j];
    /* weight gradients: rows of presynaptic neurons that were active */
    if (l == 1) {
      const uint8_t *s = sp->in + ((size_t)(t - 1) * B + b) * P;
      for (int j = 0; j < P; ++j)
        if (s[j])
          for (int i = 0; i < N; ++i) G->dW_in[0][(size_t)j * N + i] += (REAL)s[j] * dvc[i];
    } else {
      const REAL *s = sp->hid[l - 2] + ((size_t)(t - 1) * B + b) * P;
      for (int j = 0; j < P; ++j)
        if (s[j] != (REAL)0)
          for (int i = 0; i < N; ++i) G->dW_in[l - 1][(size_t)j * N + i] += s[j] * dvc[i];
    }
    if (t >= 2) {
      const REAL *s = sp->hid[l - 1] + ((size_t)(t - 2) * B + b) * N;
      for (int j = 0; j < N; ++j)
        if (s[j] != (REAL)0)
          for (int i = 0; i < N; ++i) G->dW_rec[l - 1][(size_t)j * N + i] += s[j] * dvc[i];
    }
  }
  /* dv_t becomes dv_{t+1} of the next (earlier) step */
  REAL *tmp = a->dv_next; a->dv_next = a->dv_cur; a->dv_cur = tmp;
}

typedef struct {
  int32_t *buf; int64_t cap, n; int on;
} evlog_t;
static void ev(evlog_t *e, int code, int a, int b) {
  if (!e->on) return;
  if (e->buf && e->n < e->cap) { e->buf[3 * e->n] = code; e->buf[3 * e->n + 1] = a; e->buf[3 * e->n + 2] = b; }
  e->n++;
}

static int imin(int a, int b) { return a < b ? a : b; }
static int cdiv(int a, int b) { return (a + b - 1) / b; }

/* Whole training step for one batch element b.  Returns this element's loss
 * term; adds its weight-gradient contribution into G. */
static double bptt_one(const net_t *n, const spikes_t *sp, const int32_t *labels, int b,
                       REAL *ubar_out /*[n_out]*/, REAL *const *vtraj /* optional [L] of [T][B][N_l] */,
                       grads_t *G, int do_backward, oracle_stats *st, evlog_t *elog) {
  const oracle_cfg *c = n->c;
  const int T = c->T, B = c->B, L = n->L, SN = n->SN, O = c->n_out;
  const int strat = c->strategy, C = c->C, F = c->F;
  int maxN = O;
  for (int l = 0; l < L; ++l) if (c->n_hidden[l] > maxN) maxN = c->n_hidden[l];
  REAL *scratch = (REAL *)calloc((size_t)2 * maxN, sizeof(REAL));

  /* ---- storage owned by this strategy -------------------------------- */
  /* local memory */
  REAL *traj = NULL;   /* STANDARD: x_1..x_T                                   */
  REAL *ckpt = NULL;   /* CHUNK: local checkpoints x_0, x_F, ...               */
  REAL *chunk = NULL;  /* CHUNK/REMOTE/DOUBLE: chunk buffer                     */
  REAL *fine = NULL;   /* DOUBLE: fine checkpoints of the current coarse segment*/
  REAL *loaded = NULL; /* REMOTE/DOUBLE: the one checkpoint fetched from remote */
  /* remote memory */
  REAL *remote = NULL;
  int n_ckpt = 0, chunk_len = 0, n_fine = 0;
  int64_t local_slots = 0, remote_slots = 0;
  if (strat == STRAT_STANDARD) {
    traj = (REAL *)malloc((size_t)T * SN * sizeof(REAL)); local_slots = T;
  } else if (strat == STRAT_CHUNK) {
    n_ckpt = cdiv(T, F); chunk_len = F;
    ckpt = (REAL *)malloc((size_t)n_ckpt * SN * sizeof(REAL));
    chunk = (REAL *)malloc((size_t)chunk_len * SN * sizeof(REAL));
    local_slots = (int64_t)n_ckpt + chunk_len;
  } else if (strat == STRAT_REMOTE) {
    n_ckpt = cdiv(T, C); chunk_len = C;
    remote = (REAL *)malloc((size_t)n_ckpt * SN * sizeof(REAL));
    chunk = (REAL *)malloc((size_t)chunk_len * SN * sizeof(REAL));
    loaded = (REAL *)malloc((size_t)SN * sizeof(REAL));
    local_slots = (int64_t)chunk_len + 1; remote_slots = n_ckpt;
  } else if (strat == STRAT_HIER) {
    n_ckpt = cdiv(T, F); chunk_len = F; /* C = nb_local checkpoints per batch */
    const int n_batches = cdiv(n_ckpt, C);
    ckpt = (REAL *)malloc((size_t)C * SN * sizeof(REAL));                       /* the local batch */
    chunk = (REAL *)malloc((size_t)chunk_len * SN * sizeof(REAL));
    remote = (REAL *)malloc((size_t)(n_batches > 1 ? (n_batches - 1) * C : 1) * SN * sizeof(REAL));
    local_slots = (int64_t)chunk_len + C; remote_slots = (int64_t)(n_batches - 1) * C;
  } else {
    n_ckpt = cdiv(T, C); chunk_len = F; n_fine = cdiv(C, F); /* fine[0] mirrors the loaded coarse one and is not counted twice */
    remote = (REAL *)malloc((size_t)n_ckpt * SN * sizeof(REAL));
    chunk = (REAL *)malloc((size_t)chunk_len * SN * sizeof(REAL));
    fine = (REAL *)malloc((size_t)n_fine * SN * sizeof(REAL));
    loaded = (REAL *)malloc((size_t)SN * sizeof(REAL));
    local_slots = (int64_t)chunk_len + (n_fine - 1) + 1; remote_slots = n_ckpt;
  }
  st->local_slots = local_slots; st->remote_slots = remote_slots;

  /* ---- forward pass ---------------------------------------------------- */
  REAL *x = (REAL *)calloc((size_t)SN, sizeof(REAL));   /* x_{t-1} */
  REAL *xn = (REAL *)calloc((size_t)SN, sizeof(REAL));  /* x_t     */
  REAL *u = (REAL *)calloc((size_t)O, sizeof(REAL));
  REAL *usum = (REAL *)calloc((size_t)O, sizeof(REAL));
  for (int t = 1; t <= T; ++t) {
    /* x (= x_{t-1}) is a checkpoint if t-1 is a multiple of the interval */
    if (strat == STRAT_CHUNK && (t - 1) % F == 0) {
      memcpy(ckpt + (size_t)((t - 1) / F) * SN, x, (size_t)SN * sizeof(REAL));
      ev(elog, EV_SAVE_LOCAL, t - 1, 0);
    }
    if (strat == STRAT_HIER && (t - 1) % F == 0) {
      const int k = (t - 1) / F, n_batches = cdiv(n_ckpt, C);
      memcpy(ckpt + (size_t)(k % C) * SN, x, (size_t)SN * sizeof(REAL));
      ev(elog, EV_SAVE_LOCAL, t - 1, 0);
      if (k % C == C - 1 && k / C < n_batches - 1) { /* batch complete and not the last one: one transfer */
        memcpy(remote + (size_t)(k / C) * C * SN, ckpt, (size_t)C * SN * sizeof(REAL));
        st->remote_writes++; ev(elog, EV_SAVE_BATCH, (k / C) * C * F, C);
      }
    }
    if ((strat == STRAT_REMOTE || strat == STRAT_DOUBLE) && (t - 1) % C == 0) {
      memcpy(remote + (size_t)((t - 1) / C) * SN, x, (size_t)SN * sizeof(REAL));
      st->remote_writes++; ev(elog, EV_SAVE_REMOTE, t - 1, 0);
    }
    advance_state(n, sp, b, t, x, xn, scratch, !c->forced);
    st->fwd_steps++;
    if (c->forced_states)
      for (int l = 0; l < L; ++l)
        memcpy(xn + n->off[l], vtraj[l] + ((size_t)(t - 1) * B + b) * c->n_hidden[l],
               (size_t)c->n_hidden[l] * sizeof(REAL));
    if (strat == STRAT_STANDARD) memcpy(traj + (size_t)(t - 1) * SN, xn, (size_t)SN * sizeof(REAL));
    if (vtraj && !c->forced_states)
      for (int l = 0; l < L; ++l)
        memcpy(vtraj[l] + ((size_t)(t - 1) * B + b) * c->n_hidden[l], xn + n->off[l],
               (size_t)c->n_hidden[l] * sizeof(REAL));
    /* readout */
    {
      const int N = c->n_hidden[L - 1];
      const REAL *s = sp->hid[L - 1] + ((size_t)(t - 1) * B + b) * N;
      for (int o = 0; o < O; ++o) scratch[o] = (REAL)0;
      for (int j = 0; j < N; ++j)
        if (s[j] != (REAL)0)
          for (int o = 0; o < O; ++o) scratch[o] = scratch[o] + s[j] * n->W_out[(size_t)j * O + o];
      for (int o = 0; o < O; ++o) { u[o] = n->beta * u[o] + scratch[o]; usum[o] = usum[o] + u[o]; }
    }
    REAL *tmp = x; x = xn; xn = tmp;
  }

  /* ---- loss and its gradient w.r.t. every u_t -------------------------- */
  REAL *g = (REAL *)calloc((size_t)O, sizeof(REAL));
  double loss_b;
  {
    REAL m;
    for (int o = 0; o < O; ++o) ubar_out[o] = usum[o] / (REAL)T;
    m = ubar_out[0];
    for (int o = 1; o < O; ++o) if (ubar_out[o] > m) m = ubar_out[o];
    REAL z = (REAL)0;
    for (int o = 0; o < O; ++o) z = z + (REAL)exp((double)(ubar_out[o] - m));
    REAL lse = m + (REAL)log((double)z);
    loss_b = (double)(lse - ubar_out[labels[b]]);
    /* softmax - onehot.  The softmax sums to one, so the labelled class's entry, softmax_y - 1, is minus the
     * sum of the other classes' probabilities; it is formed that way because the difference of two numbers
     * near one loses every digit once the softmax is confident (1 - softmax_y below the rounding step of
     * REAL), while the sum of the small probabilities keeps them. */
    REAL others = (REAL)0;
    for (int o = 0; o < O; ++o)
      if (o != labels[b]) others = others + (REAL)exp((double)(ubar_out[o] - m)) / z;
    for (int o = 0; o < O; ++o) {
      REAL p = (REAL)exp((double)(ubar_out[o] - m)) / z;
      g[o] = (o == labels[b] ? -others : p) / ((REAL)B * (REAL)T);
    }
  }

  /* ---- backward pass ---------------------------------------------------- */
  if (do_backward) {
    adj_t a;
    a.dv_next = (REAL *)calloc((size_t)SN, sizeof(REAL));
    a.dv_cur = (REAL *)calloc((size_t)SN, sizeof(REAL));
    a.du = (REAL *)calloc((size_t)O, sizeof(REAL));
    a.ds = (REAL *)calloc((size_t)maxN, sizeof(REAL));
    if (strat == STRAT_STANDARD) {
      ev(elog, EV_BACKWARD, T, 1);
      for (int t = T; t >= 1; --t) { backward_step(n, sp, b, t, traj + (size_t)(t - 1) * SN, g, &a, G); st->bwd_steps++; }
    } else if (strat == STRAT_CHUNK || strat == STRAT_REMOTE) {
      const int I = strat == STRAT_CHUNK ? F : C;
      for (int k = cdiv(T, I) - 1; k >= 0; --k) {
        const int s0 = k * I, e = imin((k + 1) * I, T);
        const REAL *start;
        if (strat == STRAT_REMOTE) {
          memcpy(loaded, remote + (size_t)k * SN, (size_t)SN * sizeof(REAL));
          st->remote_reads++; ev(elog, EV_LOAD_REMOTE, s0, 0); start = loaded;
        } else start = ckpt + (size_t)k * SN;
        ev(elog, EV_REFWD2, s0, e);
        for (int t = s0 + 1; t <= e; ++t) {
          advance_state(n, sp, b, t, t == s0 + 1 ? start : chunk + (size_t)(t - s0 - 2) * SN,
                        chunk + (size_t)(t - s0 - 1) * SN, scratch, 0);
          st->refwd2_steps++;
        }
        ev(elog, EV_BACKWARD, e, s0 + 1);
        for (int t = e; t > s0; --t) { backward_step(n, sp, b, t, chunk + (size_t)(t - s0 - 1) * SN, g, &a, G); st->bwd_steps++; }
      }
    } else if (strat == STRAT_HIER) {
      const int n_batches = cdiv(n_ckpt, C);
      for (int gb = n_batches - 1; gb >= 0; --gb) {
        const int k_hi = imin((gb + 1) * C, n_ckpt) - 1;
        if (gb < n_batches - 1) { /* the last batch is still in local memory */
          memcpy(ckpt, remote + (size_t)gb * C * SN, (size_t)C * SN * sizeof(REAL));
          st->remote_reads++; ev(elog, EV_LOAD_BATCH, gb * C * F, C);
        }
        for (int k = k_hi; k >= gb * C; --k) {
          const int s0 = k * F, e = imin(s0 + F, T);
          ev(elog, EV_REFWD2, s0, e);
          for (int t = s0 + 1; t <= e; ++t) {
            advance_state(n, sp, b, t, t == s0 + 1 ? ckpt + (size_t)(k % C) * SN : chunk + (size_t)(t - s0 - 2) * SN,
                          chunk + (size_t)(t - s0 - 1) * SN, scratch, 0);
            st->refwd2_steps++;
          }
          ev(elog, EV_BACKWARD, e, s0 + 1);
          for (int t = e; t > s0; --t) { backward_step(n, sp, b, t, chunk + (size_t)(t - s0 - 1) * SN, g, &a, G); st->bwd_steps++; }
        }
      }
    } else { /* DOUBLE */
      for (int K = cdiv(T, C) - 1; K >= 0; --K) {
        const int s0 = K * C, e = imin((K + 1) * C, T);
        memcpy(loaded, remote + (size_t)K * SN, (size_t)SN * sizeof(REAL));
        st->remote_reads++; ev(elog, EV_LOAD_REMOTE, s0, 0);
        /* Re-Forward_1: rebuild the fine checkpoints x_{s0+F}, x_{s0+2F}, ... < e */
        const int nf = cdiv(e - s0, F);       /* fine chunks in this segment */
        const int last = s0 + (nf - 1) * F;   /* largest fine checkpoint index */
        memcpy(fine, loaded, (size_t)SN * sizeof(REAL));
        if (last > s0) {
          ev(elog, EV_REFWD1, s0, last);
          memcpy(x, loaded, (size_t)SN * sizeof(REAL));
          for (int t = s0 + 1; t <= last; ++t) {
            advance_state(n, sp, b, t, x, xn, scratch, 0); st->refwd1_steps++;
            REAL *tmp = x; x = xn; xn = tmp;
            if ((t - s0) % F == 0) { memcpy(fine + (size_t)((t - s0) / F) * SN, x, (size_t)SN * sizeof(REAL)); ev(elog, EV_KEEP_FINE, t, 0); }
          }
        }
        for (int m = nf - 1; m >= 0; --m) {
          const int f0 = s0 + m * F, fe = imin(f0 + F, e);
          ev(elog, EV_REFWD2, f0, fe);
          for (int t = f0 + 1; t <= fe; ++t) {
            advance_state(n, sp, b, t, t == f0 + 1 ? fine + (size_t)m * SN : chunk + (size_t)(t - f0 - 2) * SN,
                          chunk + (size_t)(t - f0 - 1) * SN, scratch, 0);
            st->refwd2_steps++;
          }
          ev(elog, EV_BACKWARD, fe, f0 + 1);
          for (int t = fe; t > f0; --t) { backward_step(n, sp, b, t, chunk + (size_t)(t - f0 - 1) * SN, g, &a, G); st->bwd_steps++; }
        }
      }
    }
    free(a.dv_next); free(a.dv_cur); free(a.du); free(a.ds);
  }
  free(scratch); free(traj); free(ckpt); free(chunk); free(fine); free(loaded); free(remote);
  free(x); free(xn); free(u); free(usum); free(g);
  return loss_b;
}

/*
 * Entry point.  Arrays:
 *   W_in[l]  [N_{l-1}][N_l], W_rec[l] [N_l][N_l], W_out [N_L][n_out]   (row = presynaptic neuron)
 *   rec_mask[l] (or NULL / NULL entries): [N_l][N_l] bytes; the caller has already zeroed the
 *            masked weights; the gradient of W_rec^l is multiplied by the mask at the end.
 *   in_spikes [T][B][n_in] bytes 0/1;  labels [B]
 *   spikes[l] [T][B][N_l] REAL: output (or input when cfg->forced)
 *   vtraj[l]  [T][B][N_l] REAL or vtraj == NULL
 *   ubar [B][n_out]; loss (1 value)
 *   dW_in[l], dW_rec[l], dW_out: outputs, same shapes as the weights (may be NULL when
 *            do_backward == 0)
 *   evlog: optional int32 triples (code, a, b) of batch element 0's schedule; evcap = capacity
 * Returns 0 on success, 1 on invalid arguments.
 */
int FN(oracle_bptt)(const oracle_cfg *cfg, const REAL *const *W_in, const REAL *const *W_rec,
                    const REAL *W_out, const uint8_t *const *rec_mask, const uint8_t *in_spikes,
                    const int32_t *labels, REAL *const *spikes, REAL *const *vtraj, REAL *ubar,
                    double *loss, int do_backward, REAL *const *dW_in, REAL *const *dW_rec,
                    REAL *dW_out, oracle_stats *stats, int32_t *evlog, int64_t evcap) {
  const int L = cfg->n_layers, T = cfg->T, B = cfg->B;
  if (L < 1 || L > 16 || T < 1 || B < 1 || cfg->n_in < 1 || cfg->n_out < 1) return 1;
  if (cfg->strategy == STRAT_CHUNK && (cfg->F < 1 || cfg->F > T)) return 1;
  if (cfg->strategy == STRAT_REMOTE && (cfg->C < 1 || cfg->C > T)) return 1;
  if (cfg->strategy == STRAT_DOUBLE && (cfg->F < 1 || cfg->F > cfg->C || cfg->C > T)) return 1;
  if (cfg->strategy == STRAT_HIER && (cfg->F < 1 || cfg->F > T || cfg->C < 1)) return 1;
  if (cfg->strategy < 0 || cfg->strategy > 4) return 1;
  if (cfg->forced_states && (cfg->strategy != STRAT_STANDARD || !cfg->forced || !vtraj)) return 1;
  if (cfg->surr_window > 0 && cfg->mode != MODE_HEAVISIDE) return 1; /* S has no windowed antiderivative here */

  net_t n;
  n.c = cfg; n.L = L; n.W_in = W_in; n.W_rec = W_rec; n.W_out = W_out;
  n.alpha = (REAL)cfg->alpha; n.beta = (REAL)cfg->beta; n.theta = (REAL)cfg->theta; n.k = (REAL)cfg->surr_beta;
  n.win = (float)cfg->surr_window;
  int off[17]; off[0] = 0;
  for (int l = 0; l < L; ++l) off[l + 1] = off[l] + cfg->n_hidden[l];
  n.off = off; n.SN = off[L];
  spikes_t sp; sp.in = in_spikes; sp.hid = spikes;

  size_t sz_in[16], sz_rec[16], sz_out = (size_t)cfg->n_hidden[L - 1] * cfg->n_out;
  for (int l = 0; l < L; ++l) {
    sz_in[l] = (size_t)(l == 0 ? cfg->n_in : cfg->n_hidden[l - 1]) * cfg->n_hidden[l];
    sz_rec[l] = (size_t)cfg->n_hidden[l] * cfg->n_hidden[l];
  }
  if (do_backward) {
    for (int l = 0; l < L; ++l) {
      memset(dW_in[l], 0, sz_in[l] * sizeof(REAL));
      memset(dW_rec[l], 0, sz_rec[l] * sizeof(REAL));
    }
    memset(dW_out, 0, sz_out * sizeof(REAL));
  }

  int nth = cfg->nthreads < 1 ? 1 : cfg->nthreads;
  if (nth > B) nth = B;
#ifndef _OPENMP
  nth = 1;
#endif
  double *loss_b = (double *)calloc((size_t)B, sizeof(double));
  oracle_stats st0; memset(&st0, 0, sizeof st0);

  if (nth == 1) {
    grads_t G;
    for (int l = 0; l < L; ++l) { G.dW_in[l] = do_backward ? dW_in[l] : NULL; G.dW_rec[l] = do_backward ? dW_rec[l] : NULL; }
    G.dW_out = dW_out;
    for (int b = 0; b < B; ++b) {
      oracle_stats st; memset(&st, 0, sizeof st);
      evlog_t lg; lg.buf = evlog; lg.cap = evcap; lg.n = 0; lg.on = (b == 0);
      loss_b[b] = bptt_one(&n, &sp, labels, b, ubar + (size_t)b * cfg->n_out, vtraj, &G, do_backward, &st, &lg);
      if (b == 0) { st0 = st; st0.n_events = lg.n; }
    }
  } else {
#ifdef _OPENMP
    /* thread-private gradient accumulators, reduced afterwards in thread order */
    grads_t *Gs = (grads_t *)calloc((size_t)nth, sizeof(grads_t));
    for (int th = 0; th < nth; ++th) {
      for (int l = 0; l < L; ++l) {
        Gs[th].dW_in[l] = do_backward ? (REAL *)calloc(sz_in[l], sizeof(REAL)) : NULL;
        Gs[th].dW_rec[l] = do_backward ? (REAL *)calloc(sz_rec[l], sizeof(REAL)) : NULL;
      }
      Gs[th].dW_out = do_backward ? (REAL *)calloc(sz_out, sizeof(REAL)) : NULL;
    }
#pragma omp parallel for schedule(static) num_threads(nth)
    for (int b = 0; b < B; ++b) {
      const int th = omp_get_thread_num();
      oracle_stats st; memset(&st, 0, sizeof st);
      evlog_t lg; lg.buf = evlog; lg.cap = evcap; lg.n = 0; lg.on = (b == 0);
      loss_b[b] = bptt_one(&n, &sp, labels, b, ubar + (size_t)b * cfg->n_out, vtraj, &Gs[th], do_backward, &st, &lg);
      if (b == 0) { st0 = st; st0.n_events = lg.n; }
    }
    if (do_backward)
      for (int th = 0; th < nth; ++th) {
        for (int l = 0; l < L; ++l) {
          for (size_t i = 0; i < sz_in[l]; ++i) dW_in[l][i] += Gs[th].dW_in[l][i];
          for (size_t i = 0; i < sz_rec[l]; ++i) dW_rec[l][i] += Gs[th].dW_rec[l][i];
        }
        for (size_t i = 0; i < sz_out; ++i) dW_out[i] += Gs[th].dW_out[i];
      }
    for (int th = 0; th < nth; ++th) {
      for (int l = 0; l < L; ++l) { free(Gs[th].dW_in[l]); free(Gs[th].dW_rec[l]); }
      free(Gs[th].dW_out);
    }
    free(Gs);
#endif
  }
  /* gradient exists only on synapses that exist */
  if (do_backward && rec_mask)
    for (int l = 0; l < L; ++l)
      if (rec_mask[l])
        for (size_t i = 0; i < sz_rec[l]; ++i)
          if (!rec_mask[l][i]) dW_rec[l][i] = (REAL)0;

  double s = 0.0;
  for (int b = 0; b < B; ++b) s += loss_b[b];
  *loss = s / (double)B;
  free(loss_b);
  st0.threads_used = nth;
  if (stats) *stats = st0;
  return 0;
}
