/*
 * snn.h -- C ABI of the MI355X (gfx950) library for backpropagation through time
 * in multi-layer leaky-integrate-and-fire (LIF) spiking RNNs under the state
 * storage strategies of "Optimal Gradient Checkpointing for Sparse and Recurrent
 * Architectures using Off-Chip Memory" (Fig. 1 of that paper).
 *
 * Memory tiers.  The paper's "local" memory is a capped activation budget in HBM;
 * its "remote / streaming" memory is pinned host DRAM reached with
 * hipMemcpyAsync on a side stream.
 *
 * Strategy names follow the caption of Fig. 1:
 *   SNN_STANDARD  plain BPTT, every state stored               (eq. M_Base)
 *   SNN_CHUNK     paper Section "Standard Checkpointing"        (eq. M_Standard, T_Standard)
 *   SNN_REMOTE    paper Section "Remote Checkpointing"          (eq. M_Remote, T_Remote)
 *   SNN_DOUBLE    paper Section "Double Checkpointing"          (eq. M_Double, T_Double, N_c)
 *   SNN_HIER      paper Section "Hierarchical Checkpointing"    (eq. M_Hier, T_Hier)
 *
 * Model (layers l = 1..L, s^0 = input spikes, zero initial state, t = 1..T):
 *   I^l_t = sum_{j active in s^{l-1}_t} W_in^l[j,:] + sum_{j active in s^l_{t-1}} W_rec^l[j,:]
 *   v^l_t = (alpha v^l_{t-1} - theta s^l_{t-1}) + I^l_t ;   s^l_t = [v^l_t > theta]
 *   u_t   = beta u_{t-1} + sum_{j active in s^L_t} W_out[j,:] ;  ubar = mean_t u_t
 *   loss  = mean_b softmax-cross-entropy(ubar_b, y_b)
 * Backward pass: surrogate derivative 1/(1 + surr_beta |v - theta|)^2, full gradient
 * (also through the reset term).  With surr_window = w > 0 the derivative is cut to 0
 * wherever |v - theta| >= w, the test taken in fp32 on the stored fp32 potential.
 *
 * Conventions.  Every function returns an snn_status (0 = success) unless noted;
 * nothing throws or aborts.  Pointers marked "host or device" may be either (the
 * library asks the HIP runtime which).  The caller owns every buffer it passes and
 * keeps it alive for the duration of the call.  All calls on one context must come
 * from one thread at a time.  All functions return after the work they queued on the
 * context's stream (and on the library's private copy stream) has completed.
 */
#ifndef SNN_H
#define SNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct snn_ctx snn_ctx; /* opaque; created by snn_init, freed by snn_destroy */

typedef enum {
  SNN_OK = 0,
  SNN_E_INVAL = 1,   /* bad argument / unsupported shape                         */
  SNN_E_BUDGET = 2,  /* strategy needs more HBM activation memory than the budget */
  SNN_E_HIP = 3,     /* a HIP runtime call failed (text in snn_last_error)        */
  SNN_E_HOSTMEM = 4, /* pinned host allocation failed                             */
  SNN_E_STATE = 5    /* call order violated (e.g. snn_bptt before inputs are bound) */
} snn_status;

typedef enum { SNN_STANDARD = 0, SNN_CHUNK = 1, SNN_REMOTE = 2, SNN_DOUBLE = 3, SNN_HIER = 4 } snn_strategy;
typedef enum { SNN_W_IN = 0, SNN_W_REC = 1, SNN_W_OUT = 2 } snn_tensor_kind;

#define SNN_MAX_LAYERS 4

typedef struct {
  int32_t n_in;                     /* input channels (<= 4096)                        */
  int32_t n_layers;                 /* 1..SNN_MAX_LAYERS recurrent LIF layers          */
  int32_t n_hidden[SNN_MAX_LAYERS]; /* neurons per layer (each <= 8192)                */
  int32_t n_out;                    /* leaky non-spiking readouts (<= 1024)            */
  int32_t T;                        /* maximum sequence length this context will see   */
  int32_t batch;
  float alpha;                      /* membrane leak                                   */
  float beta_out;                   /* readout leak                                    */
  float theta;                      /* threshold = reset amount                        */
  float surr_beta;                  /* k in 1/(1+k|v-theta|)^2                          */
  float surr_window;                /* w > 0: the surrogate derivative is 0 wherever
                                       |v-theta| >= w (compact support); <= 0: no window  */
  int32_t device;                   /* HIP device ordinal                              */
  int32_t spike_tier;               /* 0: the spike bitmasks of the whole sequence stay in HBM (the paper's setting:
                                       sparse spikes are part of the local, non-optimisable memory); 1: under REMOTE
                                       and DOUBLE the hidden layers' bitmasks of finished coarse segments move to pinned
                                       host memory on the copy stream and come back before the segment is recomputed;
                                       HBM then holds a window of 2 * coarse_interval + 1600 steps of them whatever T
                                       is (the extension the paper's Discussion leaves open: what bounds the sequence
                                       length once the states are checkpointed is the spike store).  Results are the
                                       same bit for bit.  Ignored by the other strategies and when the window would
                                       not be shorter than the sequence. */
  void *stream;                     /* hipStream_t to queue work on; NULL = a stream the
                                       library creates (the legacy default stream cannot be
                                       recorded into a HIP graph)                        */
} snn_config;

/* Statistics of one training step: the quantities the paper's Results report (time per batch, peak local memory;
 * Fig. 2) plus the terms of its closed forms -- state slots (eq. M_Base, M_Standard, M_Remote, M_Hier, M_Double),
 * recompute steps (T_refwd in eq. T_Standard, T_Double) and host transfers (N_c, T_c in eq. T_Remote, T_Double).
 * Filled by snn_bptt (all times in milliseconds, measured with HIP events on the
 * context's stream; bytes are what the call actually allocated/moved). */
typedef struct {
  float ms_total, ms_forward, ms_backward_total; /* whole step; forward incl. loss; everything after */
  float ms_recompute, ms_adjoint, ms_dw;         /* sums over kernels of each kind: recompute (currents+scan),
                                                    recurrent adjoint kernels, weight-gradient kernels */
  float ms_fwd_seq, ms_fwd_currents, ms_up_gemm; /* forward: sequential per-layer kernels / parallel current and
                                                    readout kernels; adjoint: inter-layer GEMMs */
  float ms_bwd_stage;        /* launches that carry the recurrences of one pipeline stage together with the
                                weight-gradient contraction of the stage before (not in ms_adjoint / ms_dw) */
  float ms_fwd_stage;        /* launches that carry the sequential parts of one forward stage together with the
                                currents of the next (not in ms_fwd_seq / ms_fwd_currents)                    */
  float ms_scan;             /* recompute, part 2: the scans that turn a chunk's currents into states (ms_recompute
                                holds part 1, the current kernels, alone)                                      */
  int64_t bytes_states;      /* HBM: trajectory / chunk buffer / checkpoints / staging slots */
  int64_t bytes_spikes;      /* HBM: spike bitmasks of all layers, all steps                  */
  int64_t bytes_workspace;   /* HBM: readout-adjoint tile and other per-chunk scratch          */
  int64_t bytes_host;        /* pinned host memory holding remote checkpoints                  */
  int64_t d2h_bytes, h2d_bytes; /* checkpoint traffic over the host link                       */
  int32_t n_d2h, n_h2d;         /* number of checkpoint transfers (N_c = n_d2h + n_h2d)        */
  int64_t spike_d2h_bytes, spike_h2d_bytes; /* spike bitmask traffic over the host link (spike_tier 1) */
  int64_t bytes_host_spikes;    /* pinned host memory holding the hidden layers' spike bitmasks (spike_tier 1) */
  int64_t fwd_steps, refwd1_steps, refwd2_steps, bwd_steps; /* time steps per pass             */
  int64_t refwd_current_steps; /* time steps whose synaptic currents the recompute passes computed: refwd1 + refwd2
                                  unless Double kept a segment's currents between its two passes (then once per
                                  step) or the forward pass left them in that cache (then not at all)      */
  int32_t local_state_slots; /* states resident in HBM at the peak (M_s units)                 */
  int32_t remote_state_slots;
  float firing_rate[SNN_MAX_LAYERS]; /* measured mean rate of each hidden layer                */
} snn_stats;

/* Create a context: validates the configuration, allocates weights, gradients and the
 * spike store for cfg->T steps on cfg->device (the paper's M_others, Section "Standard Checkpointing": weights and
 * the sparse spike trains of the whole sequence, which no strategy recomputes).  No state storage is allocated
 * here.  *out is set even on failure (so that snn_last_error can be read) and must be passed to snn_destroy.
 * SNN_E_INVAL for a shape outside the limits noted in snn_config. */
snn_status snn_init(const snn_config *cfg, snn_ctx **out);

/* Copy one weight matrix into the context (weights are part of M_others, Section "Standard Checkpointing").
 * w: [pre][post] row-major fp32 (row = presynaptic
 * neuron), host or device.  kind SNN_W_IN/SNN_W_REC take layer 0..L-1, SNN_W_OUT ignores it.
 * mask_or_null (SNN_W_REC only): [N][N] bytes, 1 = synapse exists; masked weights must already
 * be zero in w; the gradient of a masked matrix is zero where the mask is zero. */
snn_status snn_set_weights(snn_ctx *ctx, int kind, int layer, const float *w, const uint8_t *mask_or_null);

/* Forward pass only (the two operations of the paper's forward step, Section "Standard Checkpointing": the
 * sparse matrix product that accumulates the weight rows of active presynaptic neurons, and spike generation into
 * a sparse representation; then readout and loss); binds the inputs that a following
 * snn_bptt uses.  in_spikes: [T][B][n_in] bytes 0/1, host or device; T <= cfg.T.  labels: [B]
 * int32, host or device, each in [0, n_out) (SNN_E_INVAL otherwise, checked on the host before anything is
 * queued).  loss_out: one float, host.  Stores spikes (bitmasks) but no states. */
snn_status snn_forward(snn_ctx *ctx, const uint8_t *in_spikes, const int32_t *labels, int32_t T, float *loss_out);

/* The forward pass of snn_forward for callers that cannot allocate device memory: code under HIP graph capture
 * around it, tight serving loops, harnesses that forbid hipMalloc.  Same result as snn_forward bit for bit (spike
 * trains, readout, loss; inputs bound for a following snn_bptt).  Differences: in_spikes and labels must be device
 * pointers (a host buffer would need a staging allocation: SNN_E_INVAL); the per-tile currents of the forward pass,
 * which snn_forward keeps in a workspace it allocates on demand, live in a static 16 MiB device array inside the
 * library (one per GPU, held until the process ends).  A network whose workspace --
 * 64 * batch * (8 * n_out + 2 * sum of n_hidden) * 4 bytes -- exceeds 16 MiB is refused with SNN_E_INVAL and a
 * message that says so.  The call allocates and frees nothing, on the device or through the HIP runtime.  Every
 * context on a GPU shares that GPU's array: calls that overlap in time on one GPU (two host threads, two contexts)
 * race; calls one after the other do not interfere (nothing in the array is read before the same call wrote it). */
snn_status snn_forward_noalloc(snn_ctx *ctx, const uint8_t *in_spikes, const int32_t *labels, int32_t T, float *loss_out);

/* One full training step (forward with the strategy's storage plan, loss, backward with
 * recomputation: the execution orders of Fig. 1, one panel per strategy; Sections "Standard Checkpointing",
 * "Remote Checkpointing", "Hierarchical Checkpointing", "Double Checkpointing") on the inputs bound by the last snn_forward/snn_bind_inputs.  Gradients stay in
 * the context (overwritten by each call) until snn_grads copies them out.
 *   STANDARD ignores both intervals; CHUNK uses fine_interval; REMOTE uses coarse_interval;
 *   DOUBLE needs 1 <= fine <= coarse <= T; HIER takes fine_interval = steps between checkpoints and
 *   coarse_interval = nb_local, the number of checkpoints per host transfer.  0 = default (coarse ceil(sqrt T), fine ceil(sqrt coarse),
 *   fine ceil(sqrt T) for CHUNK: the square-root rules of the paper's Hyperparameter Study).
 *   hbm_budget_bytes caps activation storage (states + spike bitmasks + workspace); 0 = unlimited.
 *   snn_bytes_required is the least the strategy can run in (one chunk buffer: the paper's state
 *   count); below it -> SNN_E_BUDGET before anything is allocated.  With room to spare (or no budget)
 *   the call takes up to n_layers + 2 more chunk buffers, which let the layers of the adjoint pass and
 *   the recompute of the next chunks overlap; DOUBLE then takes coarse_interval more state slots to keep the
 *   synaptic currents of a coarse segment between its two recompute passes (Section "Double Checkpointing":
 *   T_Double's second recomputation then costs scans only) and, for networks whose layers all have more than 256
 *   neurons, as many further slots as the budget leaves, in whole coarse segments from the end of the
 *   sequence, in which the forward pass leaves the currents it computed, so that those segments' currents are
 *   not recomputed at all (without a budget: the last segment only).  Gradients are the same bit for bit
 *   either way, and stats reports what was allocated and how many steps' currents were recomputed. */
snn_status snn_bptt(snn_ctx *ctx, snn_strategy strategy, int32_t coarse_interval, int32_t fine_interval,
                    size_t hbm_budget_bytes, snn_stats *stats_or_null);

/* Bind inputs without running anything (same arguments and checks as snn_forward). */
snn_status snn_bind_inputs(snn_ctx *ctx, const uint8_t *in_spikes, const int32_t *labels, int32_t T);

/* Copy a gradient tensor out: the plain-BPTT gradient, which every strategy reproduces exactly (Section
 * "Standard Checkpointing": checkpointing trades memory for recomputation, not accuracy).  dst: [pre][post] fp32,
 * host or device, n_elems must match (SNN_E_INVAL otherwise). */
snn_status snn_grads(snn_ctx *ctx, int kind, int layer, float *dst, size_t n_elems);

/* Parity/debug accessors (valid after snn_forward or snn_bptt; SNN_E_STATE before).  The spike trains are the
 * sparse spike tensor that stays in local memory for the whole sequence (Section "Standard Checkpointing",
 * Discussion). */
snn_status snn_get_spikes(snn_ctx *ctx, int layer /*0..L-1*/, uint8_t *dst /*[T][B][N_l] bytes, host*/);
snn_status snn_get_readout(snn_ctx *ctx, float *ubar /*[B][n_out], host*/, float *loss /*1 float, host*/);
/* Membrane potentials v^l_t of one layer at one step, t in 1..T: dst [B][N_l] fp32, host or device.  The state is
 * rebuilt the way a recompute pass rebuilds it (Section "Standard Checkpointing": from a checkpoint -- here x_0 --
 * through the stored spike trains, no spike generation), so it is available after a forward pass or a training
 * step of any strategy and equals, bit for bit, what the forward pass held at step t.  Costs a recompute pass over
 * steps 1..t and allocates (and frees) a buffer of min(t, 64) + 2 states.  SNN_E_STATE before a forward pass,
 * SNN_E_INVAL for a layer or step out of range. */
snn_status snn_get_state(snn_ctx *ctx, int layer, int32_t t, float *dst);
/* Runs a forward pass that stores every state (the storage plan of plain BPTT, eq. M_Base) and copies the
 * trajectory out: dst [T][B][sum N_l] fp32, host. */
snn_status snn_debug_states(snn_ctx *ctx, float *dst);

/* Measurement aid: one plain streaming copy kernel of `bytes` bytes (a multiple of 16), device to
 * device.  Hardware byte counters read under a profiler are scaled by what they read for this
 * kernel, whose traffic is known (bytes read + bytes written). */
snn_status snn_debug_copy(snn_ctx *ctx, const void *src, void *dst, size_t bytes);

/* Measurement aid (kernel micro-benchmark at a controlled activity level): replaces the stored
 * spike trains of the hidden layers by the ones given -- hidden[l]: [T][B][N_l] bytes 0/1, host or device, T the
 * length bound by the last snn_forward / snn_bind_inputs call; a NULL entry leaves that layer's spikes as they are
 * -- and runs the synaptic-current part of recompute (row A2 of the hot path: feed-forward and recurrent currents
 * of every layer, no scan) over the whole sequence in chunks of `chunk` steps, `reps` times.  *ms_out: mean time
 * of one pass over the sequence (HIP events on the library's stream).  The currents go to a scratch buffer of
 * chunk states that the call allocates and frees; the context's spike trains stay replaced until the next
 * snn_forward or snn_bptt.  SNN_E_STATE without bound inputs, SNN_E_INVAL for chunk or reps < 1. */
snn_status snn_debug_currents(snn_ctx *ctx, const uint8_t *const *hidden, int32_t chunk, int32_t reps, float *ms_out);

/* Activation bytes the strategy needs at least in HBM for sequence length T (no context, no GPU
 * needed): M_s times the state count of eq. M_Base / M_Standard / M_Remote / M_Hier / M_Double plus the staging
 * slots of the host tier, plus the spike bitmasks and the per-chunk workspace.  Returns 0 for invalid arguments
 * and for shapes snn_init refuses.  Equals stats.bytes_states + bytes_spikes +
 * bytes_workspace of a call whose budget is exactly this number. */
size_t snn_bytes_required(const snn_config *cfg, snn_strategy strategy, int32_t T, int32_t coarse_interval,
                          int32_t fine_interval);
/* Number of M_s-sized state slots of that plan held in HBM (the paper's closed forms plus the
 * staging slots of the host tier) and, in *remote_slots (may be NULL), on the host. */
int32_t snn_state_slots(snn_strategy strategy, int32_t T, int32_t coarse_interval, int32_t fine_interval,
                        int32_t *remote_slots);
/* The execution order of Fig. 1 for a plan.  Writes the schedule of the plan as int32 triples (op, a, b), at most cap triples, and returns
 * the number of triples the full schedule has.  Ops: 1 SAVE_LOCAL c, 2 SAVE_REMOTE c, 3 LOAD_REMOTE c,
 * 4 REFWD1 (a,b], 5 KEEP_FINE c, 6 REFWD2 (a,b], 7 BACKWARD a..b (descending), 8 SAVE_BATCH (first
 * checkpoint c, count), 9 LOAD_BATCH (first checkpoint c, count). */
int64_t snn_schedule(snn_strategy strategy, int32_t T, int32_t coarse_interval, int32_t fine_interval,
                     int32_t *out_triples, int64_t cap);

/* Intervals for a strategy under an HBM activation budget (no context, no GPU needed; paper Section
 * "Hyperparameter Study": memory is smallest at the square-root intervals, time falls with longer chunks).
 * Picks the longest chunk of at most 256 steps -- beyond that a longer chunk no longer saves time on this
 * hardware -- whose plan fits hbm_budget_bytes (snn_bytes_required), never shorter than the square-root
 * rule's; for DOUBLE then the longest coarse interval whose fine checkpoints still fit; for HIER nb_local by
 * the square-root rule.  hbm_budget_bytes = 0: no limit.  Writes the intervals to *coarse_out / *fine_out
 * (in the meaning snn_bptt gives them; 0 where the strategy ignores one).  SNN_E_BUDGET if even the
 * memory-minimal plan does not fit, SNN_E_INVAL for invalid arguments. */
snn_status snn_suggest_intervals(const snn_config *cfg, snn_strategy strategy, int32_t T, size_t hbm_budget_bytes,
                                 int32_t *coarse_out, int32_t *fine_out);

const char *snn_last_error(const snn_ctx *ctx); /* never NULL; "" if none */
void snn_destroy(snn_ctx *ctx);

/*
 * Test hooks.  The library chooses its kernels from the layer shapes, the batch size, the state size and the
 * firing rates of the previous step; every choice gives the same bits.  The parity tests force each flavour
 * through environment variables, read by the library at the points noted.  They are not part of the interface
 * proper: a caller never needs them.
 *   read by snn_init (fixed for the context's life):
 *     SNN_HOST_TIER=dma|direct   Remote/Double checkpoints by hipMemcpyAsync / written and read by the kernels
 *                                through the mapped pinned block (default: direct up to 1 MiB per state)
 *     SNN_DW=event|tile|mfma     weight gradients by the event-by-event kernel / the event-driven tiled kernel
 *                                (batch <= 64) / the matrix-core contraction (default: tiled when some weight
 *                                matrix has 32 MB or more, else the contraction)
 *     SNN_RF_CACHE=0             Double: never keep a coarse segment's currents between its two recompute passes
 *     SNN_KEEP_CURRENTS=0        Double: the forward pass never leaves the currents of the last coarse segments in
 *                                that cache (default: as many whole segments as the budget has room for)
 *     SNN_DW_CSR=0               tiled weight gradients of masked recurrent matrices over the dense tile, not per
 *                                existing synapse
 *     SNN_GRAPH=0                no HIP-graph replay of the training step
 *     SNN_BWD_PIPE=0, SNN_BWD_FUSE=0, SNN_PRE_IN_STAGE=0
 *                                adjoint pass layer by layer / weight gradients in launches of their own /
 *                                recompute of later chunks between, not inside, the stage launches
 *     SNN_NO_WS=1                no chip-wide kernels (no exchange buffer is allocated)
 *     SNN_WS_SPIN_LIMIT=n        polls before a chip-wide kernel gives up waiting (0: at once; the error path)
 *   read at the start of every call that launches kernels:
 *     SNN_CURRENTS=gather|mfma|dense   kernel of the synaptic currents
 *     SNN_WS_KERNEL=valu|stream|rows|rows_all|chip|csrw|single|pair|rows64
 *                                      VALU version of the chip-wide adjoint recurrence / one workgroup per batch
 *                                      element streaming the transposed matrix / the event-driven rows kernel of
 *                                      the surrogate window at any width above 256 / the same kernel evaluating
 *                                      every row / the chip-wide kernels over the dense-stored matrix, also under a
 *                                      surrogate window / the chip-wide kernel over compressed rows also under one /
 *                                      the matrix-core version with one batch group per workgroup, never two /
 *                                      with two wherever the batch has an even number of groups of 16 /
 *                                      with workgroups of 64 rows (eight wavefronts) and one batch group
 *     SNN_CSR=0|1                      compressed rows of masked recurrent matrices never / wherever a kernel
 *                                      for them exists (default: where the firing-rate policy picks a gather)
 *     SNN_SEQ_SLICES=1|2|4|8           workgroups per batch element in the sequential part of wide layers
 *     SNN_FWD_FUSE=0                   wide layers over compressed rows: the dense currents for the next pipeline
 *                                      stage never ride in the launch of a stage's sequential parts
 *     SNN_SEQ_KERNEL=gather|rs         sequential forward part of layers of up to 256 neurons: event-driven gather
 *                                      over the rows of the neurons that fired / the register-stationary chain
 *                                      (default: the chain; the gather was measured slower at every firing rate)
 */

#ifdef __cplusplus
}
#endif
#endif /* SNN_H */
