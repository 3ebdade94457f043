// Internal declarations shared by the host-side orchestration and the HIP kernels of the
// LIF-SNN BPTT library (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#define SNN_MAXL 4
#define SNN_CSR_SUBW 512 // postsynaptic neurons per sub-range of a compressed row (one wavefront's share)

// Device-visible description of the network and of where its data lives in HBM.
//
// Weights: fp32, [pre][post] row-major, so the synapses leaving one presynaptic neuron are one
// contiguous row (one active spike = one coalesced row read).  W_in[l] and W_rec[l] are stacked in
// one allocation (W_rec[l] = W_in[l] + pre_l * N_l) so that a gather walks one row stream.  *_T are [post][pre] copies used by
// the adjoint pass (delta_s[j] = sum_n W[j][n] * delta_v[n] becomes a coalesced column walk).
// Spikes: one bit per neuron, 64-bit words, mask[l] = [T+1][B][Wd[l]] with row 0 (t = 0) all zero;
// layer index 0 is the input layer, l >= 1 hidden layer l.
// States: slots of B*SN floats laid out [B][SN] (all layers of one batch element contiguous).
struct NetDev {
  int L, n_in, n_out, B, SN;
  int N[SNN_MAXL];        // neurons of hidden layer l (0-based here)
  int off[SNN_MAXL + 1];  // offset of layer l inside a state vector
  int Wd[SNN_MAXL + 1];   // 64-bit words per (t, b) of layer index 0..L (0 = input)
  const float *W_in[SNN_MAXL], *W_rec[SNN_MAXL], *W_out;
  const float *W_inT[SNN_MAXL], *W_recT[SNN_MAXL], *W_outT;
  uint64_t *mask[SNN_MAXL + 1];
  // > 0: mask[l] holds only a window of the sequence, as a ring of that many steps (row = step modulo the ring);
  // the rest of the spike trains is in pinned host memory and travels per coarse segment.  0: all T + 1 rows.
  int mring[SNN_MAXL + 1];
  // Compressed rows of a masked recurrent matrix (NULL: the layer has no mask, or its compressed form is switched
  // off): the existing synapses of presynaptic neuron j, ascending in the postsynaptic index, are entries
  // csr_sub[l][j * (nsub + 1) + 0] .. csr_sub[l][j * (nsub + 1) + nsub] of csr_col[l] (16-bit postsynaptic index)
  // and csr_val[l]; csr_sub[l][j * (nsub + 1) + r] is the first entry whose postsynaptic index is at least
  // r * SNN_CSR_SUBW, nsub = ceil(N_l / SNN_CSR_SUBW): a wavefront that owns the postsynaptic neurons
  // [r * SNN_CSR_SUBW, (r + 1) * SNN_CSR_SUBW) finds its part of every row without searching.
  const uint32_t *csr_sub[SNN_MAXL];
  const uint16_t *csr_col[SNN_MAXL];
  const float *csr_val[SNN_MAXL];
  uint32_t csr_nnz[SNN_MAXL]; // synapses that exist (csr_col and csr_val hold one entry more)
  // The same entries once more, packed for the gather of the forward and recompute passes: entry e as one 64-bit
  // word, weight bits in the low half, postsynaptic index in the high half (one load per row and lane).  Behind
  // the nnz entries sit nsub * 64 zero-weight entries, number r * 64 + k with postsynaptic index
  // (r + 1) * SNN_CSR_SUBW + k: where a lane has no entry of a row it loads this one, and the add goes to word k of
  // the 64 spare words that follow the SNN_CSR_SUBW accumulators of sub-range r in LDS.
  const uint64_t *csr_pk[SNN_MAXL];
  float alpha, beta, theta, k;
  float win;  // surrogate window (<= 0: none)
  // Current kernel for the layers whose weights are far beyond the L2, from the firing rates of the last step
  // (0: not known yet -> dense, 1: event-by-event gather, 2: dense matrix-core version, 3 ([1] only): dense for the
  // feed-forward part, gather over compressed rows for the recurrent part, 4 ([1] only): dense for both, but the
  // sequential forward part walks the compressed rows); [0] forward currents
  // (feed-forward part only), [1] recompute (both parts).  Every choice gives the same bits.
  unsigned char cur_pol[2][SNN_MAXL];
  // Kernel selection forced from outside (test hooks; 0 = the library's own choice).  Every choice gives the same
  // bits.  sel_currents: 1 event-by-event gather, 2 list version on the matrix cores, 3 dense version.
  // sel_adjoint: 1 VALU version of the chip-wide recurrence, 2 one-workgroup-per-batch-element streaming kernel,
  // 3 event-driven rows (neurons inside the surrogate window only), 4 the same kernel evaluating every row, 5 the
  // chip-wide kernels over the dense-stored matrix, also under a surrogate window, 6 the chip-wide kernel over
  // compressed rows also under a surrogate window, 7 the matrix-core version of the chip-wide recurrence with one
  // batch group per workgroup (never two half a step apart), 8 the same with two groups wherever the batch has an
  // even number of groups, 9 the same with workgroups of 64 rows and one group.
  // sel_slices: workgroups per batch element in the sequential part of wide layers (1, 2, 4 or 8).
  unsigned char sel_currents, sel_adjoint, sel_slices;
  unsigned char no_fwd_fuse; // 1: the dense currents of wide layers never ride in the launch of the sequential parts
  // Sequential forward part of layers of up to 256 neurons: sel_seq 1 forces the event-driven gather, 2 the
  // register-stationary chain, 0 follows seq_pol[l] (1: gather; set from the measured firing rates).
  unsigned char sel_seq, seq_pol[SNN_MAXL];
  unsigned char sel_csr; // compressed rows of masked recurrent matrices: 1 never used (dense-stored walk everywhere),
                         // 2 used wherever a kernel for them exists, 0 the library's choice
};

// Where the forward / recompute kernel writes states it has to keep.
struct StoreSpec {
  float *base;        // slot 0 of the destination array (NULL = store nothing)
  size_t slot_stride; // floats between slots (= B*SN)
  int t_base;         // state x_t goes to slot (t - t_base)/interval - 1 + slot0 ...
  int interval;       // ... when (t - t_base) % interval == 0
  int slot0;
  int t_max;          // ... and t <= t_max
  int slot_mod;       // if > 0 the slot index is taken modulo this (ring of checkpoint slots)
  // Forward pass of wide layers only (the gather kernels of layers above 256 neurons): the synaptic current
  // I_t = I_in,t + I_rec,t of every step t > cur_from also goes to cur[(t - cur_from - 1) * slot_stride + ...], laid
  // out like a chunk of recomputed currents, so that the backward pass need not compute it again (NULL: nothing).
  float *cur;
  int cur_from;
};

// Optional timing hook: the launchers bracket groups of kernels of one kind (HIP events on the
// stream the kernels run on).  Kinds: 1 recompute, 2 adjoint recurrence, 3 dW, 4 forward sequential
// part, 5 forward parallel currents + readout, 6 inter-layer GEMM of the adjoint pass, 7 fused stage
// (recurrences + weight gradients of the previous stage), 8 fused forward stage (sequential parts + the
// currents of the next stage).
struct SpanHook {
  void *ctx;
  void (*begin)(void *ctx, int kind);
  void (*end)(void *ctx);
};

struct LaunchCfg {
  int nt_neuron; // threads that own neurons (multiple of 64)
  int npt;       // neurons per owning thread (template instance)
  size_t lds_bytes;
};

// ---- launchers (defined in snn_kernels.hip) ---------------------------------------------
hipError_t launch_pack_inputs(const uint8_t *in_spikes, uint64_t *mask0, int T, int B, int n_in, int Wd0,
                              hipStream_t s);
// Forward pass (gather, LIF update, threshold, compaction, readout) over consecutive time tiles
// bounds[0..n_tiles], each at most SNN_FWD_TILE steps.  state: [B][SN], x_{bounds[0]} on entry,
// x_{bounds[n_tiles]} on return.  work: scratch of SNN_FWD_TILE * B * (2 * SN + SNN_RO_TILES * n_out) floats.
// layer_tile_done(layer, t_end) is called (on the host, in stream order) after the launch that
// completes layer `layer` up to step t_end has been queued.
#define SNN_FWD_TILE 64
#define SNN_FWD_LAG (2 * (SNN_MAXL - 1)) // tiles the lowest layer can be ahead of the top layer
#define SNN_RO_TILES 8 // tiles of readout currents per launch of the readout scan
struct FwdCallbacks {
  void *ctx;
  hipError_t (*layer_tile_done)(void *ctx, int layer, int t_end);
};
// leaky readout over one tile of readout currents (n != 0: present; the launcher turns it into a workgroup count)
struct RoJob { int n; const float *iout; int nsteps, init; };
struct SeqJob { int l, t0, t1, t_tile; const float *iin; };
struct SeqJobs { SeqJob j[SNN_MAXL]; int count; };
struct CurJob { int mode, lsel, t0, nsteps, t_base; float *out; size_t slot_stride; };
struct CurJobs { CurJob j[2 * SNN_MAXL + 1]; int count; };
struct WsArgs;
hipError_t launch_forward(const NetDev &net, const int *bounds, int n_tiles, float *state, const StoreSpec &st,
                          double *readout /*[B][2][O]*/, int readout_init, float *work, hipStream_t s,
                          const SpanHook *hook = nullptr, const FwdCallbacks *cb = nullptr, const WsArgs *ws = nullptr);
// Recompute pass over steps t0+1..t1 from state_in = x_{t0}, spikes read from the stored bitmasks:
// currents of the whole range in parallel into buf (slot of x_t = t - t_base - 1), then a scan that
// turns them into states in place (store_all) and/or writes x_{t1} to state_out.
hipError_t launch_recompute(const NetDev &net, int t0, int t1, const float *state_in, float *buf, int t_base,
                            size_t slot_stride, int store_all, float *state_out, hipStream_t s);
// Part 1 of a recompute pass alone: the currents of steps t0+1..t1 of every layer into buf.
hipError_t launch_recompute_currents(const NetDev &net, int t0, int t1, float *buf, int t_base, size_t slot_stride,
                                     hipStream_t s);
// Part 2 of a recompute pass alone: buf already holds the currents of steps t0+1..t1.
// cur_src != NULL: the currents of step t are read from slot (t - src_base - 1) of cur_src, buf only takes states.
hipError_t launch_recompute_scan(const NetDev &net, int t0, int t1, const float *state_in, float *buf, int t_base,
                                 size_t slot_stride, int store_all, float *state_out, hipStream_t s,
                                 const float *cur_src = nullptr, int src_base = 0);
hipError_t launch_loss(const double *readout, const int32_t *labels, int B, int O, int T, float *ubar,
                       float *g, float *loss, hipStream_t s);
// Adjoint pass over steps t1, t1-1, ..., t0+1 of a tile.  vbuf holds x_t at slot (t - t_base - 1) and is
// overwritten in place by delta_v_t, layer by layer from the top.  Layer l of a tile needs layer l+1 of the
// same tile and layer l of the later tile, so the layers of consecutive tiles can run one tile apart.
// carry: [B][SN + O] floats (delta_v_{t+1} of all layers, delta_u_{t+1}); carry_init zeroes a layer's part first.
// Exchange buffer, barrier counters and error flag of the chip-wide weight-stationary recurrent
// kernel (see k_adj_rec_ws); xg == NULL disables that kernel.
struct WsArgs {
  float *xg;           // SNN_MAXL x [2][B][max N_l], one per job of a launch
  int xg_stride;       // floats between the exchange buffers of two jobs
  unsigned *bar;       // SNN_MAXL x [64] counters, zeroed before every launch
  unsigned *err;       // raised if a barrier gave up waiting
  int max_groups;      // workgroups of that kernel that can be resident at once
  int max_groups_m;    // the same for its matrix-core version
  unsigned spin_limit; // barrier polls before giving up
};
// One recurrence of the adjoint pass: layer l over steps t1, ..., t0+1 of a tile whose states sit in vbuf.
// up: the inter-layer product of that layer and tile, addressed by absolute slot (row (t - t_base - 1)*B + b,
// N_l columns), i.e. the buffer's base shifted back by (t0 - t_base)*B rows.
struct AdjJob { int l, t0, t1, t_base, carry_init; float *vbuf; const float *up; };
struct AdjJobs { AdjJob j[SNN_MAXL]; int count; };
// du_t of a tile into dubuf (slot index as above, [slot][B][O]) and the top layer's product
// up_top[(t - t0 - 1)*B + b][:] = W_out du_t.
hipError_t launch_adjoint_head(const NetDev &net, int t0, int t1, int t_base, float *dubuf, const float *g,
                               float *carry, int carry_init, float *up_top, hipStream_t s,
                               const SpanHook *hook = nullptr);
// up_l[(t - t0 - 1)*B + b][:] = W_in^{l+1} dv^{l+1}_t for a tile whose layer l+1 is done (dv in vbuf).
hipError_t launch_up_product(const NetDev &net, int l, int t0, int t1, int t_base, const float *vbuf, float *up_l,
                             hipStream_t s, const SpanHook *hook = nullptr);
// The recurrences of all jobs; jobs must be independent of each other (different layers of different
// tiles).  Register-stationary layers of equal block size share one launch.
hipError_t launch_adjoint_jobs(const NetDev &net, const AdjJobs &jobs, float *carry, const WsArgs &ws, hipStream_t s,
                               const SpanHook *hook = nullptr);
int ws_max_resident_groups(int device);
int ws_max_resident_groups_mfma(int device);
void adjoint_prepare(const NetDev &net, const WsArgs &ws); // occupancy queries of the wide-layer kernel, at init
// dW[j][:] += sum over t = t1..t0+1 (descending), b ascending, of pre-spike(t - lag, b, j) * post(t, b, :)
// where post(t) sits at slot (t - t_base - 1) of postbuf with row stride post_stride (floats per batch
// element) and column offset post_off.
hipError_t launch_dw(const uint64_t *pre_mask, int pre_words, int n_pre, int lag, const float *postbuf,
                     size_t slot_stride, int post_stride, int post_off, int n_post, int B, int t0, int t1,
                     int t_base, double *dW, hipStream_t s, int pre_ring = 0);
// One weight matrix of the dense dW contraction (see k_dw_mfma).
struct DwDesc {
  const uint64_t *pre_mask; // spike words of the presynaptic layer, [T+1][B][pre_words]
  int pre_words, lag;       // lag 0: spikes of step t; lag 1: spikes of step t-1 (recurrent matrices)
  int n_pre, n_post;
  const float *post;        // adjoint buffer: slot (t - t_base - 1), row b at b*post_stride + post_off
  size_t slot_stride;
  int post_stride, post_off;
  double *acc;              // [n_pre][n_post] fp64 accumulators
  int t0, t1, t_base;       // steps t1, ..., t0+1
  int skip_empty;           // test for K-steps without a spike (pays for sparse presynaptic layers only)
  int tile0, tiles_n;       // filled by the launcher
  int pre_ring;             // > 0: pre_mask holds a ring of that many steps (row = step modulo the ring)
  // Masked recurrent matrix through its compressed rows (k_dw_csr): acc then holds one accumulator per existing
  // synapse, in the order of the compressed entries (NetDev::csr_sub / csr_col); NULL: dense accumulators
  const uint32_t *csr_sub;
  const uint16_t *csr_col;
};
struct DwBatch {
  DwDesc d[2 * SNN_MAXL + 1];
  int count;
  int wide;                 // tile shape, fixed per network (see snn_dw_wide_tiles)
};
hipError_t launch_dw_mfma(DwBatch batch, int B, hipStream_t s);
// The same update event by event from LDS tiles (see k_dw_tile); batch sizes up to 64.
hipError_t launch_dw_tile(DwBatch batch, int B, hipStream_t s);
// The recurrences of a stage and the weight-gradient contraction of the previous stage in one launch
// (see k_bwd_stage).  Only for networks bwd_stage_fusable() accepts; the caller guarantees that the two
// parts touch different tiles.
bool bwd_stage_fusable(const NetDev &net, int dw_wide);
int bwd_pre_placement(const NetDev &net);
// du_t of a tile, computed inside a stage launch (n != 0: present; the launcher turns it into a workgroup count)
struct DuJob { int n, t0, t1, t_base, carry_init; float *dubuf; };
// Recompute work of later chunks that rides in the launch between two stages: part 1 (currents, mode-0 jobs of
// all layers of one or two chunks) and/or part 2 (the scan of another chunk whose currents are already in its
// buffer).
struct PreJobs {
  CurJobs cur;          // mode-0 jobs, count 0 = none
  int ws, lcap, cur_gx; // filled by the launcher
  int n_scan;           // != 0: scan present (the launcher turns it into a workgroup count)
  int t0, t1, t_base, store_all;
  const float *state_in;
  float *buf, *state_out;
  size_t slot_stride;
};
// C[m][:] = A[m][:] W^T, an inter-layer product of the adjoint pass (kind, n_blocks, tiles_m: filled by the launcher)
struct GemmJob { const float *A; int lda; const float *W; int K, N; float *C; int M, kind, n_blocks, tiles_m; };
struct InterJobs { GemmJob g[SNN_MAXL + 1]; int n_gemm; PreJobs pre; };
// pre: recompute work to run on the compute units the contraction leaves free (or in the launch between two
// stages, via launch_bwd_inter: whichever the caller picks)
hipError_t launch_bwd_stage(const NetDev &net, const AdjJobs &jobs, float *carry, DwBatch batch, DuJob du,
                            const float *g, PreJobs pre, hipStream_t s, const SpanHook *hook = nullptr);
hipError_t launch_bwd_inter(const NetDev &net, InterJobs ij, hipStream_t s, const SpanHook *hook = nullptr);
hipError_t launch_transpose(const float *src, float *dst, int rows, int cols, hipStream_t s);
hipError_t launch_finish_grad(const double *acc, const uint8_t *mask_or_null, float *dW, size_t n, hipStream_t s);
// The same for accumulators kept per existing synapse (compressed-row order): dW = 0 where no synapse exists.
hipError_t launch_finish_grad_csr(const double *acc, const uint32_t *csr_sub, const uint16_t *csr_col, int N, float *dW,
                                  hipStream_t s);
hipError_t launch_unpack_spikes(const uint64_t *mask, int words, int N, int T, int B, uint8_t *dst,
                                hipStream_t s);
hipError_t launch_count_spikes(const uint64_t *mask, size_t n_words, unsigned long long *count, hipStream_t s);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s);
hipError_t launch_copy(const void *src, void *dst, size_t bytes, hipStream_t s);
bool snn_kernel_shape_ok(const NetDev &net, char *why, size_t why_len);

// ---- schedule / budget logic (snn_schedule.cpp; plain host code) --------------------------
enum { OP_SAVE_LOCAL = 1, OP_SAVE_REMOTE = 2, OP_LOAD_REMOTE = 3, OP_REFWD1 = 4, OP_KEEP_FINE = 5,
       OP_REFWD2 = 6, OP_BACKWARD = 7, OP_SAVE_BATCH = 8, OP_LOAD_BATCH = 9 };
struct SchedOp { int op, a, b; };
struct Plan {
  int strategy, T, C, F;
  int chunk_len;      // slots of the chunk buffer (trajectory length for STANDARD)
  int n_chunk_bufs;   // chunk buffers (1; n_layers when the adjoint pass runs its layers one chunk apart)
  int n_local_ckpt;   // HBM checkpoints (CHUNK: ceil(T/F); DOUBLE: fine checkpoints per segment)
  int n_load_slots;   // HBM slots receiving host checkpoints (prefetch double buffer)
  int n_stage_slots;  // HBM slots staging device->host copies (layers are pipelined, see launch_forward)
                      // = SNN_FWD_LAG + 2, SNN_FWD_LAG = tiles the lowest layer can be ahead of the top one
  int n_remote;       // host slots
  int n_cache_slots;  // DOUBLE, when the budget has room: the synaptic currents of a whole coarse segment, computed once
                      // by Re-Forward_1 and read again by the scans of Re-Forward_2 (C slots; 0: both passes compute them)
                      // or more: the forward pass then leaves the currents of every step after keep_from there
  int keep_from;      // DOUBLE: a multiple of C; the forward pass keeps the currents of steps (keep_from, T] in the
                      // cache (slot t - keep_from - 1), Re-Forward_1 of those coarse segments computes none (-1: keeps none)
  int local_slots() const { return chunk_len * n_chunk_bufs + n_local_ckpt + n_load_slots + n_stage_slots + n_cache_slots; }
};
// Resolves defaults (0 -> square-root rules) and validates.  Returns false on invalid arguments.
bool snn_make_plan(int strategy, int T, int C, int F, Plan *out);
// Backward-phase schedule (and forward-phase saves first), in execution order.
int64_t snn_make_schedule(const Plan &p, SchedOp *out, int64_t cap);
