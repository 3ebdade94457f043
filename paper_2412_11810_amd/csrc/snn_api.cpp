// C ABI of the LIF-SNN BPTT library: context, weights, input binding, the checkpoint manager that
// maps the paper's local/remote memory hierarchy onto HBM + pinned host memory, and the executor
// that walks a checkpoint schedule (Fig. 1 of the paper) launching the HIP kernels.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/snn.h"
#include "snn_internal.h"

#define SNN_BWD_TILE 256 // steps of the adjoint pass per launch group (bounds the per-chunk scratch)

// Workspace of snn_forward_noalloc: the per-tile currents of the forward pass, which the allocating entry points
// keep in a buffer they size and hipMalloc on demand.  One copy per GPU the library is loaded on, held until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: g_scratch_dev[device]
// is the address kernels and copies get.
#define SNN_NOALLOC_SCRATCH_BYTES ((size_t)16 << 20)
static __device__ __align__(256) unsigned char scratch[SNN_NOALLOC_SCRATCH_BYTES];
#define SNN_MAX_DEVICES 64
static void *g_scratch_dev[SNN_MAX_DEVICES]; // per device ordinal, filled by snn_init with that device current

struct snn_ctx {
  snn_config cfg{};
  NetDev net{};
  hipStream_t stream = nullptr;      // caller's stream (may be the null stream)
  hipStream_t copy_stream = nullptr; // private side stream for checkpoint traffic
  // Host tier of Remote/Double.  Checkpoints of up to host_direct_max bytes are written to and read from the
  // pinned host block by the kernels themselves (it is mapped into the device's address space): for small
  // states the cross-stream synchronisation of a DMA copy costs several times the transfer.  Larger states go
  // through hipMemcpyAsync on the copy stream, overlapped with compute.  SNN_HOST_TIER=dma|direct forces one.
  size_t host_direct_max = (size_t)1 << 20;
  float *W_in[SNN_MAXL]{}, *W_rec[SNN_MAXL]{}, *W_out = nullptr;
  float *W_inT[SNN_MAXL]{}, *W_recT[SNN_MAXL]{}, *W_outT = nullptr;
  float *dW_in[SNN_MAXL]{}, *dW_rec[SNN_MAXL]{}, *dW_out = nullptr;
  double *acc_in[SNN_MAXL]{}, *acc_rec[SNN_MAXL]{}, *acc_out = nullptr; // fp64 gradient accumulators
  uint8_t *rec_mask[SNN_MAXL]{};
  // compressed rows of the masked recurrent matrices (see NetDev::csr_sub); built by snn_set_weights
  uint32_t *csr_sub[SNN_MAXL]{};
  uint16_t *csr_col[SNN_MAXL]{};
  float *csr_val[SNN_MAXL]{};
  uint64_t *csr_pk[SNN_MAXL]{};
  size_t csr_nnz[SNN_MAXL]{};
  // fp64 gradient accumulators per existing synapse, in compressed-row order (k_dw_csr); csr_dw_ok: the entries
  // beyond the 64 per row and sub-range that kernel keeps in registers fit its LDS (64 per 16 rows and sub-range)
  double *acc_csr[SNN_MAXL]{};
  bool csr_dw_ok[SNN_MAXL]{};

  bool dw_csr = true;           // SNN_DW_CSR=0: masked recurrent matrices keep dense accumulators
  size_t mask_words[SNN_MAXL + 1]{}; // words in mask[l] ((T+1)*B*Wd)
  // Spike bitmasks on the host tier (cfg.spike_tier == 1, REMOTE / DOUBLE): the hidden layers' words of the whole
  // sequence live in pinned host memory ([T+1][B][Wd] per layer index 1..L, row 0 zero); HBM holds a ring of
  // ring_steps rows per layer.  mask_full[l] are the whole-sequence arrays in HBM (hidden layers: allocated on first
  // use when spike_tier == 1); net.mask[l] points to whichever a launch should use.
  uint64_t *mask_full[SNN_MAXL + 1]{};
  uint64_t *mask_ring[SNN_MAXL + 1]{};
  int ring_steps = 0;          // rows of the allocated rings
  uint64_t *host_spk = nullptr;
  size_t host_spk_bytes = 0;
  size_t host_spk_off[SNN_MAXL + 2]{}; // word offset of layer index l inside host_spk (for the bound T_spk_rows)
  int host_spk_rows = 0;       // rows per layer the host store is laid out for
  bool spikes_on_host = false; // the hidden spike trains of the last step are in host_spk, not in mask_full
  int32_t *labels = nullptr;
  unsigned char *host_small = nullptr; // pinned: 64 bytes (loss, error flag) + B labels, for calls that must not allocate
  int T_bound = 0;
  int T_spikes = 0; // length of the sequence whose hidden spike trains are stored (0: none since the inputs were bound)
  double *readout = nullptr;
  WsArgs ws{};                // chip-wide recurrent kernel: exchange buffer, barrier counters, error flag
  float *cur_state = nullptr; // [B][SN] state carried through the forward pass
  float *ubar = nullptr, *g = nullptr, *loss_dev = nullptr, *carry = nullptr;
  unsigned long long *counters = nullptr;
  // activation arena (HBM "local memory"), readout-adjoint tile, pinned host checkpoints
  float *arena = nullptr;
  size_t arena_bytes = 0;
  float *dubuf = nullptr; // readout adjoints of a chunk, followed by the inter-layer product scratch
  size_t dubuf_bytes = 0;
  float *host_ckpt = nullptr;
  size_t host_bytes = 0;
  std::vector<hipEvent_t> ev_pool;
  struct GraphKeyT { int strategy, T, C, F, n_chunk_bufs; void *arena, *work, *host; bool dw_event; unsigned long long cur_pol; unsigned sel; void *ring, *host_spk, *mask1; int cache; bool operator==(const GraphKeyT &o) const { return strategy == o.strategy && T == o.T && C == o.C && F == o.F && n_chunk_bufs == o.n_chunk_bufs && arena == o.arena && work == o.work && host == o.host && dw_event == o.dw_event && cur_pol == o.cur_pol && sel == o.sel && ring == o.ring && host_spk == o.host_spk && mask1 == o.mask1 && cache == o.cache; } };
  GraphKeyT graph_key{};
  hipGraphExec_t graph_exec = nullptr;
  bool graphs_enabled = true;   // SNN_GRAPH=0 turns graph replay off
  bool own_stream = false;
  bool dw_event_driven = false; // SNN_DW=event selects the row-by-row kernel instead of the MFMA contraction
  bool dw_tile = false;         // the event-driven tiled kernel instead of the dense contraction (batch <= 64; SNN_DW=tile|mfma)
  bool dw_rate_driven = false;  // ... chosen from the firing rates of the previous step (layers wider than 256, no SNN_DW)
  bool bwd_pipeline = true;     // SNN_BWD_PIPE=0: the adjoint pass finishes every layer of a chunk before the next chunk
  bool bwd_fuse = true;         // SNN_BWD_FUSE=0: weight gradients always in launches of their own
  bool pre_in_stage = true;     // SNN_PRE_IN_STAGE=0: recompute of later chunks in the launch between two stages
  bool rate_driven = false;     // some weight matrix is far beyond the L2: the current kernel follows the firing rates
  bool rf_cache = true;         // SNN_RF_CACHE=0: Double never keeps a segment's currents between its two recompute passes
  bool keep_currents = true;    // SNN_KEEP_CURRENTS=0: the forward pass never leaves currents in that cache
  std::string err;
  size_t Ms() const { return (size_t)cfg.batch * net.SN * sizeof(float); }
};

namespace {

snn_status fail(snn_ctx *c, snn_status s, const std::string &msg) {
  if (c) c->err = msg;
  return s;
}

#define HIPCHK(ctx, call)                                                                          \
  do {                                                                                             \
    hipError_t e_ = (call);                                                                        \
    if (e_ != hipSuccess)                                                                          \
      return fail(ctx, SNN_E_HIP, std::string(#call) + ": " + hipGetErrorString(e_));              \
  } while (0)

bool is_device_ptr(const void *p) {
  hipPointerAttribute_t a;
  if (hipPointerGetAttributes(&a, p) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return a.type == hipMemoryTypeDevice;
}

// Pool of uncached device blocks (never returned to the driver before the process ends).
struct UncachedBlock { int device; size_t bytes; void *ptr; bool busy; };
std::vector<UncachedBlock> &uncached_pool() { static std::vector<UncachedBlock> pool; return pool; }
void *uncached_block(int device, size_t bytes) {
  bytes = (bytes + 320 + 4095) & ~(size_t)4095;
  for (auto &b : uncached_pool())
    if (!b.busy && b.device == device && b.bytes >= bytes) { b.busy = true; return b.ptr; }
  void *p = nullptr;
  if (hipExtMallocWithFlags(&p, bytes, hipDeviceMallocUncached) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  uncached_pool().push_back(UncachedBlock{device, bytes, p, true});
  return p;
}
void uncached_release(int device, void *ptr) {
  for (auto &b : uncached_pool())
    if (b.device == device && b.ptr == ptr) b.busy = false;
}

bool valid_cfg(const snn_config *c, std::string *why) {
  if (!c) { *why = "null config"; return false; }
  if (c->n_in < 1 || c->n_out < 1 || c->n_out > 1024 || c->T < 1 || c->batch < 1) { *why = "sizes must be positive (n_out <= 1024)"; return false; }
  if (c->n_layers < 1 || c->n_layers > SNN_MAX_LAYERS) { *why = "n_layers must be 1..4"; return false; }
  for (int l = 0; l < c->n_layers; ++l)
    if (c->n_hidden[l] < 1 || c->n_hidden[l] > 65535) { *why = "n_hidden must be 1..65535"; return false; }
  if (c->n_in > 65535) { *why = "n_in must be <= 65535"; return false; }
  if (!(c->surr_window == c->surr_window)) { *why = "surr_window must not be NaN"; return false; }
  if (c->spike_tier != 0 && c->spike_tier != 1) { *why = "spike_tier must be 0 or 1"; return false; }
  return true;
}

void fill_shape(const snn_config &c, NetDev *n) {
  n->L = c.n_layers; n->n_in = c.n_in; n->n_out = c.n_out; n->B = c.batch;
  n->off[0] = 0;
  n->Wd[0] = (c.n_in + 63) / 64;
  for (int l = 0; l < c.n_layers; ++l) {
    n->N[l] = c.n_hidden[l];
    n->off[l + 1] = n->off[l] + c.n_hidden[l];
    n->Wd[l + 1] = (c.n_hidden[l] + 63) / 64;
  }
  n->SN = n->off[c.n_layers];
  n->alpha = c.alpha; n->beta = c.beta_out; n->theta = c.theta; n->k = c.surr_beta;
  n->win = c.surr_window;
}

int pre_of(const NetDev &n, int l) { return l == 0 ? n.n_in : n.N[l - 1]; }

// Does the recurrent matrix of layer l accumulate its gradient per existing synapse (k_dw_csr)?  Where the tiled
// event-driven kernel runs, the compressed rows are in use (net.csr_sub follows the SNN_CSR hook), no row is too
// long for it and a time step fits its tile.  Constant during a training step.
bool dw_rec_csr(const snn_ctx *c, int l) {
  return c->dw_tile && c->dw_csr && !c->dw_event_driven && c->net.csr_sub[l] && c->csr_dw_ok[l] && c->acc_csr[l] &&
         c->net.B <= 32;
}

// Test hooks that force a kernel flavour (documented in snn.h): read from the environment at the start of every
// call that launches kernels, so that a test can switch them between two calls on one context.
void read_kernel_hooks(snn_ctx *c) {
  NetDev &n = c->net;
  n.sel_currents = n.sel_adjoint = n.sel_slices = n.sel_csr = n.sel_seq = 0;
  if (const char *e = std::getenv("SNN_SEQ_KERNEL")) n.sel_seq = !std::strcmp(e, "gather") ? 1 : !std::strcmp(e, "rs") ? 2 : 0;
  n.no_fwd_fuse = 0;
  if (const char *e = std::getenv("SNN_FWD_FUSE")) n.no_fwd_fuse = !std::strcmp(e, "0") ? 1 : 0;
  if (const char *e = std::getenv("SNN_CSR")) n.sel_csr = !std::strcmp(e, "0") ? 1 : !std::strcmp(e, "1") ? 2 : 0;
  for (int l = 0; l < n.L; ++l) {
    const bool on = c->csr_sub[l] && n.sel_csr != 1;
    n.csr_sub[l] = on ? c->csr_sub[l] : nullptr;
    n.csr_col[l] = on ? c->csr_col[l] : nullptr;
    n.csr_val[l] = on ? c->csr_val[l] : nullptr;
    n.csr_nnz[l] = on ? (uint32_t)c->csr_nnz[l] : 0u;
    n.csr_pk[l] = on ? c->csr_pk[l] : nullptr;
  }
  if (const char *e = std::getenv("SNN_CURRENTS"))
    n.sel_currents = !std::strcmp(e, "gather") ? 1 : !std::strcmp(e, "mfma") ? 2 : !std::strcmp(e, "dense") ? 3 : 0;
  if (const char *e = std::getenv("SNN_WS_KERNEL"))
    n.sel_adjoint = !std::strcmp(e, "valu") ? 1 : !std::strcmp(e, "stream") ? 2 : !std::strcmp(e, "rows") ? 3 :
                    !std::strcmp(e, "rows_all") ? 4 : !std::strcmp(e, "chip") ? 5 : !std::strcmp(e, "csrw") ? 6 : !std::strcmp(e, "single") ? 7 : !std::strcmp(e, "pair") ? 8 : !std::strcmp(e, "rows64") ? 9 : 0;
  if (const char *e = std::getenv("SNN_SEQ_SLICES")) {
    const int v = std::atoi(e);
    n.sel_slices = (v == 1 || v == 2 || v == 4 || v == 8) ? (unsigned char)v : 0;
  }
}

// per-tile scratch of the adjoint pass: readout adjoints 3 x [tile][B][O] (three tiles alive) + one inter-layer product per layer
// [tile][B][N_l] (the layers run one tile apart, so every layer's product is alive at once); the forward pass
// uses the same scratch for the currents of one time tile
size_t work_bytes(const NetDev &n, int chunk_len) {
  const size_t bwd = (size_t)std::min(chunk_len, SNN_BWD_TILE) * n.B * (3 * n.n_out + n.SN) * sizeof(float);
  // currents of two tiles of every layer (double-buffered) + readout currents of SNN_RO_TILES tiles
  const size_t fwd = (size_t)SNN_FWD_TILE * n.B * (SNN_RO_TILES * n.n_out + 2 * n.SN) * sizeof(float);
  return bwd > fwd ? bwd : fwd;
}

// tile shape of the dense weight-gradient contraction: wide tiles when the network's matrices fill the chip with them
bool dw_wide_tiles(const NetDev &n) {
  int tiles4 = ((n.N[n.L - 1] + 63) / 64) * ((n.n_out + 63) / 64);
  for (int l = 0; l < n.L; ++l)
    tiles4 += ((pre_of(n, l) + 63) / 64) * ((n.N[l] + 63) / 64) + ((n.N[l] + 63) / 64) * ((n.N[l] + 63) / 64);
  return tiles4 >= 256;
}

// rows of the hidden layers' spike ring for a plan (0: the whole sequence stays in HBM).  The ring must hold, in the
// forward pass, the rows between the lowest layer's newest step and the oldest segment whose copy to the host is
// not complete (a segment + the pipeline lag of the layers + a tile), in the backward pass the segment being
// processed, the one being prefetched and the rows the lower layers of the pipelined adjoint pass still read.
int spike_ring_steps(const snn_config &cfg, int strategy, int T, int C) {
  if (cfg.spike_tier != 1 || (strategy != SNN_REMOTE && strategy != SNN_DOUBLE)) return 0;
  const long long r = 2ll * C + 1600;
  return r >= (long long)T + 1 ? 0 : (int)r;
}
size_t spike_bytes(const NetDev &n, int T, int ring = 0) {
  size_t w = (size_t)(T + 1) * n.B * n.Wd[0];
  for (int l = 1; l <= n.L; ++l) w += (size_t)(ring > 0 ? ring : T + 1) * n.B * n.Wd[l];
  return w * 8;
}

void free_csr(snn_ctx *c, int l) {
  (void)hipFree(c->csr_sub[l]); (void)hipFree(c->csr_col[l]); (void)hipFree(c->csr_val[l]); (void)hipFree(c->acc_csr[l]);
  (void)hipFree(c->csr_pk[l]);
  c->csr_sub[l] = nullptr; c->csr_col[l] = nullptr; c->csr_val[l] = nullptr; c->csr_pk[l] = nullptr; c->csr_nnz[l] = 0;
  c->acc_csr[l] = nullptr; c->csr_dw_ok[l] = false;
}

// Compressed rows of a masked recurrent matrix (layout: NetDev::csr_sub).  An entry exists where the mask says a
// synapse exists, whatever its weight; its order inside a row is the ascending postsynaptic index.  Built on the
// host (one pass over the matrix), uploaded once; the stream is idle when this is called.
snn_status build_csr(snn_ctx *c, int l, const float *w, const uint8_t *mask) {
  const int N = c->net.N[l], nsub = (N + SNN_CSR_SUBW - 1) / SNN_CSR_SUBW;
  const size_t ne = (size_t)N * N;
  std::vector<float> wh;
  std::vector<uint8_t> mh;
  if (is_device_ptr(w)) { wh.resize(ne); HIPCHK(c, hipMemcpy(wh.data(), w, ne * 4, hipMemcpyDeviceToHost)); w = wh.data(); }
  if (is_device_ptr(mask)) { mh.resize(ne); HIPCHK(c, hipMemcpy(mh.data(), mask, ne, hipMemcpyDeviceToHost)); mask = mh.data(); }
  size_t nnz = 0;
  for (size_t i = 0; i < ne; ++i) nnz += mask[i] != 0;
  if (nnz > 0x1FF00000ull) return fail(c, SNN_E_INVAL, "recurrent matrix has too many synapses for 32-bit byte offsets of its entries");
  std::vector<uint32_t> sub((size_t)N * (nsub + 1));
  std::vector<uint16_t> col(nnz + 1);
  std::vector<float> val(nnz + 1);
  size_t p = 0;
  for (int j = 0; j < N; ++j) {
    const uint8_t *mr = mask + (size_t)j * N;
    const float *wr = w + (size_t)j * N;
    uint32_t *sr = sub.data() + (size_t)j * (nsub + 1);
    for (int r = 0; r < nsub; ++r) {
      sr[r] = (uint32_t)p;
      const int n1 = std::min(N, (r + 1) * SNN_CSR_SUBW);
      for (int n = r * SNN_CSR_SUBW; n < n1; ++n)
        if (mr[n]) { col[p] = (uint16_t)n; val[p] = wr[n]; ++p; }
    }
    sr[nsub] = (uint32_t)p;
  }
  // k_dw_csr: a wavefront owns 16 consecutive rows of a block of 256 and keeps 64 entries per row and sub-range in
  // registers, up to 64 more per wavefront (and per row) in LDS
  bool dw_ok = true;
  for (int j0 = 0; j0 < N && dw_ok; j0 += 16)
    for (int r = 0; r < nsub && dw_ok; ++r) {
      uint32_t extra = 0;
      for (int j = j0; j < std::min(N, j0 + 16); ++j) {
        const uint32_t *sr = sub.data() + (size_t)j * (nsub + 1);
        const uint32_t n = sr[r + 1] - sr[r];
        if (n > 64) extra += n - 64;
      }
      if (extra > 64) dw_ok = false;
    }
  free_csr(c, l);
  HIPCHK(c, hipMalloc(&c->acc_csr[l], (nnz + 1) * sizeof(double)));
  c->csr_dw_ok[l] = dw_ok;
  HIPCHK(c, hipMalloc(&c->csr_sub[l], sub.size() * 4));
  HIPCHK(c, hipMalloc(&c->csr_col[l], col.size() * 2));
  HIPCHK(c, hipMalloc(&c->csr_val[l], val.size() * 4));
  HIPCHK(c, hipMemcpy(c->csr_sub[l], sub.data(), sub.size() * 4, hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(c->csr_col[l], col.data(), col.size() * 2, hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(c->csr_val[l], val.data(), val.size() * 4, hipMemcpyHostToDevice));
  {
    // packed copy for the gather (layout: NetDev::csr_pk)
    std::vector<uint64_t> pk(nnz + (size_t)nsub * 64);
    for (size_t e = 0; e < nnz; ++e) {
      uint32_t bits;
      memcpy(&bits, &val[e], 4);
      pk[e] = (uint64_t)bits | ((uint64_t)col[e] << 32);
    }
    for (int r = 0; r < nsub; ++r)
      for (int k = 0; k < 64; ++k) pk[nnz + (size_t)r * 64 + k] = (uint64_t)((r + 1) * SNN_CSR_SUBW + k) << 32;
    HIPCHK(c, hipMalloc(&c->csr_pk[l], pk.size() * 8));
    HIPCHK(c, hipMemcpy(c->csr_pk[l], pk.data(), pk.size() * 8, hipMemcpyHostToDevice));
  }
  c->csr_nnz[l] = nnz;
  return SNN_OK;
}

} // namespace

extern "C" {

const char *snn_last_error(const snn_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int32_t snn_state_slots(snn_strategy strategy, int32_t T, int32_t C, int32_t F, int32_t *remote_slots) {
  Plan p;
  if (!snn_make_plan((int)strategy, T, C, F, &p)) return 0;
  if (remote_slots) *remote_slots = p.n_remote;
  return p.local_slots();
}

int64_t snn_schedule(snn_strategy strategy, int32_t T, int32_t C, int32_t F, int32_t *out, int64_t cap) {
  Plan p;
  if (!snn_make_plan((int)strategy, T, C, F, &p)) return -1;
  static_assert(sizeof(SchedOp) == 3 * sizeof(int32_t), "triples");
  return snn_make_schedule(p, reinterpret_cast<SchedOp *>(out), out ? cap : 0);
}

size_t snn_bytes_required(const snn_config *cfg, snn_strategy strategy, int32_t T, int32_t C, int32_t F) {
  std::string why;
  if (!valid_cfg(cfg, &why)) return 0;
  Plan p;
  if (!snn_make_plan((int)strategy, T, C, F, &p)) return 0;
  NetDev n{};
  fill_shape(*cfg, &n);
  char why_shape[160];
  if (!snn_kernel_shape_ok(n, why_shape, sizeof why_shape)) return 0; // a shape snn_init refuses
  const size_t Ms = (size_t)n.B * n.SN * sizeof(float);
  return (size_t)p.local_slots() * Ms + spike_bytes(n, T, spike_ring_steps(*cfg, (int)strategy, T, p.C)) + work_bytes(n, p.chunk_len);
}

snn_status snn_suggest_intervals(const snn_config *cfg, snn_strategy strategy, int32_t T, size_t budget,
                                 int32_t *coarse_out, int32_t *fine_out) {
  std::string why;
  if (!valid_cfg(cfg, &why) || T < 1 || !coarse_out || !fine_out || (int)strategy < 0 || (int)strategy > SNN_HIER)
    return SNN_E_INVAL;
  auto fits = [&](int C, int F) {
    const size_t need = snn_bytes_required(cfg, strategy, T, C, F);
    return need != 0 && (budget == 0 || need <= budget);
  };
  auto isqrt_ceil = [](int x) {
    int r = (int)std::ceil(std::sqrt((double)x));
    while ((long long)r * r < x) ++r;
    while (r > 1 && (long long)(r - 1) * (r - 1) >= x) --r;
    return r < 1 ? 1 : r;
  };
  const int cap = std::min<int>(T, 256); // longer chunks no longer save time (chunk-size study)
  int C = 0, F = 0;
  switch (strategy) {
    case SNN_STANDARD:
      if (!fits(0, 0)) return SNN_E_BUDGET;
      break;
    case SNN_CHUNK:
    case SNN_HIER: {
      // state slots F + ceil(T/F) (+ ring): smallest at sqrt(T), growing with F beyond it
      const int lo = std::min(isqrt_ceil(T), cap);
      const int nb = strategy == SNN_HIER ? isqrt_ceil((T + lo - 1) / lo) : 0;
      for (F = cap; F >= lo && !fits(strategy == SNN_HIER ? isqrt_ceil((T + F - 1) / F) : 0, F); --F) {}
      if (F < lo) {
        if (!fits(nb, lo)) return SNN_E_BUDGET;
        F = lo;
      }
      C = strategy == SNN_HIER ? isqrt_ceil((T + F - 1) / F) : 0;
      break;
    }
    case SNN_REMOTE:
      for (C = cap; C >= 1 && !fits(C, 0); --C) {}
      if (C < 1) return SNN_E_BUDGET;
      break;
    case SNN_DOUBLE: {
      // slots F + ceil(C/F) + const: first the longest chunk F that fits with one fine checkpoint (C = F),
      // then the longest coarse interval (a multiple of F) whose fine checkpoints still fit
      for (F = cap; F >= 1 && !fits(F, F); --F) {}
      if (F < 1) return SNN_E_BUDGET;
      int lo_m = 1, hi_m = (T + F - 1) / F; // C = m * F, capped at T
      auto Cm = [&](int m) { return (int)std::min<long long>((long long)m * F, T); };
      while (lo_m < hi_m) {
        const int mid = lo_m + (hi_m - lo_m + 1) / 2;
        if (fits(Cm(mid), F)) lo_m = mid; else hi_m = mid - 1;
      }
      C = Cm(lo_m);
      break;
    }
  }
  *coarse_out = C;
  *fine_out = F;
  return SNN_OK;
}

snn_status snn_init(const snn_config *cfg, snn_ctx **out) {
  if (!out) return SNN_E_INVAL;
  *out = nullptr;
  std::string why;
  snn_ctx *c = new snn_ctx();
  *out = c; // returned even on failure so that the caller can read the error text
  if (!valid_cfg(cfg, &why)) return fail(c, SNN_E_INVAL, why);
  c->cfg = *cfg;
  fill_shape(*cfg, &c->net);
  if (const char *e = std::getenv("SNN_DW")) c->dw_event_driven = std::strcmp(e, "event") == 0;
  if (const char *e = std::getenv("SNN_HOST_TIER")) {
    if (std::strcmp(e, "dma") == 0) c->host_direct_max = 0;
    else if (std::strcmp(e, "direct") == 0) c->host_direct_max = ~(size_t)0;
  }
  if (const char *e = std::getenv("SNN_GRAPH")) c->graphs_enabled = std::strcmp(e, "0") != 0;
  if (const char *e = std::getenv("SNN_BWD_PIPE")) c->bwd_pipeline = std::strcmp(e, "0") != 0;
  if (const char *e = std::getenv("SNN_BWD_FUSE")) c->bwd_fuse = std::strcmp(e, "0") != 0;
  if (const char *e = std::getenv("SNN_PRE_IN_STAGE")) c->pre_in_stage = std::strcmp(e, "0") != 0;
  if (const char *e = std::getenv("SNN_RF_CACHE")) c->rf_cache = std::strcmp(e, "0") != 0;
  if (const char *e = std::getenv("SNN_KEEP_CURRENTS")) c->keep_currents = std::strcmp(e, "0") != 0;
  if (const char *e = std::getenv("SNN_DW_CSR")) c->dw_csr = std::strcmp(e, "0") != 0;
  read_kernel_hooks(c);
  char buf[256];
  if (!snn_kernel_shape_ok(c->net, buf, sizeof buf)) return fail(c, SNN_E_INVAL, buf);
  int ndev = 0;
  HIPCHK(c, hipGetDeviceCount(&ndev));
  if (cfg->device < 0 || cfg->device >= ndev) return fail(c, SNN_E_INVAL, "no such device");
  HIPCHK(c, hipSetDevice(cfg->device));
  c->stream = (hipStream_t)cfg->stream;
  if (!c->stream) {
    // the legacy default stream cannot be recorded into a graph: work runs on a stream of the library's
    // own; every entry point returns only after that stream has drained, so callers see no difference
    HIPCHK(c, hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking));
    c->own_stream = true;
  }
  HIPCHK(c, hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
  if (cfg->device < SNN_MAX_DEVICES && !g_scratch_dev[cfg->device]) {
    void *p = nullptr;
    HIPCHK(c, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_scratch_dev[cfg->device] = p;
  }
  NetDev &n = c->net;
  const int L = n.L, B = n.B, O = n.n_out;
  if (hipHostMalloc(reinterpret_cast<void **>(&c->host_small), 64 + (size_t)B * 4, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    c->host_small = nullptr;
    return fail(c, SNN_E_HOSTMEM, "pinned host allocation failed");
  }
  for (int l = 0; l < L; ++l) {
    const size_t ni = (size_t)pre_of(n, l) * n.N[l], nr = (size_t)n.N[l] * n.N[l];
    HIPCHK(c, hipMalloc(&c->W_in[l], (ni + nr) * 4)); // [W_in ; W_rec] stacked row-wise
    c->W_rec[l] = c->W_in[l] + ni;
    HIPCHK(c, hipMalloc(&c->W_inT[l], ni * 4));
    HIPCHK(c, hipMalloc(&c->dW_in[l], ni * 4));
    HIPCHK(c, hipMalloc(&c->acc_in[l], ni * 8));
    HIPCHK(c, hipMalloc(&c->acc_rec[l], nr * 8));
    HIPCHK(c, hipMalloc(&c->W_recT[l], nr * 4));
    HIPCHK(c, hipMalloc(&c->dW_rec[l], nr * 4));
    HIPCHK(c, hipMemsetAsync(c->W_in[l], 0, ni * 4, c->stream));
    HIPCHK(c, hipMemsetAsync(c->W_inT[l], 0, ni * 4, c->stream));
    HIPCHK(c, hipMemsetAsync(c->W_rec[l], 0, nr * 4, c->stream));
    HIPCHK(c, hipMemsetAsync(c->W_recT[l], 0, nr * 4, c->stream));
    n.W_in[l] = c->W_in[l]; n.W_rec[l] = c->W_rec[l]; n.W_inT[l] = c->W_inT[l]; n.W_recT[l] = c->W_recT[l];
  }
  const size_t no = (size_t)n.N[L - 1] * O;
  HIPCHK(c, hipMalloc(&c->W_out, no * 4));
  HIPCHK(c, hipMalloc(&c->W_outT, no * 4));
  HIPCHK(c, hipMalloc(&c->dW_out, no * 4));
  HIPCHK(c, hipMalloc(&c->acc_out, no * 8));
  HIPCHK(c, hipMemsetAsync(c->W_out, 0, no * 4, c->stream));
  HIPCHK(c, hipMemsetAsync(c->W_outT, 0, no * 4, c->stream));
  n.W_out = c->W_out; n.W_outT = c->W_outT;
  for (int l = 0; l <= L; ++l) {
    c->mask_words[l] = (size_t)(cfg->T + 1) * B * n.Wd[l];
    if (l > 0 && cfg->spike_tier == 1) continue; // hidden layers: allocated when a call needs the whole sequence in HBM
    HIPCHK(c, hipMalloc(&c->mask_full[l], c->mask_words[l] * 8));
    HIPCHK(c, hipMemsetAsync(c->mask_full[l], 0, c->mask_words[l] * 8, c->stream));
    n.mask[l] = c->mask_full[l];
  }
  HIPCHK(c, hipMalloc(&c->labels, (size_t)B * 4));
  HIPCHK(c, hipMalloc(&c->readout, (size_t)B * 2 * O * 8));
  HIPCHK(c, hipMalloc(&c->ubar, (size_t)B * O * 4));
  HIPCHK(c, hipMalloc(&c->g, (size_t)B * O * 4));
  HIPCHK(c, hipMalloc(&c->loss_dev, 16));
  HIPCHK(c, hipMalloc(&c->carry, (size_t)B * (n.SN + O) * 4));
  HIPCHK(c, hipMalloc(&c->cur_state, (size_t)B * n.SN * 4));
  {
    int nmax = 0;
    for (int l = 0; l < L; ++l) nmax = n.N[l] > nmax ? n.N[l] : nmax;
    if (nmax > 256 && nmax <= 16384 && !std::getenv("SNN_NO_WS")) {
      // exchange buffer + barrier counters in uncached device memory (coherent across the chip
      // without cache maintenance).  Such memory is never freed while the process lives: blocks are
      // kept in a per-process pool and handed out again.
      // one exchange buffer and one set of 64 counters per job of a launch (layers of equal width that are one
      // tile apart share a launch), one error flag
      const size_t n_bar = (size_t)64 * SNN_MAXL + 16; // counters + error flag, padded to a multiple of 64 bytes
      // (the kernel for layers wider than 1024 pads the batch to whole blocks of 16: 1, 2 or 4 of them)
      const size_t bp = nmax > 1024 && B <= 64 ? (size_t)((B + 15) / 16 == 3 ? 4 : (B + 15) / 16) * 16 : (size_t)B;
      const size_t xg_stride = ((size_t)4 * bp * nmax + 15) & ~(size_t)15; // [2][B][N] entries of 8 bytes (value + step tag)
      // (+ 16 KB: readers of the tagged exchange address a row padded to 1024 entries of 8 bytes)
      const size_t bytes = n_bar * sizeof(unsigned) + (size_t)SNN_MAXL * xg_stride * 4 + 16384;
      void *blk = uncached_block(cfg->device, bytes);
      if (!blk) return fail(c, SNN_E_HIP, "uncached device allocation failed");
      c->ws.bar = (unsigned *)blk;
      c->ws.xg = (float *)((char *)blk + n_bar * sizeof(unsigned));
      c->ws.xg_stride = (int)xg_stride;
      HIPCHK(c, hipMemsetAsync(c->ws.bar, 0, n_bar * sizeof(unsigned), c->stream));
      c->ws.err = c->ws.bar + 64 * SNN_MAXL;
      c->ws.max_groups = ws_max_resident_groups(cfg->device);
      c->ws.max_groups_m = ws_max_resident_groups_mfma(cfg->device);
      c->ws.spin_limit = 4000000u; // ~1 s of polling: far beyond any real wait
      if (const char *e = std::getenv("SNN_WS_SPIN_LIMIT")) c->ws.spin_limit = (unsigned)std::strtoul(e, nullptr, 10);
      adjoint_prepare(n, c->ws);
    }
  }
  HIPCHK(c, hipMalloc(&c->counters, 8 * (SNN_MAXL + 1)));
  for (int l = 0; l < L; ++l) {
    const size_t pmax = (size_t)std::max(l == 0 ? n.n_in : n.N[l - 1], n.N[l]);
    if (pmax * n.N[l] * sizeof(float) >= ((size_t)32 << 20)) c->rate_driven = true;
  }
  // The weight-gradient kernel (both give the same bits: per time step an fp32 sum over the batch elements in
  // ascending order, then one fp64 add): the event-driven tiled kernel pays per presynaptic spike, the dense
  // contraction per presynaptic neuron.  Networks with a weight matrix far beyond the L2 always take the tiled kernel
  // (with compressed rows for masked matrices it stays ahead of the dense contraction at 20 % activity as well);
  // other networks with layers wider than 256 follow the firing rates of the previous step, like the current
  // kernels, and start with the dense contraction.
  c->dw_tile = c->rate_driven && B <= 64;
  {
    int nmax = 0;
    for (int l = 0; l < L; ++l) nmax = n.N[l] > nmax ? n.N[l] : nmax;
    c->dw_rate_driven = nmax > 256 && B <= 64 && !c->rate_driven;
  }
  if (const char *e = std::getenv("SNN_DW")) {
    c->dw_rate_driven = false;
    if (!std::strcmp(e, "tile")) c->dw_tile = B <= 64;
    else if (!std::strcmp(e, "mfma") || !std::strcmp(e, "event")) c->dw_tile = false;
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return SNN_OK;
}

void snn_destroy(snn_ctx *c) {
  if (!c) return;
  (void)hipSetDevice(c->cfg.device);
  (void)hipDeviceSynchronize();
  for (int l = 0; l < SNN_MAXL; ++l) {
    (void)hipFree(c->W_in[l]); (void)hipFree(c->W_inT[l]); (void)hipFree(c->W_recT[l]);
    (void)hipFree(c->dW_in[l]); (void)hipFree(c->dW_rec[l]); (void)hipFree(c->rec_mask[l]);
    (void)hipFree(c->csr_sub[l]); (void)hipFree(c->csr_col[l]); (void)hipFree(c->csr_val[l]);
    (void)hipFree(c->csr_pk[l]);
    (void)hipFree(c->acc_in[l]); (void)hipFree(c->acc_rec[l]);
  }
  for (int l = 0; l <= SNN_MAXL; ++l) { (void)hipFree(c->mask_full[l]); (void)hipFree(c->mask_ring[l]); }
  if (c->host_spk) (void)hipHostFree(c->host_spk);
  (void)hipFree(c->W_out); (void)hipFree(c->W_outT); (void)hipFree(c->dW_out); (void)hipFree(c->acc_out);
  (void)hipFree(c->labels); (void)hipFree(c->readout); (void)hipFree(c->ubar); (void)hipFree(c->g);
  (void)hipFree(c->loss_dev); (void)hipFree(c->carry); (void)hipFree(c->cur_state);
  if (c->ws.bar) uncached_release(c->cfg.device, c->ws.bar); (void)hipFree(c->counters);
  (void)hipFree(c->arena); (void)hipFree(c->dubuf);
  if (c->host_ckpt) (void)hipHostFree(c->host_ckpt);
  if (c->host_small) (void)hipHostFree(c->host_small);
  for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
  if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
  if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
  if (c->own_stream && c->stream) (void)hipStreamDestroy(c->stream);
  delete c;
}

snn_status snn_set_weights(snn_ctx *c, int kind, int layer, const float *w, const uint8_t *mask) {
  if (!c || !w) return fail(c, SNN_E_INVAL, "null argument");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  NetDev &n = c->net;
  float *dst, *dstT;
  int rows, cols;
  if (kind == SNN_W_OUT) {
    dst = c->W_out; dstT = c->W_outT; rows = n.N[n.L - 1]; cols = n.n_out;
  } else if ((kind == SNN_W_IN || kind == SNN_W_REC) && layer >= 0 && layer < n.L) {
    dst = kind == SNN_W_IN ? c->W_in[layer] : c->W_rec[layer];
    dstT = kind == SNN_W_IN ? c->W_inT[layer] : c->W_recT[layer];
    rows = kind == SNN_W_IN ? pre_of(n, layer) : n.N[layer];
    cols = n.N[layer];
  } else {
    return fail(c, SNN_E_INVAL, "bad tensor kind/layer");
  }
  if (mask && kind != SNN_W_REC) return fail(c, SNN_E_INVAL, "mask only for recurrent matrices");
  // a recorded step holds the mask pointers of its gradient epilogue: record again after any change of weights
  if (c->graph_exec) {
    HIPCHK(c, hipStreamSynchronize(c->stream));
    (void)hipGraphExecDestroy(c->graph_exec);
    c->graph_exec = nullptr;
  }
  const size_t ne = (size_t)rows * cols;
  HIPCHK(c, hipMemcpyAsync(dst, w, ne * 4, hipMemcpyDefault, c->stream));
  HIPCHK(c, launch_transpose(dst, dstT, rows, cols, c->stream));
  if (kind == SNN_W_REC) {
    if (mask) {
      if (!c->rec_mask[layer]) HIPCHK(c, hipMalloc(&c->rec_mask[layer], ne));
      HIPCHK(c, hipMemcpyAsync(c->rec_mask[layer], mask, ne, hipMemcpyDefault, c->stream));
      HIPCHK(c, hipStreamSynchronize(c->stream));
      const snn_status rs = build_csr(c, layer, w, mask);
      if (rs != SNN_OK) return rs;
    } else if (c->rec_mask[layer]) {
      HIPCHK(c, hipStreamSynchronize(c->stream));
      HIPCHK(c, hipFree(c->rec_mask[layer]));
      c->rec_mask[layer] = nullptr;
      free_csr(c, layer);
    }
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return SNN_OK;
}

snn_status snn_bind_inputs(snn_ctx *c, const uint8_t *in_spikes, const int32_t *labels, int32_t T) {
  if (!c || !in_spikes || !labels) return fail(c, SNN_E_INVAL, "null argument");
  if (T < 1 || T > c->cfg.T) return fail(c, SNN_E_INVAL, "T out of range for this context");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  // inputs may have been produced on the caller's default stream, which the library's own stream
  // does not synchronise with implicitly
  if (c->own_stream) HIPCHK(c, hipStreamSynchronize(nullptr));
  const NetDev &n = c->net;
  {
    // the loss kernel indexes the readout with the label: range-check the B labels on the host first
    std::vector<int32_t> lab((size_t)n.B);
    HIPCHK(c, hipMemcpy(lab.data(), labels, (size_t)n.B * 4, hipMemcpyDefault));
    for (int b = 0; b < n.B; ++b)
      if (lab[b] < 0 || lab[b] >= n.n_out) {
        char msg[96];
        snprintf(msg, sizeof msg, "label %d of batch element %d is outside [0, %d)", (int)lab[b], b, n.n_out);
        return fail(c, SNN_E_INVAL, msg);
      }
  }
  const size_t bytes = (size_t)T * n.B * n.n_in;
  const uint8_t *src = in_spikes;
  uint8_t *tmp = nullptr;
  if (!is_device_ptr(in_spikes)) {
    HIPCHK(c, hipMalloc(&tmp, bytes));
    hipError_t e = hipMemcpyAsync(tmp, in_spikes, bytes, hipMemcpyHostToDevice, c->stream);
    if (e != hipSuccess) { (void)hipFree(tmp); return fail(c, SNN_E_HIP, hipGetErrorString(e)); }
    src = tmp;
  }
  hipError_t e = launch_pack_inputs(src, n.mask[0], T, n.B, n.n_in, n.Wd[0], c->stream);
  if (e == hipSuccess) e = hipMemcpyAsync(c->labels, labels, (size_t)n.B * 4, hipMemcpyDefault, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (tmp) (void)hipFree(tmp);
  if (e != hipSuccess) return fail(c, SNN_E_HIP, hipGetErrorString(e));
  c->T_bound = T;
  c->T_spikes = 0;
  return SNN_OK;
}

// Tile boundaries of a forward pass over (t0, t1]: at most SNN_FWD_TILE steps per tile, and a
// boundary at every multiple of `seg` (the coarse checkpoints of the host tier).
static std::vector<int> tile_bounds(int t0, int t1, int seg) {
  std::vector<int> b{t0};
  for (int a = t0; a < t1;) {
    int e = std::min(a + SNN_FWD_TILE, t1);
    const int next_seg = (a / seg + 1) * seg;
    if (next_seg < e) e = next_seg;
    b.push_back(e);
    a = e;
  }
  return b;
}

static snn_status ensure_work(snn_ctx *c, size_t bytes) {
  if (c->dubuf_bytes >= bytes) return SNN_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (c->dubuf) HIPCHK(c, hipFree(c->dubuf));
  c->dubuf = nullptr; c->dubuf_bytes = 0;
  HIPCHK(c, hipMalloc(&c->dubuf, bytes));
  c->dubuf_bytes = bytes;
  return SNN_OK;
}

// The whole-sequence spike arrays in HBM, which the forward-only pass and the accessors work on.  A context with
// spike_tier 1 allocates its hidden layers' arrays on first use; if the last training step left the hidden spike
// trains in host memory they are brought back first.
static snn_status ensure_full_masks(snn_ctx *c) {
  NetDev &n = c->net;
  for (int l = 1; l <= n.L; ++l)
    if (!c->mask_full[l]) {
      HIPCHK(c, hipMalloc(&c->mask_full[l], c->mask_words[l] * 8));
      HIPCHK(c, hipMemsetAsync(c->mask_full[l], 0, c->mask_words[l] * 8, c->stream));
    }
  if (c->spikes_on_host) {
    for (int l = 1; l <= n.L; ++l)
      HIPCHK(c, hipMemcpyAsync(c->mask_full[l], c->host_spk + c->host_spk_off[l],
                               (size_t)(c->T_spikes + 1) * n.B * n.Wd[l] * 8, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    c->spikes_on_host = false;
  }
  for (int l = 0; l <= n.L; ++l) { n.mask[l] = c->mask_full[l]; n.mring[l] = 0; }
  return SNN_OK;
}

static snn_status forward_only(snn_ctx *c, float *traj_or_null, float *work_or_null = nullptr) {
  read_kernel_hooks(c);
  c->spikes_on_host = false; // this pass rewrites the hidden spike trains, in HBM
  {
    const snn_status rm = ensure_full_masks(c);
    if (rm != SNN_OK) return rm;
  }
  const NetDev &n = c->net;
  StoreSpec st{};
  if (traj_or_null) {
    st.base = traj_or_null; st.slot_stride = (size_t)n.B * n.SN; st.t_base = 0; st.interval = 1; st.slot0 = 0;
    st.t_max = c->T_bound;
  }
  float *work = work_or_null;
  if (!work) { // the caller brought no workspace: the context's own, grown on demand
    snn_status rs = ensure_work(c, work_bytes(n, 1));
    if (rs != SNN_OK) return rs;
    work = c->dubuf;
  }
  HIPCHK(c, launch_fill_zero(c->cur_state, c->Ms(), c->stream));
  std::vector<int> bounds = tile_bounds(0, c->T_bound, c->T_bound);
  HIPCHK(c, launch_forward(n, bounds.data(), (int)bounds.size() - 1, c->cur_state, st, c->readout, 1, work, c->stream, nullptr, nullptr, &c->ws));
  HIPCHK(c, launch_loss(c->readout, c->labels, n.B, n.n_out, c->T_bound, c->ubar, c->g, c->loss_dev, c->stream));
  c->T_spikes = c->T_bound;
  return SNN_OK;
}

static snn_status check_ws_error(snn_ctx *c);
snn_status snn_forward(snn_ctx *c, const uint8_t *in_spikes, const int32_t *labels, int32_t T, float *loss_out) {
  snn_status s = snn_bind_inputs(c, in_spikes, labels, T);
  if (s != SNN_OK) return s;
  s = forward_only(c, nullptr);
  if (s != SNN_OK) return s;
  float loss = 0.f;
  HIPCHK(c, hipMemcpyAsync(&loss, c->loss_dev, 4, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (loss_out) *loss_out = loss;
  return check_ws_error(c); // the sliced sequential kernels of wide layers wait for each other, with a bound
}

snn_status snn_forward_noalloc(snn_ctx *c, const uint8_t *in_spikes, const int32_t *labels, int32_t T, float *loss_out) {
  if (!c || !in_spikes || !labels) return fail(c, SNN_E_INVAL, "null argument");
  if (T < 1 || T > c->cfg.T) return fail(c, SNN_E_INVAL, "T out of range for this context");
  const NetDev &n = c->net;
  const int dev = c->cfg.device;
  if (dev >= SNN_MAX_DEVICES || !g_scratch_dev[dev]) return fail(c, SNN_E_STATE, "no static workspace on this device");
  const size_t need = work_bytes(n, 1);
  if (need > SNN_NOALLOC_SCRATCH_BYTES) {
    char msg[160];
    snprintf(msg, sizeof msg, "snn_forward_noalloc: the forward workspace of this network is %zu B, the static one holds %zu B; "
             "use snn_forward", need, (size_t)SNN_NOALLOC_SCRATCH_BYTES);
    return fail(c, SNN_E_INVAL, msg);
  }
  HIPCHK(c, hipSetDevice(dev));
  for (int l = 1; l <= n.L; ++l)
    if (!c->mask_full[l])
      return fail(c, SNN_E_STATE, "snn_forward_noalloc: this spike_tier-1 context has not allocated its whole-sequence spike "
                                  "arrays yet; call snn_forward once first");
  if (!is_device_ptr(in_spikes) || !is_device_ptr(labels))
    return fail(c, SNN_E_INVAL, "snn_forward_noalloc takes device pointers (a host buffer would need a staging allocation)");
  if (c->own_stream) HIPCHK(c, hipStreamSynchronize(nullptr));
  hipStream_t s = c->stream;
  // labels: to the context and, through the pinned block, to the host for the range check
  int32_t *lab_host = reinterpret_cast<int32_t *>(c->host_small + 64);
  HIPCHK(c, hipMemcpyAsync(lab_host, labels, (size_t)n.B * 4, hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipStreamSynchronize(s));
  for (int b = 0; b < n.B; ++b)
    if (lab_host[b] < 0 || lab_host[b] >= n.n_out) {
      char msg[96];
      snprintf(msg, sizeof msg, "label %d of batch element %d is outside [0, %d)", (int)lab_host[b], b, n.n_out);
      return fail(c, SNN_E_INVAL, msg);
    }
  HIPCHK(c, launch_pack_inputs(in_spikes, n.mask[0], T, n.B, n.n_in, n.Wd[0], s));
  HIPCHK(c, hipMemcpyAsync(c->labels, labels, (size_t)n.B * 4, hipMemcpyDeviceToDevice, s));
  c->T_bound = T;
  c->T_spikes = 0;
  // every current the sequential kernels read from the workspace is written earlier in the same call: nothing in
  // it has to start at zero, and what the previous call left there is never read
  const snn_status rs = forward_only(c, nullptr, static_cast<float *>(g_scratch_dev[dev]));
  if (rs != SNN_OK) return rs;
  float *loss_host = reinterpret_cast<float *>(c->host_small);
  unsigned *err_host = reinterpret_cast<unsigned *>(c->host_small + 16);
  *err_host = 0u;
  HIPCHK(c, hipMemcpyAsync(loss_host, c->loss_dev, 4, hipMemcpyDeviceToHost, s));
  if (c->ws.err) HIPCHK(c, hipMemcpyAsync(err_host, c->ws.err, 4, hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipStreamSynchronize(s));
  if (loss_out) *loss_out = *loss_host;
  if (*err_host) {
    HIPCHK(c, launch_fill_zero(c->ws.err, 4, s));
    HIPCHK(c, hipStreamSynchronize(s));
    return fail(c, SNN_E_HIP, "a workgroup barrier of a chip-wide kernel timed out; results are invalid");
  }
  return SNN_OK;
}

snn_status snn_debug_states(snn_ctx *c, float *dst) {
  if (!c || !dst) return fail(c, SNN_E_INVAL, "null argument");
  if (c->T_bound < 1) return fail(c, SNN_E_STATE, "no inputs bound");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  float *traj = nullptr;
  const size_t bytes = (size_t)c->T_bound * c->Ms();
  HIPCHK(c, hipMalloc(&traj, bytes));
  snn_status s = forward_only(c, traj);
  hipError_t e = hipSuccess;
  if (s == SNN_OK) e = hipMemcpyAsync(dst, traj, bytes, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  (void)hipFree(traj);
  if (s != SNN_OK) return s;
  if (e != hipSuccess) return fail(c, SNN_E_HIP, hipGetErrorString(e));
  return SNN_OK;
}

snn_status snn_get_state(snn_ctx *c, int layer, int32_t t, float *dst) {
  if (!c || !dst || layer < 0 || layer >= c->net.L) return fail(c, SNN_E_INVAL, "bad argument");
  if (c->T_spikes < 1) return fail(c, SNN_E_STATE, "no forward pass since the inputs were bound");
  if (t < 1 || t > c->T_spikes) return fail(c, SNN_E_INVAL, "t outside 1..T");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  read_kernel_hooks(c);
  {
    const snn_status rm = ensure_full_masks(c);
    if (rm != SNN_OK) return rm;
  }
  const NetDev &n = c->net;
  // what a recompute pass does: from x_0 = 0 through the stored spike trains, a chunk of currents at a time
  const int chunk = std::min<int>(t, SNN_FWD_TILE);
  const size_t slot = (size_t)n.B * n.SN;
  float *buf = nullptr;
  HIPCHK(c, hipMalloc(&buf, ((size_t)chunk + 2) * slot * sizeof(float)));
  float *st[2] = {buf + (size_t)chunk * slot, buf + ((size_t)chunk + 1) * slot};
  hipError_t e = launch_fill_zero(st[0], slot * sizeof(float), c->stream);
  int cur = 0;
  for (int a = 0; a < t && e == hipSuccess; a += chunk, cur ^= 1)
    e = launch_recompute(n, a, std::min(a + chunk, (int)t), st[cur], buf, a, slot, 0, st[cur ^ 1], c->stream);
  if (e == hipSuccess)
    e = hipMemcpy2DAsync(dst, (size_t)n.N[layer] * 4, st[cur] + n.off[layer], (size_t)n.SN * 4, (size_t)n.N[layer] * 4,
                         (size_t)n.B, hipMemcpyDefault, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  (void)hipFree(buf);
  if (e != hipSuccess) return fail(c, SNN_E_HIP, hipGetErrorString(e));
  return SNN_OK;
}

snn_status snn_get_spikes(snn_ctx *c, int layer, uint8_t *dst) {
  if (!c || !dst || layer < 0 || layer >= c->net.L) return fail(c, SNN_E_INVAL, "bad argument");
  if (c->T_bound < 1) return fail(c, SNN_E_STATE, "no inputs bound");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  {
    const snn_status rm = ensure_full_masks(c);
    if (rm != SNN_OK) return rm;
  }
  const NetDev &n = c->net;
  const size_t bytes = (size_t)c->T_bound * n.B * n.N[layer];
  uint8_t *tmp = nullptr;
  HIPCHK(c, hipMalloc(&tmp, bytes));
  hipError_t e = launch_unpack_spikes(n.mask[layer + 1], n.Wd[layer + 1], n.N[layer], c->T_bound, n.B, tmp, c->stream);
  if (e == hipSuccess) e = hipMemcpyAsync(dst, tmp, bytes, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  (void)hipFree(tmp);
  if (e != hipSuccess) return fail(c, SNN_E_HIP, hipGetErrorString(e));
  return SNN_OK;
}

snn_status snn_get_readout(snn_ctx *c, float *ubar, float *loss) {
  if (!c) return SNN_E_INVAL;
  if (c->T_bound < 1) return fail(c, SNN_E_STATE, "no inputs bound");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  if (ubar) HIPCHK(c, hipMemcpyAsync(ubar, c->ubar, (size_t)c->net.B * c->net.n_out * 4, hipMemcpyDeviceToHost, c->stream));
  if (loss) HIPCHK(c, hipMemcpyAsync(loss, c->loss_dev, 4, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return SNN_OK;
}

snn_status snn_debug_copy(snn_ctx *c, const void *src, void *dst, size_t bytes) {
  if (!c || !src || !dst) return fail(c, SNN_E_INVAL, "null argument");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  HIPCHK(c, launch_copy(src, dst, bytes, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return SNN_OK;
}

snn_status snn_debug_currents(snn_ctx *c, const uint8_t *const *hidden, int32_t chunk, int32_t reps, float *ms_out) {
  if (!c || !hidden || !ms_out) return fail(c, SNN_E_INVAL, "null argument");
  if (c->T_bound < 1) return fail(c, SNN_E_STATE, "no inputs bound");
  if (chunk < 1 || reps < 1) return fail(c, SNN_E_INVAL, "chunk and reps must be positive");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  read_kernel_hooks(c);
  {
    const snn_status rm = ensure_full_masks(c);
    if (rm != SNN_OK) return rm;
  }
  const NetDev &n = c->net;
  const int T = c->T_bound, B = n.B;
  hipStream_t s = c->stream;
  if (c->own_stream) HIPCHK(c, hipStreamSynchronize(nullptr));
  for (int l = 0; l < n.L; ++l) {
    if (!hidden[l]) continue;
    const size_t bytes = (size_t)T * B * n.N[l];
    const uint8_t *src = hidden[l];
    uint8_t *tmp = nullptr;
    if (!is_device_ptr(src)) {
      HIPCHK(c, hipMalloc(&tmp, bytes));
      hipError_t e = hipMemcpyAsync(tmp, src, bytes, hipMemcpyHostToDevice, s);
      if (e != hipSuccess) { (void)hipFree(tmp); return fail(c, SNN_E_HIP, hipGetErrorString(e)); }
      src = tmp;
    }
    hipError_t e = launch_pack_inputs(src, n.mask[l + 1], T, B, n.N[l], n.Wd[l + 1], s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (tmp) (void)hipFree(tmp);
    if (e != hipSuccess) return fail(c, SNN_E_HIP, hipGetErrorString(e));
  }
  if (chunk > T) chunk = T;
  float *buf = nullptr;
  const size_t slot = (size_t)B * n.SN;
  HIPCHK(c, hipMalloc(&buf, (size_t)chunk * slot * sizeof(float)));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  auto pass = [&]() {
    for (int t0 = 0; t0 < T && e == hipSuccess; t0 += chunk)
      e = launch_recompute_currents(n, t0, std::min(t0 + chunk, T), buf, t0, slot, s);
  };
  if (e == hipSuccess) pass(); // warm-up
  if (e == hipSuccess) e = hipEventRecord(e0, s);
  for (int r = 0; r < reps && e == hipSuccess; ++r) pass();
  if (e == hipSuccess) e = hipEventRecord(e1, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipStreamSynchronize(s);
  (void)hipFree(buf);
  if (e != hipSuccess) return fail(c, SNN_E_HIP, hipGetErrorString(e));
  *ms_out = ms / (float)reps;
  return SNN_OK;
}

snn_status snn_grads(snn_ctx *c, int kind, int layer, float *dst, size_t n_elems) {
  if (!c || !dst) return fail(c, SNN_E_INVAL, "null argument");
  const NetDev &n = c->net;
  const float *src;
  size_t ne;
  if (kind == SNN_W_OUT) { src = c->dW_out; ne = (size_t)n.N[n.L - 1] * n.n_out; }
  else if ((kind == SNN_W_IN || kind == SNN_W_REC) && layer >= 0 && layer < n.L) {
    src = kind == SNN_W_IN ? c->dW_in[layer] : c->dW_rec[layer];
    ne = (size_t)(kind == SNN_W_IN ? pre_of(n, layer) : n.N[layer]) * n.N[layer];
  } else return fail(c, SNN_E_INVAL, "bad tensor kind/layer");
  if (ne != n_elems) return fail(c, SNN_E_INVAL, "n_elems does not match the tensor");
  HIPCHK(c, hipSetDevice(c->cfg.device));
  HIPCHK(c, hipMemcpyAsync(dst, src, ne * 4, hipMemcpyDefault, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return SNN_OK;
}

// ---- the training step ----------------------------------------------------------------------

namespace {
struct Timer {
  snn_ctx *c;
  bool on;
  size_t used = 0;
  struct Span { hipEvent_t a, b; int kind; };
  std::vector<Span> spans;
  hipEvent_t get() {
    if (used == c->ev_pool.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      c->ev_pool.push_back(e);
    }
    return c->ev_pool[used++];
  }
  hipEvent_t mark() {
    hipEvent_t e = get();
    if (e) (void)hipEventRecord(e, c->stream);
    return e;
  }
  void begin(int kind) { if (on) spans.push_back(Span{mark(), nullptr, kind}); }
  void end() { if (on) spans.back().b = mark(); }
  static void hook_begin(void *self, int kind) { static_cast<Timer *>(self)->begin(kind); }
  static void hook_end(void *self) { static_cast<Timer *>(self)->end(); }
  SpanHook hook() { return SpanHook{this, &Timer::hook_begin, &Timer::hook_end}; }
};
} // namespace

// Firing rates of the step that was just queued (spike counts of all stored bitmasks), and from them the current
// kernel of the layers with very large weight matrices for the next step: the event-by-event gather pays per
// presynaptic spike, the dense matrix-core version per presynaptic neuron; measured break-even about 3.5 %.
// (weight gradients of 1024-wide layers, batch 64: tiled kernel 17 / 33 ms at 4.6 / 12 % activity, dense contraction 25.5)
static constexpr double DW_TILE_MAX_ACTIVITY = 0.08;
static snn_status update_current_policy(snn_ctx *c, int T, float *rates_out, bool hidden_counted) {
  const NetDev &n = c->net;
  const int L = n.L, B = n.B;
  hipStream_t s = c->stream;
  // with the spike bitmasks on the host tier the step itself counted the hidden layers' spikes, segment by segment
  if (!hidden_counted) HIPCHK(c, launch_fill_zero(c->counters, 8 * (SNN_MAXL + 1), s));
  for (int l = 0; l <= (hidden_counted ? 0 : L); ++l)
    HIPCHK(c, launch_count_spikes(c->mask_full[l] + (size_t)B * n.Wd[l], (size_t)T * B * n.Wd[l], c->counters + l, s));
  HIPCHK(c, hipStreamSynchronize(s));
  unsigned long long cnt[SNN_MAXL + 1];
  HIPCHK(c, hipMemcpy(cnt, c->counters, sizeof cnt, hipMemcpyDeviceToHost));
  double r[SNN_MAXL + 1];
  for (int l = 0; l <= L; ++l) r[l] = (double)cnt[l] / ((double)T * B * (l == 0 ? n.n_in : n.N[l - 1]));
  if (rates_out)
    for (int l = 0; l < L; ++l) rates_out[l] = (float)r[l + 1];
  // presynaptic activity averaged over the weight rows of all layers
  double ev_fw = 0, ev_re = 0, rows_fw = 0, rows_re = 0;
  for (int l = 0; l < L; ++l) {
    const double p_in = l == 0 ? n.n_in : n.N[l - 1], p_rec = n.N[l], w = n.N[l];
    ev_fw += r[l] * p_in * w; rows_fw += p_in * w;
    ev_re += (r[l] * p_in + r[l + 1] * p_rec) * w; rows_re += (p_in + p_rec) * w;
  }
  // weight gradients: measured break-even of the tiled event-driven kernel and the dense contraction
  if (c->dw_rate_driven) c->dw_tile = ev_re < DW_TILE_MAX_ACTIVITY * rows_re;
  if (c->rate_driven) {
    // one choice for the whole network (jobs of one launch then stay in one launch)
    for (int l = 0; l < L; ++l) {
      c->net.cur_pol[0][l] = ev_fw < 0.035 * rows_fw ? 1 : 2;
      c->net.cur_pol[1][l] = ev_re < 0.035 * rows_re ? 1 : 2;
    }
    // A masked recurrent matrix kept as compressed rows: the gather over them pays per presynaptic spike and per
    // synapse that exists.  Measured at configuration 4's widths (10 % density) the recurrent part of the recompute
    // over compressed rows takes 0.39 of the dense kernel's time at 5 % activity and still wins at 20 % (23.2 against
    // 26.2 ms per 100 steps, feed-forward part dense in both): below (firing rate x density) = 0.025 it goes through
    // the compressed rows (3) while the feed-forward part stays dense.  Above that the recompute is all dense, but the
    // sequential forward part -- event-driven either way -- keeps walking the compressed rows (4) as long as a row's
    // part of a sub-range fits one entry per lane on average (density <= 1/8): at 15-45 % activity it takes 109-134 ms
    // where the walk over the dense-stored rows takes 124-150 (T = 200).
    for (int l = 0; l < L; ++l)
      if (c->csr_sub[l] && c->net.cur_pol[1][l] == 2) {
        const double dens = (double)c->csr_nnz[l] / ((double)n.N[l] * n.N[l]);
        if (r[l + 1] * dens < 0.025) c->net.cur_pol[1][l] = 3;
        else if (dens <= 0.125) c->net.cur_pol[1][l] = 4;
      }
  }
  return SNN_OK;
}

static snn_status check_ws_error(snn_ctx *c) {
  if (!c->ws.err) return SNN_OK;
  unsigned e = 0;
  HIPCHK(c, hipMemcpy(&e, c->ws.err, sizeof e, hipMemcpyDeviceToHost));
  if (e) {
    HIPCHK(c, hipMemset(c->ws.err, 0, sizeof e));
    return fail(c, SNN_E_HIP, "a workgroup barrier of the recurrent adjoint kernel timed out; gradients are invalid");
  }
  return SNN_OK;
}

// Spike bitmasks on the host tier (spike_tier 1): the hidden layers' words of segment g -- steps (g C, (g+1) C] --
// go to pinned host memory on the copy stream once nothing in the forward pass reads them any more, and the ring
// rows they occupied are reused; in the backward pass a segment's rows come back before its recomputation, the
// segment before it is prefetched meanwhile.  Row r of the sequence sits at ring row r % R.
struct SpikeOff {
  snn_ctx *c; int R, C, T; hipStream_t s, cs; Timer *tm; snn_stats *st;
  const FwdCallbacks *inner = nullptr;
  std::vector<hipEvent_t> ev_ready, ev_done; // per segment, reused modulo their number
  int nseg = 0, issued = 0, waited = 0, top_prev_end = 0;
  bool init() {
    nseg = (T + C - 1) / C;
    const int nev = R / C + 6;
    for (int i = 0; i < nev; ++i) {
      ev_ready.push_back(tm->get()); ev_done.push_back(tm->get());
      if (!ev_ready.back() || !ev_done.back()) return false;
    }
    return true;
  }
  // rows r0..r1 (inclusive) of every hidden layer between the ring and the host store
  hipError_t copy_rows(int r0, int r1, bool to_host, hipStream_t q) {
    const NetDev &n = c->net;
    for (int l = 1; l <= n.L; ++l) {
      const size_t rw = (size_t)n.B * n.Wd[l]; // words per row
      for (int a = r0; a <= r1;) {
        const int pos = a % R, len = std::min(r1 - a + 1, R - pos);
        uint64_t *dev = c->mask_ring[l] + (size_t)pos * rw, *host = c->host_spk + c->host_spk_off[l] + (size_t)a * rw;
        const hipError_t e = to_host ? hipMemcpyAsync(host, dev, (size_t)len * rw * 8, hipMemcpyDeviceToHost, q)
                                     : hipMemcpyAsync(dev, host, (size_t)len * rw * 8, hipMemcpyHostToDevice, q);
        if (e != hipSuccess) return e;
        (to_host ? st->spike_d2h_bytes : st->spike_h2d_bytes) += (int64_t)((size_t)len * rw * 8);
        a += len;
      }
    }
    return hipSuccess;
  }
  // spike counts of rows r0..r1 (firing rates), on the compute stream
  hipError_t count_rows(int r0, int r1) {
    const NetDev &n = c->net;
    for (int l = 1; l <= n.L; ++l) {
      const size_t rw = (size_t)n.B * n.Wd[l];
      for (int a = r0; a <= r1;) {
        const int pos = a % R, len = std::min(r1 - a + 1, R - pos);
        const hipError_t e = launch_count_spikes(c->mask_ring[l] + (size_t)pos * rw, (size_t)len * rw, c->counters + l, s);
        if (e != hipSuccess) return e;
        a += len;
      }
    }
    return hipSuccess;
  }
  hipError_t issue(int g) { // segment g leaves for the host
    const int r0 = g * C + 1, r1 = std::min((g + 1) * C, T), k = g % (int)ev_ready.size();
    hipError_t e = count_rows(r0, r1);
    if (e == hipSuccess) e = hipEventRecord(ev_ready[k], s);
    if (e == hipSuccess) e = hipStreamWaitEvent(cs, ev_ready[k], 0);
    if (e == hipSuccess) e = copy_rows(r0, r1, true, cs);
    if (e == hipSuccess) e = hipEventRecord(ev_done[k], cs);
    return e;
  }
  hipError_t issue_upto(int row_limit) { // every segment that ends at or before row_limit
    while (issued < nseg && std::min((issued + 1) * C, T) <= row_limit) {
      const hipError_t e = issue(issued);
      if (e != hipSuccess) return e;
      ++issued;
    }
    return hipSuccess;
  }
  static hipError_t done(void *self, int layer, int t_end) {
    SpikeOff &q = *static_cast<SpikeOff *>(self);
    const NetDev &n = q.c->net;
    hipError_t e = hipSuccess;
    if (layer == 0) {
      // the lowest layer is about to write rows up to t_end + 128 (its next two tiles): the rows R below them must
      // have reached the host
      const int old_row = std::min(t_end + 128, q.T) - q.R;
      if (old_row >= 1) {
        const int g = std::min((old_row - 1) / q.C, q.nseg - 1);
        while (q.waited <= g) {
          if (q.waited >= q.issued) return hipErrorAssert; // the ring is too short for the pipeline lag (never, by its size)
          e = hipStreamWaitEvent(q.s, q.ev_done[q.waited % (int)q.ev_done.size()], 0);
          if (e != hipSuccess) return e;
          ++q.waited;
        }
      }
    }
    if (layer == n.L - 1) {
      // everything that reads rows up to the START of the tile the top layer just finished has been queued
      // (the readout currents of a tile are computed one stage after the top layer's sequential part)
      e = q.issue_upto(q.top_prev_end);
      if (e != hipSuccess) return e;
      q.top_prev_end = t_end;
    }
    return q.inner ? q.inner->layer_tile_done(q.inner->ctx, layer, t_end) : hipSuccess;
  }
};

// Adjoint pass, layers one tile apart.  Layer l of a tile needs layer l+1 of the same tile (through the
// inter-layer product) and layer l of the tile after it in time (through the carried dv): while the top layer
// works on the newest tile, layer L-2 works on the one before, and so on.  The L recurrences of a stage are
// independent and go out together, so the sequential part of the backward pass is as long as one layer's, not
// the sum over layers.  Nothing in the arithmetic depends on the grouping: each recurrence, product and
// weight-gradient update sees the same operands in the same order as when a tile is finished layer by layer.
struct BwdTile { int t0, t1, base, layer; float *vbuf, *du; };
struct BwdPipe {
  snn_ctx *c; const SpanHook *hk; Timer *tm; snn_stats *st; hipStream_t s;
  float *du_base[3]{}, *up[SNN_MAXL]{};
  int du_sel = 0;
  // head of the next tile (du_t and the top layer's product) already computed by the previous stage's launches
  bool head_ready = false;
  float *head_du = nullptr;
  int head_t0 = 0, head_t1 = 0;
  bool first[SNN_MAXL + 1];
  bool dw_wide = false;
  bool fused = false; // the weight gradients of a stage ride along with the recurrences of the next one
  bool pre_in_stage = true; // recompute work of later chunks: in the stage launch (else in the launch between stages)
  std::vector<BwdTile> inflight; // oldest (lowest layer) first
  std::vector<BwdTile> done;     // (tile, layer) pairs whose weight gradients are still to be added
  bool dw_every_stage = true;

  void init(int tile_rows) {
    const NetDev &n = c->net;
    for (int k = 0; k < 3; ++k) du_base[k] = c->dubuf + (size_t)k * tile_rows * n.B * n.n_out;
    float *q = c->dubuf + (size_t)3 * tile_rows * n.B * n.n_out;
    for (int l = 0; l < n.L; ++l) { up[l] = q; q += (size_t)tile_rows * n.B * n.N[l]; }
    for (int l = 0; l <= n.L; ++l) first[l] = true;
    dw_wide = dw_wide_tiles(n);
  }

  // one stage: optionally admit a new tile at the top layer, run one layer of every tile in flight
  struct NextTile { int t0, t1; };
  snn_status stage(const BwdTile *fresh, const NextTile *next = nullptr, const PreJobs *pre = nullptr) {
    const NetDev &n = c->net;
    const int B = n.B, O = n.n_out, L = n.L;
    if (fresh) {
      BwdTile t = *fresh;
      t.layer = L - 1;
      if (head_ready) {
        if (t.t0 != head_t0 || t.t1 != head_t1) return fail(c, SNN_E_STATE, "internal: tile order differs from the one planned");
        t.du = head_du - (size_t)(t.t0 - t.base) * B * O;
        head_ready = false;
      } else {
        // slot (t - base - 1) of the tile lands at row t - t0 - 1; the du of the two tiles before this one is
        // still to be read by their weight-gradient updates
        t.du = du_base[du_sel] - (size_t)(t.t0 - t.base) * B * O;
        du_sel = (du_sel + 1) % 3;
        HIPCHK(c, launch_adjoint_head(n, t.t0, t.t1, t.base, t.du, c->g, c->carry, first[L] ? 1 : 0, up[L - 1], s, hk));
        first[L] = false;
      }
      inflight.push_back(t);
    }
    if (inflight.empty()) return SNN_OK;
    AdjJobs jobs{};
    for (const BwdTile &t : inflight) {
      const int l = t.layer;
      jobs.j[jobs.count++] = AdjJob{l, t.t0, t.t1, t.base, first[l] ? 1 : 0, t.vbuf,
                                    up[l] - (size_t)(t.t0 - t.base) * B * n.N[l]};
      first[l] = false;
    }
    const bool have_pre = pre && (pre->cur.count > 0 || pre->n_scan != 0);
    if (fused) {
      // launch 1: the recurrences, the weight gradients of the previous stage, du_t of the next tile
      DwBatch db{};
      fill_dw_batch(&db);
      DuJob du{};
      if (next) {
        du = DuJob{1, next->t0, next->t1, next->t0, first[L] ? 1 : 0, du_base[du_sel]};
        first[L] = false;
        head_du = du_base[du_sel];
        head_t0 = next->t0; head_t1 = next->t1;
        du_sel = (du_sel + 1) % 3;
      }
      HIPCHK(c, launch_bwd_stage(n, jobs, c->carry, db, du, c->g, (have_pre && pre_in_stage) ? *pre : PreJobs{}, s, hk));
      done.clear();
      // launch 2: the products the next stage's recurrences need, and recompute work for later chunks
      InterJobs ij{};
      for (const BwdTile &t : inflight)
        if (t.layer > 0) {
          const int l = t.layer;
          ij.g[ij.n_gemm++] = GemmJob{t.vbuf + (size_t)(t.t0 - t.base) * B * n.SN + n.off[l], n.SN, n.W_in[l], n.N[l],
                                      n.N[l - 1], up[l - 1], (t.t1 - t.t0) * B, 0, 0, 0};
        }
      if (next) {
        ij.g[ij.n_gemm++] = GemmJob{head_du, O, n.W_out, O, n.N[L - 1], up[L - 1], (next->t1 - next->t0) * B, 0, 0, 0};
        head_ready = true;
      }
      if (have_pre && !pre_in_stage) ij.pre = *pre;
      HIPCHK(c, launch_bwd_inter(n, ij, s, hk));
    } else {
      if (have_pre) return fail(c, SNN_E_STATE, "internal: recompute work attached to an unfused stage");
      HIPCHK(c, launch_adjoint_jobs(n, jobs, c->carry, c->ws, s, hk));
      // what each finished layer feeds: the product for the layer below.  The products of a stage are independent
      // of each other: one launch for all of them (two 160-workgroup products of configuration 2 fill the chip
      // together, not one after the other)
      InterJobs ij{};
      for (const BwdTile &t : inflight)
        if (t.layer > 0) {
          const int l = t.layer;
          ij.g[ij.n_gemm++] = GemmJob{t.vbuf + (size_t)(t.t0 - t.base) * B * n.SN + n.off[l], n.SN, n.W_in[l], n.N[l],
                                      n.N[l - 1], up[l - 1], (t.t1 - t.t0) * B, 0, 0, 0};
        }
      if (ij.n_gemm == 1) {
        for (const BwdTile &t : inflight)
          if (t.layer > 0) HIPCHK(c, launch_up_product(n, t.layer - 1, t.t0, t.t1, t.base, t.vbuf, up[t.layer - 1], s, hk));
      } else if (ij.n_gemm > 1) {
        HIPCHK(c, launch_bwd_inter(n, ij, s, hk));
      }
    }
    for (const BwdTile &t : inflight) done.push_back(t);
    for (BwdTile &t : inflight) --t.layer;
    if (inflight.front().layer < 0) {
      st->bwd_steps += inflight.front().t1 - inflight.front().t0;
      inflight.erase(inflight.begin());
    }
    // weight gradients of everything finished so far: every stage when the layers are pipelined (a full set
    // of matrices per stage), otherwise once per tile, when its last layer is done
    if (fused ? inflight.empty() : (dw_every_stage || inflight.empty())) return emit_dw();
    return SNN_OK;
  }
  void fill_dw_batch(DwBatch *db) const {
    const NetDev &n = c->net;
    const int B = n.B, O = n.n_out, L = n.L, SN = n.SN;
    const size_t slot = (size_t)B * SN;
    db->wide = dw_wide ? 1 : 0;
    for (const BwdTile &t : done) {
      const int l = t.layer;
      if (l == L - 1)
        db->d[db->count++] = DwDesc{n.mask[L], n.Wd[L], 0, n.N[L - 1], O, t.du, (size_t)B * O, O, 0, c->acc_out, t.t0, t.t1, t.base, 0, 0, 0, n.mring[L], nullptr, nullptr};
      db->d[db->count++] = DwDesc{n.mask[l], n.Wd[l], 0, pre_of(n, l), n.N[l], t.vbuf, slot, SN, n.off[l], c->acc_in[l], t.t0, t.t1, t.base, l == 0 ? 1 : 0, 0, 0, n.mring[l], nullptr, nullptr};
      if (dw_rec_csr(c, l))
        db->d[db->count++] = DwDesc{n.mask[l + 1], n.Wd[l + 1], 1, n.N[l], n.N[l], t.vbuf, slot, SN, n.off[l], c->acc_csr[l], t.t0, t.t1, t.base, 0, 0, 0, n.mring[l + 1], n.csr_sub[l], n.csr_col[l]};
      else
        db->d[db->count++] = DwDesc{n.mask[l + 1], n.Wd[l + 1], 1, n.N[l], n.N[l], t.vbuf, slot, SN, n.off[l], c->acc_rec[l], t.t0, t.t1, t.base, 0, 0, 0, n.mring[l + 1], nullptr, nullptr};
    }
  }
  snn_status emit_dw() {
    const NetDev &n = c->net;
    const int B = n.B, O = n.n_out, L = n.L, SN = n.SN;
    const size_t slot = (size_t)B * SN;
    if (done.empty()) return SNN_OK;
    tm->begin(3);
    if (c->dw_event_driven || B > 128) {
      for (const BwdTile &t : done) {
        const int l = t.layer;
        if (l == L - 1)
          HIPCHK(c, launch_dw(n.mask[L], n.Wd[L], n.N[L - 1], 0, t.du, (size_t)B * O, O, 0, O, B, t.t0, t.t1, t.base, c->acc_out, s, n.mring[L]));
        HIPCHK(c, launch_dw(n.mask[l], n.Wd[l], pre_of(n, l), 0, t.vbuf, slot, SN, n.off[l], n.N[l], B, t.t0, t.t1, t.base, c->acc_in[l], s, n.mring[l]));
        HIPCHK(c, launch_dw(n.mask[l + 1], n.Wd[l + 1], n.N[l], 1, t.vbuf, slot, SN, n.off[l], n.N[l], B, t.t0, t.t1, t.base, c->acc_rec[l], s, n.mring[l + 1]));
      }
    } else {
      DwBatch db{};
      fill_dw_batch(&db);
      if (c->dw_tile) HIPCHK(c, launch_dw_tile(db, B, s));
      else HIPCHK(c, launch_dw_mfma(db, B, s));
    }
    tm->end();
    done.clear();
    return SNN_OK;
  }
  snn_status flush() {
    while (!inflight.empty()) {
      const snn_status r = stage(nullptr);
      if (r != SNN_OK) return r;
    }
    return SNN_OK;
  }
};

// Queues one whole training step on the context's streams; no host synchronisation inside, no
// allocation, no hipMemsetAsync (fill kernels instead), so that the same code can be recorded into
// a HIP graph.  The copy stream is forked from and joined back into the compute stream with events.
static snn_status enqueue_step(snn_ctx *c, const Plan &p, snn_stats &st, Timer &tm, hipEvent_t *ev_fwd_out) {
  NetDev &n = c->net;
  const int T = p.T, B = n.B, O = n.n_out, L = n.L, SN = n.SN;
  const int strategy = p.strategy;
  const size_t Ms = c->Ms(), slot = (size_t)B * SN;
  hipStream_t s = c->stream, cs = c->copy_stream;
  const SpanHook hk = tm.hook();
  float *const chunk0 = c->arena;                            // chunk buffer(s) / trajectory
  float *lckpt = chunk0 + (size_t)p.chunk_len * p.n_chunk_bufs * slot; // local checkpoints
  float *loadb = lckpt + (size_t)p.n_local_ckpt * slot;      // 2 slots receiving host checkpoints
  float *stage = loadb + (size_t)p.n_load_slots * slot;      // 2 slots staging D2H copies
  float *ccache = p.n_cache_slots ? stage + (size_t)p.n_stage_slots * slot : nullptr; // currents of a coarse segment
  int cache_a = -1, cache_b = -1; // ccache holds the currents of steps (cache_a, cache_b], slot t - cache_a - 1

  for (int l = 0; l < L; ++l) {
    HIPCHK(c, launch_fill_zero(c->acc_in[l], (size_t)pre_of(n, l) * n.N[l] * 8, s));
    if (dw_rec_csr(c, l)) HIPCHK(c, launch_fill_zero(c->acc_csr[l], c->csr_nnz[l] * 8, s));
    else HIPCHK(c, launch_fill_zero(c->acc_rec[l], (size_t)n.N[l] * n.N[l] * 8, s));
  }
  HIPCHK(c, launch_fill_zero(c->acc_out, (size_t)n.N[L - 1] * O * 8, s));

  // events for the host tier
  const int n_load_ev = strategy == SNN_HIER ? p.n_local_ckpt / p.C : 2; // load slots (HIER: ring positions)
  std::vector<hipEvent_t> ev_load_ready(n_load_ev, nullptr), ev_load_free(n_load_ev, nullptr);
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  std::vector<char> load_used(n_load_ev, 0);
  const bool direct = (strategy == SNN_REMOTE || strategy == SNN_DOUBLE) && Ms <= c->host_direct_max;
  const bool remote = (strategy == SNN_REMOTE || strategy == SNN_DOUBLE || strategy == SNN_HIER) && !direct;
  if (remote) {
    for (int i = 0; i < n_load_ev; ++i) {
      ev_load_ready[i] = tm.get(); ev_load_free[i] = tm.get();
      if (!ev_load_ready[i] || !ev_load_free[i]) return fail(c, SNN_E_HIP, "hipEventCreate failed");
    }
    ev_fork = tm.get(); ev_join = tm.get();
    if (!ev_fork || !ev_join) return fail(c, SNN_E_HIP, "hipEventCreate failed");
    // fork: everything the copy stream does in this step is ordered after this point
    HIPCHK(c, hipEventRecord(ev_fork, s));
    HIPCHK(c, hipStreamWaitEvent(cs, ev_fork, 0));
  }

  // ---- spike bitmasks on the host tier: the launches of this step see the hidden layers' ring ----------------
  const int R = spike_ring_steps(c->cfg, strategy, T, p.C);
  struct MaskGuard { // net.mask / net.mring are per-launch arguments: point them at the ring for this step only
    snn_ctx *c; bool on;
    ~MaskGuard() {
      if (!on) return;
      for (int l = 1; l <= c->net.L; ++l) { c->net.mask[l] = c->mask_full[l]; c->net.mring[l] = 0; }
    }
  } mask_guard{c, R > 0};
  SpikeOff so{c, R, p.C, T, s, cs, &tm, &st};
  hipEvent_t ev_spk[2] = {nullptr, nullptr}, ev_spk_go[2] = {nullptr, nullptr};
  bool spk_first_load = true;
  if (R > 0) {
    for (int l = 1; l <= L; ++l) { n.mask[l] = c->mask_ring[l]; n.mring[l] = R; }
    if (!so.init()) return fail(c, SNN_E_HIP, "hipEventCreate failed");
    for (int i = 0; i < 2; ++i) {
      ev_spk[i] = tm.get(); ev_spk_go[i] = tm.get();
      if (!ev_spk[i] || !ev_spk_go[i]) return fail(c, SNN_E_HIP, "hipEventCreate failed");
    }
    HIPCHK(c, launch_fill_zero(c->counters, 8 * (SNN_MAXL + 1), s));
    // step 0 of every hidden layer (all silent) sits at ring row 0
    for (int l = 1; l <= L; ++l) HIPCHK(c, launch_fill_zero(c->mask_ring[l], (size_t)B * n.Wd[l] * 8, s));
    if (!remote) { // the copy stream joins this step also when the states take the direct tier
      ev_fork = tm.get(); ev_join = tm.get();
      if (!ev_fork || !ev_join) return fail(c, SNN_E_HIP, "hipEventCreate failed");
      HIPCHK(c, hipEventRecord(ev_fork, s));
      HIPCHK(c, hipStreamWaitEvent(cs, ev_fork, 0));
    }
  }
  const FwdCallbacks cb_spk{&so, &SpikeOff::done};

  // ---- forward ------------------------------------------------------------------------------
  HIPCHK(c, launch_fill_zero(c->cur_state, Ms, s)); // x_0
  if (strategy == SNN_STANDARD) {
    StoreSpec sp{chunk0, slot, 0, 1, 0, T, 0};
    const std::vector<int> bounds = tile_bounds(0, T, T);
    HIPCHK(c, launch_forward(n, bounds.data(), (int)bounds.size() - 1, c->cur_state, sp, c->readout, 1, c->dubuf, s, &hk, nullptr, &c->ws));
  } else if (strategy == SNN_CHUNK) {
    HIPCHK(c, launch_fill_zero(lckpt, Ms, s)); // x_0
    StoreSpec sp{lckpt, slot, 0, p.F, 1, T - 1, 0};
    const std::vector<int> bounds = tile_bounds(0, T, T);
    HIPCHK(c, launch_forward(n, bounds.data(), (int)bounds.size() - 1, c->cur_state, sp, c->readout, 1, c->dubuf, s, &hk, nullptr, &c->ws));
  } else if (strategy == SNN_HIER) {
    // Checkpoint k = x_{kF} goes to slot k mod 2*nb_local of a ring of two batches.  When every layer
    // has passed the last checkpoint of a batch (and it is not the final batch), the batch travels to
    // the host as one transfer; the ring half is reused two batches later.
    const int NL = p.C, n_ckpt = (T + p.F - 1) / p.F, n_batches = (n_ckpt + NL - 1) / NL;
    const int RB = p.n_local_ckpt / NL; // ring positions (batches)
    struct Hier {
      snn_ctx *c; const Plan *p; float *ring; size_t slot, Ms; int NL, RB, n_batches; hipStream_t s, cs;
      std::vector<hipEvent_t> ready, freed; std::vector<char> busy; int waited_for; snn_stats *st;
      static hipError_t done(void *self, int layer, int t_end) {
        Hier &q = *static_cast<Hier *>(self);
        const NetDev &n = q.c->net;
        const int F = q.p->F, T = q.p->T;
        hipError_t e = hipSuccess;
        if (layer == 0) {
          // the first checkpoint of batch g lands at step g*NL*F: before the tile that ends there is
          // queued, the ring position it reuses (batch g - RB) must have left for the host
          const int g = (t_end + F) / (q.NL * F);
          if (g >= q.RB && g < q.n_batches && t_end < g * q.NL * F && q.waited_for < g && q.busy[g % q.RB]) {
            e = hipStreamWaitEvent(q.s, q.freed[g % q.RB], 0);
            q.waited_for = g;
          }
          if (e != hipSuccess) return e;
        }
        if (layer != n.L - 1 || t_end % F != 0 || t_end >= T) return e;
        const int k = t_end / F; // checkpoint index just completed by every layer
        if (k % q.NL != q.NL - 1 || k / q.NL >= q.n_batches - 1) return e;
        const int g = k / q.NL, pos = g % q.RB;
        e = hipEventRecord(q.ready[pos], q.s);
        if (e == hipSuccess) e = hipStreamWaitEvent(q.cs, q.ready[pos], 0);
        if (e == hipSuccess)
          e = hipMemcpyAsync(q.c->host_ckpt + (size_t)g * q.NL * q.slot, q.ring + (size_t)pos * q.NL * q.slot,
                             (size_t)q.NL * q.Ms, hipMemcpyDeviceToHost, q.cs);
        if (e == hipSuccess) e = hipEventRecord(q.freed[pos], q.cs);
        q.busy[pos] = 1;
        q.st->n_d2h++; q.st->d2h_bytes += (int64_t)q.NL * (int64_t)q.Ms;
        return e;
      }
    } hier{c, &p, lckpt, slot, Ms, NL, RB, n_batches, s, cs, {}, {}, {}, 0, &st};
    for (int i = 0; i < RB; ++i) {
      hier.ready.push_back(tm.get()); hier.freed.push_back(tm.get()); hier.busy.push_back(0);
      if (!hier.ready.back() || !hier.freed.back()) return fail(c, SNN_E_HIP, "hipEventCreate failed");
    }
    HIPCHK(c, launch_fill_zero(lckpt, Ms, s)); // x_0 = checkpoint 0
    StoreSpec sp{lckpt, slot, 0, p.F, 1, T - 1, RB * NL};
    const FwdCallbacks cb{&hier, &Hier::done};
    const std::vector<int> bounds = tile_bounds(0, T, p.F);
    HIPCHK(c, launch_forward(n, bounds.data(), (int)bounds.size() - 1, c->cur_state, sp, c->readout, 1, c->dubuf, s, &hk, &cb, &c->ws));
  } else if (direct) {
    // x_0 lives in host slot 0 (zeroed on the host); the sequential kernels store x_{KC} into host slot K
    StoreSpec sp{c->host_ckpt, slot, 0, p.C, 1, T - 1, 0};
    if (ccache && p.keep_from >= 0) { // the currents of the last coarse segment(s) stay for the backward pass
      sp.cur = ccache;
      sp.cur_from = p.keep_from;
      cache_a = p.keep_from; cache_b = T;
    }
    const std::vector<int> bounds = tile_bounds(0, T, T); // no host-side work at the checkpoints: full tiles
    HIPCHK(c, launch_forward(n, bounds.data(), (int)bounds.size() - 1, c->cur_state, sp, c->readout, 1, c->dubuf, s, &hk, R > 0 ? &cb_spk : nullptr, &c->ws));
    st.n_d2h += p.n_remote - 1;
    st.d2h_bytes += (int64_t)(p.n_remote - 1) * (int64_t)Ms;
  } else {
    // x_0 lives in host slot 0, zeroed when the pinned block was allocated and never written again.
    // The sequential kernels write each layer's part of a coarse checkpoint x_{KC} straight into a
    // staging slot (ring of n_stage slots: the layers run one tile apart, so several checkpoints are
    // being assembled at once); when the last layer's part is in, the slot goes to the host on the
    // copy stream.  Before the lowest layer starts the tile that ends at a boundary, the compute
    // stream waits for the copy that last used that boundary's slot.
    struct Snap {
      snn_ctx *c; const Plan *p; float *stage; size_t slot, Ms; int n_stage; hipStream_t s, cs;
      std::vector<hipEvent_t> ready, freed; std::vector<char> busy; snn_stats *st;
      int waited_for = 0; // highest checkpoint index whose slot has been waited for
      hipError_t reserve(int t_done) { // layer 0 has finished step t_done: make the next boundary's slot writable
        const int K = t_done / p->C + 1, so = K % n_stage;
        if (K <= waited_for || (long long)K * p->C >= p->T) return hipSuccess;
        waited_for = K;
        return busy[so] ? hipStreamWaitEvent(s, freed[so], 0) : hipSuccess;
      }
      static hipError_t done(void *self, int layer, int t_end) {
        Snap &q = *static_cast<Snap *>(self);
        const NetDev &n = q.c->net;
        hipError_t e = hipSuccess;
        if (layer == 0) e = q.reserve(t_end);
        if (e != hipSuccess || layer != n.L - 1 || t_end % q.p->C != 0 || t_end >= q.p->T) return e;
        const int K = t_end / q.p->C, so = K % q.n_stage; // checkpoint x_{K*C} -> host slot K
        e = hipEventRecord(q.ready[so], q.s);
        if (e == hipSuccess) e = hipStreamWaitEvent(q.cs, q.ready[so], 0);
        if (e == hipSuccess)
          e = hipMemcpyAsync(q.c->host_ckpt + (size_t)K * q.slot, q.stage + (size_t)so * q.slot, q.Ms, hipMemcpyDeviceToHost, q.cs);
        if (e == hipSuccess) e = hipEventRecord(q.freed[so], q.cs);
        q.busy[so] = 1;
        q.st->n_d2h++; q.st->d2h_bytes += (int64_t)q.Ms;
        return e;
      }
    } snap{c, &p, stage, slot, Ms, p.n_stage_slots, s, cs, {}, {}, {}, &st};
    for (int i = 0; i < p.n_stage_slots; ++i) {
      snap.ready.push_back(tm.get()); snap.freed.push_back(tm.get()); snap.busy.push_back(0);
      if (!snap.ready.back() || !snap.freed.back()) return fail(c, SNN_E_HIP, "hipEventCreate failed");
    }
    const FwdCallbacks cb{&snap, &Snap::done};
    so.inner = &cb;
    const std::vector<int> bounds = tile_bounds(0, T, p.C);
    HIPCHK(c, snap.reserve(0)); // nothing to wait for yet; marks checkpoint 1 as reserved
    StoreSpec sp{stage, slot, 0, p.C, 1, T - 1, p.n_stage_slots}; // x_{KC} -> staging slot K % n_stage
    if (ccache && p.keep_from >= 0) { // the currents of the last coarse segment(s) stay for the backward pass
      sp.cur = ccache;
      sp.cur_from = p.keep_from;
      cache_a = p.keep_from; cache_b = T;
    }
    HIPCHK(c, launch_forward(n, bounds.data(), (int)bounds.size() - 1, c->cur_state, sp, c->readout, 1, c->dubuf, s, &hk, R > 0 ? &cb_spk : &cb, &c->ws));
    so.inner = nullptr;
  }
  if (R > 0) HIPCHK(c, so.issue_upto(T)); // everything of the forward pass is queued: the remaining segments leave
  st.fwd_steps = T;
  HIPCHK(c, launch_loss(c->readout, c->labels, B, O, T, c->ubar, c->g, c->loss_dev, s));
  if (ev_fwd_out) *ev_fwd_out = tm.mark();

  // ---- backward: walk the schedule ------------------------------------------------------------
  std::vector<SchedOp> ops((size_t)snn_make_schedule(p, nullptr, 0));
  snn_make_schedule(p, ops.data(), (int64_t)ops.size());
  int seg_start = 0, chunk_base = 0, cur_load = 0, n_loads = 0;
  const float *seg_src = nullptr; // state the current remote segment starts from (HBM load slot or host slot)
  // Chunk buffers form a ring of n_chunk_bufs: with the layers of the adjoint pass one chunk apart, the
  // lower layers of the previous chunk(s) are still being worked on while the next one is recomputed.
  int n_chunks_done = 0;
  float *chunk = chunk0; // buffer the next recomputation fills
  const bool pipelined = L > 1 && c->bwd_pipeline && (strategy == SNN_STANDARD || p.n_chunk_bufs >= L);
  BwdPipe pipe{c, &hk, &tm, &st, s};
  pipe.init(std::min(p.chunk_len, SNN_BWD_TILE));
  pipe.dw_every_stage = pipelined;
  pipe.pre_in_stage = c->pre_in_stage;
  pipe.fused = pipelined && c->bwd_fuse && !c->dw_event_driven && !c->dw_tile && bwd_stage_fusable(n, pipe.dw_wide) &&
               (strategy == SNN_STANDARD || p.n_chunk_bufs >= L + 1);
  // Recompute ahead: with two more chunk buffers the currents of the chunk two stages ahead and the scan of
  // the chunk one stage ahead ride in the stage launch (see k_bwd_stage).  pre_state[i] tells how far the
  // recompute of the REFWD2 op at index i has got (0 nothing, 1 currents in its buffer, 2 states in its buffer).
  const int pre_place = bwd_pre_placement(n);
  const bool prefetch = pipe.fused && strategy != SNN_STANDARD && p.n_chunk_bufs >= L + 3 && pre_place > 0;
  if (pre_place < 2) pipe.pre_in_stage = false;
  std::vector<char> pre_state(ops.size(), 0);
  std::vector<int> refwd2_ordinal(ops.size(), -1);
  {
    int k = 0;
    for (size_t i = 0; i < ops.size(); ++i)
      if (ops[i].op == OP_REFWD2) refwd2_ordinal[i] = k++;
  }
  // every tile of the adjoint pass in order (their time ranges are fixed by the schedule): the head of a
  // tile (du_t, the top layer's product) is computed one stage early
  std::vector<BwdPipe::NextTile> all_tiles;
  for (const SchedOp &o : ops)
    if (o.op == OP_BACKWARD)
      for (int t1 = o.a; t1 >= o.b; t1 -= SNN_BWD_TILE) all_tiles.push_back({std::max(o.b - 1, t1 - SNN_BWD_TILE), t1});
  size_t tile_no = 0;
  auto buf_of = [&](size_t i) { return chunk0 + (size_t)(refwd2_ordinal[i] % p.n_chunk_bufs) * p.chunk_len * slot; };
  // Looks past op index `from` for the next `want` REFWD2 ops that can be started early: nothing between here
  // and them may change what they read (a fine-checkpoint pass, a batch or DMA load).  Returns how many were
  // found; idx[k] is the op index, src[k] the state the k-th one starts from.
  auto peek = [&](size_t from, int want, size_t *idx, const float **src) {
    int found = 0, ss = seg_start;
    const float *sp = seg_src;
    for (size_t j = from + 1; j < ops.size() && found < want; ++j) {
      const SchedOp &o = ops[j];
      if (o.op == OP_REFWD1 || o.op == OP_LOAD_BATCH) break;
      if (o.op == OP_LOAD_REMOTE) {
        if (!direct || R > 0) break; // (with the spike bitmasks on the host tier the next segment's rows are not in yet)
        ss = o.a;
        sp = c->host_ckpt + (size_t)(o.a / p.C) * slot;
        continue;
      }
      if (o.op != OP_REFWD2) continue;
      const float *q;
      if (strategy == SNN_CHUNK) q = lckpt + (size_t)(o.a / p.F) * slot;
      else if (strategy == SNN_HIER) q = lckpt + (size_t)((o.a / p.F) % p.n_local_ckpt) * slot;
      else if (strategy == SNN_REMOTE || o.a == ss) q = sp;
      else q = lckpt + (size_t)((o.a - ss) / p.F - 1) * slot;
      idx[found] = j;
      src[found] = q;
      ++found;
    }
    return found;
  };
  // host->device loads run on the copy stream, behind every device->host copy of the forward pass
  auto issue_load = [&](int K, int slot_i) -> hipError_t {
    hipError_t e = hipSuccess;
    if (load_used[slot_i]) e = hipStreamWaitEvent(cs, ev_load_free[slot_i], 0);
    if (e == hipSuccess) e = hipMemcpyAsync(loadb + (size_t)slot_i * slot, c->host_ckpt + (size_t)K * slot, Ms, hipMemcpyHostToDevice, cs);
    if (e == hipSuccess) e = hipEventRecord(ev_load_ready[slot_i], cs);
    st.n_h2d++; st.h2d_bytes += (int64_t)Ms;
    return e;
  };
  // HIER: one transfer brings a whole batch of nb_local checkpoints into a half of the ring
  auto issue_batch_load = [&](int g) -> hipError_t {
    const int half = g % n_load_ev;
    hipError_t e = hipSuccess;
    if (load_used[half]) e = hipStreamWaitEvent(cs, ev_load_free[half], 0);
    if (e == hipSuccess)
      e = hipMemcpyAsync(lckpt + (size_t)half * p.C * slot, c->host_ckpt + (size_t)g * p.C * slot, (size_t)p.C * Ms, hipMemcpyHostToDevice, cs);
    if (e == hipSuccess) e = hipEventRecord(ev_load_ready[half], cs);
    st.n_h2d++; st.h2d_bytes += (int64_t)p.C * (int64_t)Ms;
    return e;
  };
  const int hier_batches = strategy == SNN_HIER ? (((T + p.F - 1) / p.F) + p.C - 1) / p.C : 0;
  int hier_cur = hier_batches - 1; // batch whose ring half the chunks are reading
  if (strategy == SNN_HIER) {
    // the final batch is still in its ring half; the one before it can start travelling back now,
    // as soon as the forward pass no longer needs the other half (its last device->host copy is
    // ordered before this on the copy stream)
    if (hier_batches >= 2) HIPCHK(c, issue_batch_load(hier_batches - 2));
  } else if (remote) HIPCHK(c, issue_load(p.n_remote - 1, (p.n_remote - 1) & 1));
  for (size_t i = 0; i < ops.size(); ++i) {
    const SchedOp &op = ops[i];
    switch (op.op) {
      case OP_LOAD_REMOTE: {
        const int K = op.a / p.C;
        if (R > 0) {
          // this segment's spike rows [K C, end] are in the ring before anything of the segment is recomputed
          // (row K C is the previous step of its first one); the rows of the segment before it follow while this
          // one is worked on.  A load waits for everything queued so far: what it overwrites was read by work of
          // segments at least 1600 steps later in the sequence, beyond the lag of the pipelined adjoint pass.
          if (spk_first_load) {
            HIPCHK(c, hipEventRecord(ev_spk_go[K & 1], s));
            HIPCHK(c, hipStreamWaitEvent(cs, ev_spk_go[K & 1], 0));
            HIPCHK(c, so.copy_rows(K * p.C, std::min((K + 1) * p.C, T), false, cs));
            HIPCHK(c, hipEventRecord(ev_spk[K & 1], cs));
            spk_first_load = false;
          }
          HIPCHK(c, hipStreamWaitEvent(s, ev_spk[K & 1], 0));
          if (K > 0) {
            HIPCHK(c, hipEventRecord(ev_spk_go[(K - 1) & 1], s));
            HIPCHK(c, hipStreamWaitEvent(cs, ev_spk_go[(K - 1) & 1], 0));
            HIPCHK(c, so.copy_rows((K - 1) * p.C, K * p.C - 1, false, cs));
            HIPCHK(c, hipEventRecord(ev_spk[(K - 1) & 1], cs));
          }
        }
        if (direct) { // the recompute kernels read x_{KC} from the host slot themselves
          seg_start = op.a;
          seg_src = c->host_ckpt + (size_t)K * slot;
          st.n_h2d++; st.h2d_bytes += (int64_t)Ms;
          break;
        }
        if (n_loads > 0) {
          // the segment that used the previous slot is fully queued: mark that slot reusable
          HIPCHK(c, hipEventRecord(ev_load_free[cur_load], s));
          load_used[cur_load] = 1;
        }
        cur_load = K & 1;
        seg_start = op.a;
        HIPCHK(c, hipStreamWaitEvent(s, ev_load_ready[cur_load], 0));
        seg_src = loadb + (size_t)cur_load * slot;
        ++n_loads;
        // prefetch the next (earlier) coarse checkpoint into the other slot, overlapped with this
        // segment's recomputation and backward pass
        if (K > 0) HIPCHK(c, issue_load(K - 1, (K - 1) & 1));
        break;
      }
      case OP_LOAD_BATCH: {
        const int g = op.a / (p.C * p.F);
        // every chunk of the batch processed before this one is queued: its ring half may be reused
        HIPCHK(c, hipEventRecord(ev_load_free[hier_cur % n_load_ev], s));
        load_used[hier_cur % n_load_ev] = 1;
        hier_cur = g;
        HIPCHK(c, hipStreamWaitEvent(s, ev_load_ready[g % n_load_ev], 0));
        if (g > 0) HIPCHK(c, issue_batch_load(g - 1));
        break;
      }
      case OP_REFWD1: {
        // rebuild the fine checkpoints x_{a+F}, x_{a+2F}, ..., x_b, one fine interval at a time: the
        // chunk buffer takes the currents of the interval, the scan keeps only its last state
        if (ccache && !(cache_a >= 0 && op.a >= cache_a && op.b <= cache_b)) { // (the forward pass left none for it)
          // the currents of the whole segment in one launch, kept for Re-Forward_2
          const int seg_end = std::min((op.a / p.C + 1) * p.C, T);
          tm.begin(1);
          HIPCHK(c, launch_recompute_currents(n, op.a, seg_end, ccache, op.a, slot, s));
          tm.end();
          st.refwd_current_steps += seg_end - op.a;
          cache_a = op.a; cache_b = seg_end;
        }
        for (int a = op.a, m = 0; a < op.b; a += p.F, ++m) {
          const float *src = m == 0 ? seg_src : lckpt + (size_t)(m - 1) * slot;
          if (!ccache) {
            tm.begin(1);
            HIPCHK(c, launch_recompute_currents(n, a, a + p.F, chunk, a, slot, s));
            tm.end();
            st.refwd_current_steps += p.F;
          }
          tm.begin(9);
          if (ccache) HIPCHK(c, launch_recompute_scan(n, a, a + p.F, src, ccache, cache_a, slot, 0, lckpt + (size_t)m * slot, s));
          else HIPCHK(c, launch_recompute_scan(n, a, a + p.F, src, chunk, a, slot, 0, lckpt + (size_t)m * slot, s));
          tm.end();
        }
        st.refwd1_steps += op.b - op.a;
        break;
      }
      case OP_REFWD2: {
        const float *src;
        if (strategy == SNN_CHUNK) src = lckpt + (size_t)(op.a / p.F) * slot;
        else if (strategy == SNN_HIER) src = lckpt + (size_t)((op.a / p.F) % p.n_local_ckpt) * slot;
        else if (strategy == SNN_REMOTE || op.a == seg_start) src = seg_src;
        else src = lckpt + (size_t)((op.a - seg_start) / p.F - 1) * slot;
        chunk_base = op.a;
        if (pre_state[i] < 2) {
          const bool cached = ccache && cache_a >= 0 && op.a >= cache_a && op.b <= cache_b; // Re-Forward_1 left them
          if (pre_state[i] == 0 && !cached) {
            tm.begin(1);
            HIPCHK(c, launch_recompute_currents(n, op.a, op.b, chunk, op.a, slot, s));
            tm.end();
            st.refwd_current_steps += op.b - op.a;
          }
          tm.begin(9);
          HIPCHK(c, launch_recompute_scan(n, op.a, op.b, src, chunk, op.a, slot, 1, nullptr, s, cached ? ccache : nullptr, cache_a));
          tm.end();
        }
        st.refwd2_steps += op.b - op.a;
        break;
      }
      case OP_BACKWARD: {
        // long spans (Standard: the whole sequence) are walked in tiles of SNN_BWD_TILE steps so that
        // the per-tile scratch stays small; neither the adjoint recurrence (carried state) nor the
        // weight-gradient accumulation (continued per element) depends on where the cuts fall
        const int base = strategy == SNN_STANDARD ? 0 : chunk_base;
        for (int t1 = op.a; t1 >= op.b; t1 -= SNN_BWD_TILE) {
          const int t0 = std::max(op.b - 1, t1 - SNN_BWD_TILE);
          const BwdTile tile{t0, t1, base, 0, chunk, nullptr};
          PreJobs pre{};
          if (prefetch && t1 == op.a) { // once per chunk, with its first tile
            size_t idx[2];
            const float *src[2];
            const int found = peek(i, 2, idx, src);
            if (found >= 1 && pre_state[idx[0]] == 1) { // scan of the next chunk
              const SchedOp &o = ops[idx[0]];
              pre.n_scan = 1;
              pre.t0 = o.a; pre.t1 = o.b; pre.t_base = o.a; pre.store_all = 1;
              pre.state_in = src[0]; pre.buf = buf_of(idx[0]); pre.state_out = nullptr; pre.slot_stride = slot;
              pre_state[idx[0]] = 2;
            }
            for (int k = 0; k < found; ++k) // currents of the chunks that have none yet (two only when the pipeline starts)
              if (pre_state[idx[k]] == 0) {
                const SchedOp &o = ops[idx[k]];
                for (int l = 0; l < L; ++l)
                  pre.cur.j[pre.cur.count++] = CurJob{0, l, o.a, o.b - o.a, o.a, buf_of(idx[k]), slot};
                pre_state[idx[k]] = 1;
              }
          }
          const BwdPipe::NextTile *next = tile_no + 1 < all_tiles.size() ? &all_tiles[tile_no + 1] : nullptr;
          ++tile_no;
          snn_status rs = pipe.stage(&tile, pipe.fused ? next : nullptr, &pre);
          if (rs == SNN_OK && !pipelined) rs = pipe.flush();
          if (rs != SNN_OK) return rs;
        }
        if (strategy != SNN_STANDARD) { // the next recomputation goes to the next buffer of the ring
          ++n_chunks_done;
          chunk = chunk0 + (size_t)(n_chunks_done % p.n_chunk_bufs) * p.chunk_len * slot;
        }
        break;
      }
      default:
        break; // SAVE_* happen in the forward pass; KEEP_FINE is part of REFWD1
    }
  }
  {
    const snn_status rs = pipe.flush();
    if (rs != SNN_OK) return rs;
  }
  for (int l = 0; l < L; ++l) {
    HIPCHK(c, launch_finish_grad(c->acc_in[l], nullptr, c->dW_in[l], (size_t)pre_of(n, l) * n.N[l], s));
    if (dw_rec_csr(c, l)) HIPCHK(c, launch_finish_grad_csr(c->acc_csr[l], n.csr_sub[l], n.csr_col[l], n.N[l], c->dW_rec[l], s));
    else HIPCHK(c, launch_finish_grad(c->acc_rec[l], c->rec_mask[l], c->dW_rec[l], (size_t)n.N[l] * n.N[l], s));
  }
  HIPCHK(c, launch_finish_grad(c->acc_out, nullptr, c->dW_out, (size_t)n.N[L - 1] * O, s));
  if (remote || R > 0) { // join the copy stream back
    HIPCHK(c, hipEventRecord(ev_join, cs));
    HIPCHK(c, hipStreamWaitEvent(s, ev_join, 0));
  }
  return SNN_OK;
}

snn_status snn_bptt(snn_ctx *c, snn_strategy strategy, int32_t C_in, int32_t F_in, size_t budget, snn_stats *stats) {
  if (!c) return SNN_E_INVAL;
  if (c->T_bound < 1) return fail(c, SNN_E_STATE, "snn_bptt needs inputs bound by snn_forward/snn_bind_inputs");
  const int T = c->T_bound;
  Plan p;
  if (!snn_make_plan((int)strategy, T, C_in, F_in, &p)) return fail(c, SNN_E_INVAL, "invalid strategy/intervals");
  read_kernel_hooks(c);
  NetDev &n = c->net;
  const int L = n.L;
  const size_t Ms = c->Ms();
  const int ring = spike_ring_steps(c->cfg, (int)strategy, T, p.C); // > 0: the hidden spike bitmasks live on the host tier
  // One chunk buffer per layer lets the adjoint pass run its layers one chunk apart (see BwdPipe).  The extra
  // (L - 1) * chunk_len state slots are taken only if the budget has room for them; the results are the same
  // bit for bit either way.
  if (L > 1 && c->bwd_pipeline && strategy != SNN_STANDARD) {
    // one more buffer when the weight gradients of a stage are fused into the next stage's launch, and two
    // more again when the recompute of the next two chunks rides in it as well
    const bool fuse = c->bwd_fuse && !c->dw_event_driven && !c->dw_tile && bwd_stage_fusable(n, dw_wide_tiles(n) ? 1 : 0);
    const int cand[3] = {fuse ? L + 3 : L, fuse ? L + 1 : L, L};
    for (int nb : cand) {
      Plan q = p;
      q.n_chunk_bufs = nb;
      if (!budget || (size_t)q.local_slots() * Ms + work_bytes(n, p.chunk_len) + spike_bytes(n, T, ring) <= budget) { p = q; break; }
    }
  }
  // Double: with room for C more state slots, Re-Forward_1 computes the synaptic currents of its whole coarse
  // segment once and keeps them; the scans of Re-Forward_2 read them instead of computing them again (the two
  // recompute passes of the paper's Double Checkpointing then cost one pass of currents and two of scans).
  // Same values, same order: bit-identical.  Not with the fused stage launches, which recompute ahead on their own.
  if (strategy == SNN_DOUBLE && p.C > p.F && c->rf_cache &&
      !(L > 1 && c->bwd_pipeline && c->bwd_fuse && !c->dw_event_driven && !c->dw_tile && bwd_stage_fusable(n, dw_wide_tiles(n) ? 1 : 0))) {
    Plan q = p;
    q.n_cache_slots = p.C;
    if (!budget || (size_t)q.local_slots() * Ms + work_bytes(n, p.chunk_len) + spike_bytes(n, T, ring) <= budget) p = q;
    // The forward pass computes the same currents (I_t = I_in,t + I_rec,t is a value of its own there too): with
    // the cache in place it leaves those of the last coarse segment(s) in it -- as many whole segments, counted
    // from the end of the sequence, as the budget has room for (without a budget: the last one, which the cache
    // holds anyway) -- and Re-Forward_1 of those segments computes none.  With room for the whole sequence the
    // backward pass recomputes states by scans only.  Layers above 256 neurons only: their sequential kernels
    // write the currents out.
    bool wide_only = true;
    for (int l = 0; l < L; ++l) wide_only = wide_only && n.N[l] > 256;
    if (p.n_cache_slots && c->keep_currents && wide_only) {
      size_t room = (size_t)p.C;
      if (budget) {
        const size_t fixed = (size_t)(p.local_slots() - p.n_cache_slots) * Ms + work_bytes(n, p.chunk_len) + spike_bytes(n, T, ring);
        room = std::min<size_t>((size_t)T, (budget - fixed) / Ms);
      }
      const int keep_from = (int)(((size_t)T - room + (size_t)p.C - 1) / (size_t)p.C) * p.C; // a coarse boundary
      if (keep_from < T) {
        p.keep_from = keep_from;
        p.n_cache_slots = std::max(p.C, T - keep_from);
      }
    }
  }
  const size_t need_states = (size_t)p.local_slots() * Ms;
  const size_t need_work = work_bytes(n, p.chunk_len);
  const size_t need_spikes = spike_bytes(n, T, ring);
  if (budget && need_states + need_work + need_spikes > budget) {
    char buf[200];
    snprintf(buf, sizeof buf, "needs %zu B of HBM activation memory (%d state slots), budget is %zu B",
             need_states + need_work + need_spikes, p.local_slots(), budget);
    return fail(c, SNN_E_BUDGET, buf);
  }
  HIPCHK(c, hipSetDevice(c->cfg.device));
  hipStream_t s = c->stream;
  // ---- storage (before anything is queued or recorded) -----------------------------------------
  if (c->arena_bytes < need_states) {
    HIPCHK(c, hipStreamSynchronize(s));
    if (c->arena) HIPCHK(c, hipFree(c->arena));
    c->arena = nullptr; c->arena_bytes = 0;
    HIPCHK(c, hipMalloc(&c->arena, need_states));
    c->arena_bytes = need_states;
  }
  {
    snn_status rs = ensure_work(c, need_work);
    if (rs != SNN_OK) return rs;
  }
  const size_t need_host = (size_t)p.n_remote * Ms;
  if (c->host_bytes < need_host) {
    HIPCHK(c, hipStreamSynchronize(s));
    if (c->host_ckpt) HIPCHK(c, hipHostFree(c->host_ckpt));
    c->host_ckpt = nullptr; c->host_bytes = 0;
    if (hipHostMalloc(&c->host_ckpt, need_host, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return fail(c, SNN_E_HOSTMEM, "pinned host allocation for remote checkpoints failed");
    }
    c->host_bytes = need_host;
  }
  if (need_host) std::memset(c->host_ckpt, 0, Ms); // host slot 0 = x_0 (nothing is in flight here)
  size_t need_host_spk = 0;
  if (ring > 0) {
    if (c->ring_steps != ring) {
      HIPCHK(c, hipStreamSynchronize(s));
      for (int l = 1; l <= L; ++l) {
        if (c->mask_ring[l]) HIPCHK(c, hipFree(c->mask_ring[l]));
        c->mask_ring[l] = nullptr;
      }
      c->ring_steps = 0;
      for (int l = 1; l <= L; ++l) HIPCHK(c, hipMalloc(&c->mask_ring[l], (size_t)ring * n.B * n.Wd[l] * 8));
      c->ring_steps = ring;
    }
    size_t words = 0;
    for (int l = 1; l <= L; ++l) { c->host_spk_off[l] = words; words += (size_t)(T + 1) * n.B * n.Wd[l]; }
    need_host_spk = words * 8;
    if (c->host_spk_bytes < need_host_spk) {
      HIPCHK(c, hipStreamSynchronize(s));
      if (c->host_spk) HIPCHK(c, hipHostFree(c->host_spk));
      c->host_spk = nullptr; c->host_spk_bytes = 0;
      if (hipHostMalloc(reinterpret_cast<void **>(&c->host_spk), need_host_spk, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        return fail(c, SNN_E_HOSTMEM, "pinned host allocation for the spike bitmasks failed");
      }
      c->host_spk_bytes = need_host_spk;
    }
    c->host_spk_rows = T + 1;
    for (int l = 1; l <= L; ++l) std::memset(c->host_spk + c->host_spk_off[l], 0, (size_t)n.B * n.Wd[l] * 8); // step 0: silent
  } else {
    // the whole sequence in HBM (a spike_tier-1 context allocates its hidden layers' arrays here on first use)
    c->spikes_on_host = false; // the step rewrites the hidden spike trains
    const snn_status rm = ensure_full_masks(c);
    if (rm != SNN_OK) return rm;
  }

  snn_stats st{};
  st.bytes_states = (int64_t)need_states; st.bytes_spikes = (int64_t)need_spikes; st.bytes_workspace = (int64_t)need_work;
  st.bytes_host = (int64_t)need_host; st.local_state_slots = p.local_slots(); st.remote_state_slots = p.n_remote;
  st.bytes_host_spikes = (int64_t)need_host_spk;

  // A step whose launches are recorded once and replayed as a HIP graph: the per-launch host cost
  // (hundreds of small dependent kernels per step) disappears.  Used when no per-kernel timing is
  // requested; the recording is redone whenever the plan or a buffer it refers to changes.
  const bool use_graph = c->graphs_enabled && !stats;
  if (use_graph) {
    unsigned long long pol = 0;
    for (int l = 0; l < L; ++l) pol = pol * 64 + c->net.cur_pol[0][l] * 16 + c->net.cur_pol[1][l] * 2 + c->net.seq_pol[l];
    pol = pol * 2 + (c->dw_tile ? 1u : 0u);
    const unsigned sel = (unsigned)n.sel_currents | (unsigned)n.sel_adjoint << 8 | (unsigned)n.sel_slices << 16 | (unsigned)n.sel_csr << 24 | (unsigned)n.sel_seq << 28 | (unsigned)n.no_fwd_fuse << 30;
    snn_ctx::GraphKeyT key{(int)strategy, T, p.C, p.F, p.n_chunk_bufs, c->arena, c->dubuf, c->host_ckpt, c->dw_event_driven, pol, sel,
                           ring > 0 ? (void *)c->mask_ring[1] : nullptr, ring > 0 ? (void *)c->host_spk : nullptr, (void *)c->mask_full[1], p.n_cache_slots};
    if (!c->graph_exec || !(key == c->graph_key)) {
      if (c->graph_exec) { (void)hipGraphExecDestroy(c->graph_exec); c->graph_exec = nullptr; }
      Timer tm{c, false};
      snn_stats scratch{};
      HIPCHK(c, hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
      snn_status rs = enqueue_step(c, p, scratch, tm, nullptr);
      hipGraph_t graph = nullptr;
      hipError_t e = hipStreamEndCapture(s, &graph);
      if (rs != SNN_OK) { if (graph) (void)hipGraphDestroy(graph); return rs; }
      if (e != hipSuccess) return fail(c, SNN_E_HIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
      e = hipGraphInstantiate(&c->graph_exec, graph, nullptr, nullptr, 0);
      (void)hipGraphDestroy(graph);
      if (e != hipSuccess) { c->graph_exec = nullptr; return fail(c, SNN_E_HIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(e)); }
      c->graph_key = key;
    }
    HIPCHK(c, hipGraphLaunch(c->graph_exec, s));
    if (c->rate_driven || c->dw_rate_driven) {
      snn_status rr = update_current_policy(c, T, nullptr, ring > 0);
      if (rr != SNN_OK) return rr;
    }
    HIPCHK(c, hipStreamSynchronize(s));
    c->T_spikes = T;
    c->spikes_on_host = ring > 0;
    return check_ws_error(c);
  }

  Timer tm{c, stats != nullptr};
  hipEvent_t ev_start = tm.mark(), ev_fwd = nullptr;
  if (!ev_start) return fail(c, SNN_E_HIP, "hipEventCreate failed");
  snn_status rs = enqueue_step(c, p, st, tm, &ev_fwd);
  if (rs != SNN_OK) { (void)hipStreamSynchronize(c->copy_stream); (void)hipStreamSynchronize(s); return rs; }
  hipEvent_t ev_end = tm.mark();
  if (stats || c->rate_driven || c->dw_rate_driven) {
    snn_status rr = update_current_policy(c, T, st.firing_rate, ring > 0);
    if (rr != SNN_OK) return rr;
  }
  HIPCHK(c, hipStreamSynchronize(s));
  if (stats) {
    (void)hipEventElapsedTime(&st.ms_total, ev_start, ev_end);
    (void)hipEventElapsedTime(&st.ms_forward, ev_start, ev_fwd);
    (void)hipEventElapsedTime(&st.ms_backward_total, ev_fwd, ev_end);
    for (const auto &sp : tm.spans) {
      float ms = 0.f;
      if (sp.a && sp.b) (void)hipEventElapsedTime(&ms, sp.a, sp.b);
      switch (sp.kind) {
        case 1: st.ms_recompute += ms; break;
        case 2: st.ms_adjoint += ms; break;
        case 3: st.ms_dw += ms; break;
        case 4: st.ms_fwd_seq += ms; break;
        case 5: st.ms_fwd_currents += ms; break;
        case 7: st.ms_bwd_stage += ms; break;
        case 8: st.ms_fwd_stage += ms; break;
        case 9: st.ms_scan += ms; break;
        default: st.ms_up_gemm += ms; break;
      }
    }
    *stats = st;
  }
  c->T_spikes = T;
  c->spikes_on_host = ring > 0;
  return check_ws_error(c);
}

} // extern "C"
