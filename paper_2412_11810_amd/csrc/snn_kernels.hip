// HIP kernels (gfx950, wave64) for event-driven LIF-SNN forward / recompute passes, the
// surrogate-gradient adjoint recurrence and the weight-gradient accumulation over active spikes.
//
// Arithmetic contract (what makes spike trains reproducible bit for bit, and every storage
// strategy give identical gradients):
//   * the synaptic current of a neuron is two separate fp32 sums that start from 0.0f and add
//     the weight rows of the active presynaptic neurons in ascending index order (input rows,
//     then recurrent rows); they are added together, then to (alpha*v - theta*s_prev);
//   * no fused multiply-add in the forward/recompute path (this file is compiled with
//     -ffp-contract=off; the adjoint pass uses explicit fmaf);
//   * a recompute pass runs the very same code as the forward pass, minus spike generation;
//   * weight gradients are accumulated per element in a fixed order (time descending, batch
//     ascending) that does not depend on where chunk boundaries fall;
//   * no floating-point atomics anywhere.
#include "snn_internal.h"
#include <stdlib.h>
#include <type_traits>
#include <string.h>

#define WAVE 64
#define SNN_SEQ_GROUP 8 // steps whose per-step operands the sequential kernels load ahead in one go
typedef float v16f __attribute__((ext_vector_type(16)));

static __device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }
// Sum of x over the 64 lanes, the same bits in every lane (all lanes must be active): neighbours within quads
// (xor 1, xor 2), the two quads of a half row, the two halves of a row of 16 -- row-local DPP moves, no LDS -- then
// the four row sums as (r0 + r1) + (r2 + r3).
// The same sum with the same bits, valid in lane 63 only: the four row sums meet through two row broadcasts
// ((r1 + r0) in row 1 and (r3 + r2) in row 3, then (r3 + r2) + (r1 + r0) in row 3; additions commute bit for bit)
// instead of four lane reads and three adds.
static __device__ __forceinline__ float wave_sum_lane63(float x) {
  auto dpp = [](float v, auto ctrl, auto rows) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value,
                                                                 decltype(rows)::value, 0xF, false));
  };
  using all = std::integral_constant<int, 0xF>;
  x = x + dpp(x, std::integral_constant<int, 0xB1>{}, all{});  // quad_perm [1, 0, 3, 2]
  x = x + dpp(x, std::integral_constant<int, 0x4E>{}, all{});  // quad_perm [2, 3, 0, 1]
  x = x + dpp(x, std::integral_constant<int, 0x141>{}, all{}); // row_half_mirror
  x = x + dpp(x, std::integral_constant<int, 0x140>{}, all{}); // row_mirror: every lane of a row holds the row's sum
  x = x + dpp(x, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xA>{}); // row_bcast 15 into rows 1, 3
  x = x + dpp(x, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xC>{}); // row_bcast 31 into rows 2, 3
  return x;
}
static __device__ __forceinline__ float wave_sum(float x) {
  auto dpp = [](float v, auto ctrl) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value, 0xF, 0xF, true));
  };
  x = x + dpp(x, std::integral_constant<int, 0xB1>{});  // quad_perm [1, 0, 3, 2]
  x = x + dpp(x, std::integral_constant<int, 0x4E>{});  // quad_perm [2, 3, 0, 1]
  x = x + dpp(x, std::integral_constant<int, 0x141>{}); // row_half_mirror: the other quad of the half row
  x = x + dpp(x, std::integral_constant<int, 0x140>{}); // row_mirror: the other half of the row
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
  return (r0 + r1) + (r2 + r3);
}

static __device__ __forceinline__ uint64_t lanemask_lt() { return (1ull << lane_id()) - 1ull; }
// Row of the stored spike words of layer index li that holds step t: the rows form a ring in time when only a
// window of the sequence is kept in HBM (net.mring[li] rows; the rest lives in host memory), otherwise row t.
static __device__ __forceinline__ size_t mrow_of(const NetDev &net, int li, int t) {
  const int r = net.mring[li];
  return (size_t)(r > 0 ? t % r : t);
}

// acc = fma(x[lane n of the own 16-lane row], w[n], acc) for n = 0..15, one VOP2 instruction each:
// the DPP row broadcast (row_newbcast:n) feeds lane n of every row to all 16 lanes of that row, so a
// register whose lanes hold 16 consecutive operands replaces 16 scalar broadcasts.  The leading
// s_nop covers the wait states a DPP read needs after a VALU write of its source or of EXEC (the
// compiler does not see into the asm).  One accumulator: a strictly sequential chain.
#define DPP_BC(n) " row_newbcast:" #n " row_mask:0xf bank_mask:0xf\n\t"
#define FMAC16_1(acc, x, w, b)                                                                              \
  asm volatile("s_nop 4\n\t"                                                                                \
               "v_fmac_f32_dpp %0, %1, %2" DPP_BC(0) "v_fmac_f32_dpp %0, %1, %3" DPP_BC(1)                  \
               "v_fmac_f32_dpp %0, %1, %4" DPP_BC(2) "v_fmac_f32_dpp %0, %1, %5" DPP_BC(3)                  \
               "v_fmac_f32_dpp %0, %1, %6" DPP_BC(4) "v_fmac_f32_dpp %0, %1, %7" DPP_BC(5)                  \
               "v_fmac_f32_dpp %0, %1, %8" DPP_BC(6) "v_fmac_f32_dpp %0, %1, %9" DPP_BC(7)                  \
               "v_fmac_f32_dpp %0, %1, %10" DPP_BC(8) "v_fmac_f32_dpp %0, %1, %11" DPP_BC(9)                \
               "v_fmac_f32_dpp %0, %1, %12" DPP_BC(10) "v_fmac_f32_dpp %0, %1, %13" DPP_BC(11)              \
               "v_fmac_f32_dpp %0, %1, %14" DPP_BC(12) "v_fmac_f32_dpp %0, %1, %15" DPP_BC(13)              \
               "v_fmac_f32_dpp %0, %1, %16" DPP_BC(14) "v_fmac_f32_dpp %0, %1, %17" DPP_BC(15)              \
               : "+v"(acc)                                                                                  \
               : "v"(x), "v"(w[b + 0]), "v"(w[b + 1]), "v"(w[b + 2]), "v"(w[b + 3]), "v"(w[b + 4]),         \
                 "v"(w[b + 5]), "v"(w[b + 6]), "v"(w[b + 7]), "v"(w[b + 8]), "v"(w[b + 9]), "v"(w[b + 10]), \
                 "v"(w[b + 11]), "v"(w[b + 12]), "v"(w[b + 13]), "v"(w[b + 14]), "v"(w[b + 15]))

// ------------------------------------------------------------------------------------------
// A1 (inputs): byte spikes [T][B][n_in] -> bit words mask0[t+1][b][w] (row 0 = step 0 = zeros)
// One workgroup of one wave per (t, b); the wave ballots 64 channels at a time.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(WAVE) k_pack_inputs(const uint8_t *__restrict__ in, uint64_t *__restrict__ mask0,
                                                      int B, int n_in, int Wd0) {
  const size_t tb = blockIdx.x; // t*B + b, t zero-based
  const uint8_t *row = in + tb * (size_t)n_in;
  uint64_t *dst = mask0 + ((size_t)B + tb) * Wd0; // skip row 0
  for (int w = 0; w < Wd0; ++w) {
    const int j = w * WAVE + lane_id();
    const bool s = j < n_in && row[j] != 0;
    const uint64_t word = __ballot(s);
    if (lane_id() == 0) dst[w] = word;
  }
}

// ------------------------------------------------------------------------------------------
// Forward / recompute: one workgroup per batch element, time loop on the device.
// ------------------------------------------------------------------------------------------
// Synaptic currents of the NPT neurons n0 + k*nt this thread owns: a_in = sum of the rows of Wcat
// selected by lst_in, a_rec = sum of the rows rec_row0 + lst_rec (each in ascending list order,
// starting from 0.0f).  Wcat is [W_in ; W_rec] stacked row-wise, so both sums are one stream of row
// reads.  The wave fetches 64 stream entries with one LDS read (lane i holds entry i) and broadcasts
// them through a scalar register: each row costs a scalar address computation, one coalesced load
// per owned neuron and two selects+adds; 32 loads per thread are in flight before the adds (in
// stream order) consume them.  Slots past the end of the stream read row 0 and add +0.0f, which
// leaves a sum unchanged bit for bit.
template <int NPT>
static __device__ __forceinline__ void gather2(const float *__restrict__ Wcat, int N, uint32_t rec_row0, int n0, int nt,
                                               const uint16_t *lst_in, int cnt_in, const uint16_t *lst_rec,
                                               int cnt_rec, float (&a_in)[NPT], float (&a_rec)[NPT]) {
  constexpr int U = NPT >= 32 ? 1 : 32 / NPT;
  const int ci = __builtin_amdgcn_readfirstlane(cnt_in), cr = __builtin_amdgcn_readfirstlane(cnt_rec);
  const int tot = ci + cr;
  uint32_t off[NPT];
  bool ok[NPT];
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    a_in[k] = 0.0f;
    a_rec[k] = 0.0f;
    const int n = n0 + k * nt;
    ok[k] = n < N;
    off[k] = ok[k] ? (uint32_t)n : 0u; // out-of-range lanes read column 0 and discard it
  }
  for (int e0 = 0; e0 < tot; e0 += WAVE) {
    const int m = tot - e0 < WAVE ? tot - e0 : WAVE;
    const int e = e0 + lane_id();
    uint32_t mine = 0u;
    if (e < tot) mine = e < ci ? (uint32_t)lst_in[e] : rec_row0 + (uint32_t)lst_rec[e - ci];
    for (int q = 0; q < m; q += U) {
      float w[U][NPT];
#pragma unroll
      for (int r = 0; r < U; ++r) {
        const uint32_t j = __builtin_amdgcn_readlane(mine, (q + r) & (WAVE - 1));
        const float *row = Wcat + (size_t)j * (uint32_t)N;
#pragma unroll
        for (int k = 0; k < NPT; ++k) w[r][k] = row[off[k]];
      }
#pragma unroll
      for (int r = 0; r < U; ++r) {
        const int pos = e0 + q + r;
        const bool is_in = pos < ci, is_rec = pos >= ci && pos < tot;
#pragma unroll
        for (int k = 0; k < NPT; ++k) {
          a_in[k] = a_in[k] + (is_in ? w[r][k] : 0.0f);
          a_rec[k] = a_rec[k] + (is_rec ? w[r][k] : 0.0f);
        }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    a_in[k] = ok[k] ? a_in[k] : 0.0f;
    a_rec[k] = ok[k] ? a_rec[k] : 0.0f;
  }
}

// Turns the bit words of one spike row into the ascending list of active indices (A1, second half).  Every
// wavefront takes a contiguous block of words: the number of spikes before the block is one lane-parallel
// popcount sum, inside the block a running count; the rank of the own bit inside its word gives the position.
// (A wavefront summing the popcounts of all earlier words for each of its words costs Wd^2 / 2 LDS reads per
// step: at 128 words that was half of the time of a step of the sequential forward kernels.)
template <typename Emit, typename Finish>
static __device__ __forceinline__ void expand_words(const uint64_t *words, int Wd, int tid, int nt, Emit emit, Finish finish) {
  const int lane = lane_id(), wave = tid >> 6, nw = nt >> 6;
  const int per = (Wd + nw - 1) / nw;
  const int wb = wave * per, we = wb + per < Wd ? wb + per : Wd;
  if (wb >= Wd) return;
  int pre = 0;
  for (int q = lane; q < wb; q += WAVE) pre += __popcll(words[q]);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) pre += __shfl_xor(pre, o, WAVE);
  for (int widx = wb; widx < we; ++widx) {
    const uint64_t word = words[widx];
    if ((word >> lane) & 1ull) emit(pre + __popcll(word & lanemask_lt()), widx * WAVE + lane);
    pre += __popcll(word);
  }
  if (we == Wd) finish(pre); // the wavefront that holds the last word knows the total
}
static __device__ __forceinline__ void expand_all(const uint64_t *words, int Wd, uint16_t *list, int *cnt, int tid,
                                                  int nt) {
  expand_words(words, Wd, tid, nt, [&](int pos, int idx) { list[pos] = (uint16_t)idx; },
               [&](int total) { if (lane_id() == 0) *cnt = total; });
}

// The same expansion for the sequential kernels of wide layers: entry = byte offset of the weight row (index * n4),
// so that a row load needs no address arithmetic beyond one add, and four entries past the end that point at row 0
// (a wavefront reads entries four at a time).
static __device__ __forceinline__ void expand_offsets(const uint64_t *words, int Wd, uint32_t *offs, int *cnt, int tid,
                                                      int nt, uint32_t n4) {
  expand_words(words, Wd, tid, nt, [&](int pos, int idx) { offs[pos] = (uint32_t)idx * n4; },
               [&](int total) {
                 if (lane_id() == 0) *cnt = total;
                 if (lane_id() < 4) offs[total + lane_id()] = 0u;
               });
}

// Sum of the weight rows offs[0..cnt) (ascending, from 0.0f) for the NPT columns of this thread (byte offsets
// coff[k] inside a row).  Entries come from LDS four at a time (every lane the same address), the row segment
// through a buffer load with a per-lane offset: per row one add, one load per owned neuron and one add per owned
// neuron -- nothing passes through scalar registers.  U rows are in flight before their adds; only the last
// group of four needs a select for the entries past the end.
template <int NPT>
static __device__ __forceinline__ void gather1(__amdgpu_buffer_rsrc_t wres, const uint32_t (&coff)[NPT],
                                               const uint32_t *offs, int cnt_in, float (&acc)[NPT]) {
  // rows per chunk, a multiple of 4: 64 loads in flight (128 measured slower on the widest layers)
  constexpr int U = NPT >= 16 ? 4 : (64 / NPT > 32 ? 32 : 64 / NPT);
  constexpr int G = U / 4;
  const int cnt = __builtin_amdgcn_readfirstlane(cnt_in);
#pragma unroll
  for (int k = 0; k < NPT; ++k) acc[k] = 0.0f;
  const uint4 *offs4 = reinterpret_cast<const uint4 *>(offs);
  int q = 0;
  // whole chunks: straight-line code -- all entries of the chunk in one batch of LDS reads (one wait, not one per
  // four rows), all loads issued, and the adds start when the first row arrives while the rest is still in flight
  // (the number of loads after it is known at compile time).  (A second register set that keeps the next chunk's
  // loads in flight during the adds was measured: no gain at one and two neurons per thread, a loss from four.)
  for (; q + U <= cnt; q += U) {
    uint4 e[G];
#pragma unroll
    for (int g = 0; g < G; ++g) e[g] = offs4[(q >> 2) + g];
    float w[U][NPT];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const uint32_t ev[4] = {e[g].x, e[g].y, e[g].z, e[g].w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < NPT; ++k)
          w[4 * g + i][k] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wres, ev[i] + coff[k], 0, 0));
    }
#pragma unroll
    for (int r = 0; r < U; ++r)
#pragma unroll
      for (int k = 0; k < NPT; ++k) acc[k] = acc[k] + w[r][k];
  }
  // the last, partial chunk: groups of four behind uniform guards, a select for the entries past the end
  if (q < cnt) {
    float w[U][NPT];
#pragma unroll
    for (int r0 = 0; r0 < U; r0 += 4) {
      if (q + r0 >= cnt) continue; // uniform
      const uint4 e = offs4[(q + r0) >> 2];
      const uint32_t ev[4] = {e.x, e.y, e.z, e.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < NPT; ++k)
          w[r0 + i][k] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wres, ev[i] + coff[k], 0, 0));
    }
#pragma unroll
    for (int r0 = 0; r0 < U; r0 += 4) {
      if (q + r0 >= cnt) continue; // uniform
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < NPT; ++k) acc[k] = acc[k] + (q + r0 + i < cnt ? w[r0 + i][k] : 0.0f);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Forward pass.  The time axis is cut into tiles; inside a tile the layers run one after the other:
//   1. k_currents (mode 1): feed-forward currents I_in^l of every step of the tile, in parallel -- they
//      depend only on the spikes of the layer below, which are complete for the tile;
//   2. k_layer_seq_*: the only sequential part, one workgroup per batch element looping over the
//      steps of the tile: recurrent current, LIF update, threshold, ballot -> stored spike words;
//   3. after the last layer, k_currents (mode 2) + k_readout_scan for the leaky readout.
// v^l_t = (alpha v^l_{t-1} - theta s^l_{t-1}) + (I_in + I_rec): same operations, same order, as the
// definition, so spike trains match a plain sequential implementation bit for bit.
// ------------------------------------------------------------------------------------------

// Which steps of a tile store their state (StoreSpec), without a division per step: remainder and quotient of
// (t - t_base) by the interval are carried from step to step.
struct StoreCursor {
  int rem, quo;
  bool on;
  __device__ __forceinline__ void init(const StoreSpec &st, int t_first) {
    on = st.base != nullptr;
    rem = quo = 0;
    if (on) {
      const int d = t_first - st.t_base;
      quo = d / st.interval;
      rem = d - quo * st.interval;
    }
  }
  __device__ __forceinline__ int slot(const StoreSpec &st, int t) const { // -1: step t stores nothing
    if (!on || rem != 0 || t > st.t_max) return -1;
    int sl = quo - 1 + st.slot0;
    if (st.slot_mod > 0) sl %= st.slot_mod;
    return sl;
  }
  __device__ __forceinline__ void next(const StoreSpec &st) {
    if (on && ++rem == st.interval) { rem = 0; ++quo; }
  }
};

// Sequential part, layers of up to NW neurons: the recurrent matrix stays in registers (thread i keeps
// column i, W_rec[0..NW)[i]).  The previous step's spike words are shared through LDS; each lane turns
// bits into 0.0f/1.0f (lane L of register g: spike 16g + L%16), a DPP row broadcast feeds spike j to
// every lane and I_rec = fma(s_j, w_j, I_rec) runs over ascending j: fma(1, w, a) = a + w rounded once
// and fma(0, w, a) = a, i.e. exactly the ascending sum over the active neurons.  One instruction per
// presynaptic neuron, no memory traffic in the loop, one barrier per step.
template <int NW>
__device__ __forceinline__ void layer_seq_rs_body(const NetDev &net, const SeqJob &jb, float *__restrict__ state,
                                                  const StoreSpec &st, int b) {
  constexpr int NWD = NW / 64;
  __shared__ uint64_t sw[2][NWD];
  __shared__ float ring[SNN_SEQ_GROUP][NW];
  const int l = jb.l, t0 = jb.t0, t1 = jb.t1;
  const int t_tile = jb.t_tile;
  const float *__restrict__ iin = jb.iin;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, Wd = net.Wd[l + 1];
  const int i = threadIdx.x, lane = lane_id(), wave = i >> 6;
  const bool own = i < N;
  float w[NW];
#pragma unroll
  for (int q = 0; q < NW; ++q) w[q] = (own && q < N) ? net.W_rec[l][(size_t)q * N + i] : 0.0f;
  float v = own ? state[(size_t)b * SN + off + i] : 0.0f;
  uint64_t *mrow = net.mask[l + 1] + (size_t)b * Wd + wave;
  const size_t mstride = (size_t)B * Wd;
  if (i < NWD) sw[0][i] = i < Wd ? net.mask[l + 1][mrow_of(net, l + 1, t0) * mstride + (size_t)b * Wd + i] : 0ull;
  __syncthreads();
  bool sprev = (sw[0][wave] >> lane) & 1ull;
  int cur = 0;
  const float *icol = iin + (size_t)b * N + i;
  const size_t istride = (size_t)B * N;
  // The feed-forward currents of G steps are loaded one group ahead, parked in a thread-private
  // column of an LDS ring when their group starts (the only point that waits for them) and read
  // from there: no step waits on global memory.
  constexpr int G = SNN_SEQ_GROUP;
  float ri[G];
  auto stage_issue = [&](int t_lo) { // steps t_lo + 1 .. t_lo + G (steps past the end re-read the last one)
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const int t = t_lo + 1 + k <= t1 ? t_lo + 1 + k : t1;
      ri[k] = icol[(size_t)(t - 1 - t_tile) * istride];
    }
  };
  // the weights are in registers from here on (otherwise the compiler, which cannot tell their loads
  // from the staged ones, would wait for every outstanding load before each block of FMAs)
  __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
  if (own && t1 > t0) stage_issue(t0);
  StoreCursor sc;
  sc.init(st, t0 + 1);
  for (int tg = t0; tg < t1; tg += G) {
    if (own) {
#pragma unroll
      for (int k = 0; k < G; ++k) ring[k][i] = ri[k];
      if (tg + G < t1) stage_issue(tg + G);
    }
    const int thi = tg + G < t1 ? tg + G : t1;
    for (int t = tg + 1; t <= thi; ++t) {
      const float in_t = own ? ring[t - tg - 1][i] : 0.0f;
      // lane L of sb[g] holds spike 16g + L%16 of the previous step as 0.0f / 1.0f
      // (one bit-field extract from the 32-bit half that holds the 16 spikes, one convert)
      float sb[NW / 16];
      const uint32_t *sw32 = reinterpret_cast<const uint32_t *>(sw[cur]);
#pragma unroll
      for (int g = 0; g < NW / 16; ++g)
        sb[g] = (float)__builtin_amdgcn_ubfe(sw32[g >> 1], (uint32_t)(16 * (g & 1) + (lane & 15)), 1u);
      float acc = 0.0f;
#pragma unroll
      for (int g = 0; g < NW / 16; ++g) FMAC16_1(acc, sb[g], w, 16 * g);
      float a = net.alpha * v;
      if (sprev) a = a - net.theta;
      v = a + (in_t + acc);
      sprev = own && v > net.theta;
      const uint64_t word = __ballot(sprev);
      if (lane == 0) {
        sw[cur ^ 1][wave] = word;
        if (wave < Wd) mrow[mrow_of(net, l + 1, t) * mstride] = word;
      }
      const int sl = sc.slot(st, t);
      if (own && sl >= 0) st.base[(size_t)sl * st.slot_stride + (size_t)b * SN + off + i] = v;
      sc.next(st);
      __syncthreads();
      cur ^= 1;
    }
  }
  if (own) state[(size_t)b * SN + off + i] = v;
}

// blockIdx.y selects the (layer, tile) this workgroup runs: the layers are pipelined, a few tiles apart
template <int NW>
__global__ void __launch_bounds__(256)
k_layer_seq_rs(NetDev net, SeqJobs jobs, float *__restrict__ state, StoreSpec st) {
  layer_seq_rs_body<NW>(net, jobs.j[blockIdx.y], state, st, (int)blockIdx.x);
}

// Sequential part, any layer width: event-driven.  The layer's spikes of the previous step are kept
// as an ascending index list in LDS (ballot words -> popcount prefix -> list) and only the weight
// rows of those neurons are gathered.  NPT neurons per thread; two barriers per step.
template <int NPT>
__global__ void __launch_bounds__(512)
k_layer_seq_gather(NetDev net, SeqJobs jobs, float *__restrict__ state, StoreSpec st) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int l = jobs.j[blockIdx.y].l, t0 = jobs.j[blockIdx.y].t0, t1 = jobs.j[blockIdx.y].t1;
  const int t_tile = jobs.j[blockIdx.y].t_tile;
  const float *__restrict__ iin = jobs.j[blockIdx.y].iin;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, Wd = net.Wd[l + 1];
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x, lane = lane_id();
  uint64_t *words = (uint64_t *)smem;       // [Wd]
  int *cnt = (int *)(words + Wd);           // [1] (+3 pad)
  uint32_t *offs = (uint32_t *)(cnt + 4);   // [N + 4] byte offsets of the active rows
  uint64_t *mbase = net.mask[l + 1] + (size_t)b * Wd;
  const size_t mstride = (size_t)B * Wd;
  const uint32_t n4 = (uint32_t)N * 4u;
  const __amdgpu_buffer_rsrc_t wres =
      __builtin_amdgcn_make_buffer_rsrc((void *)net.W_rec[l], 0, (int)((size_t)N * N * sizeof(float)), 0x00027000);
  uint32_t coff[NPT];
#pragma unroll
  for (int k = 0; k < NPT; ++k) coff[k] = (uint32_t)(tid + k * nt < N ? tid + k * nt : 0) * 4u;
  float v[NPT];
  uint32_t sp = 0;
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    const int n = tid + k * nt, widx = n >> 6;
    v[k] = n < N ? state[(size_t)b * SN + off + n] : 0.0f;
    if (widx < Wd) {
      const uint64_t word = mbase[mrow_of(net, l + 1, t0) * mstride + widx];
      if (lane == 0) words[widx] = word;
      if ((word >> lane) & 1ull) sp |= 1u << k;
    }
  }
  if (tid == 0) *cnt = 0;
  __syncthreads();
  expand_offsets(words, Wd, offs, cnt, tid, nt, n4);
  __syncthreads();
  const size_t istride = (size_t)B * N;
  StoreCursor sc;
  sc.init(st, t0 + 1);
  for (int t = t0 + 1; t <= t1; ++t) {
    const int store_slot = sc.slot(st, t);
    sc.next(st);
    const float *irow = iin + (size_t)(t - 1 - t_tile) * istride + (size_t)b * N;
    float in_t[NPT];
#pragma unroll
    for (int k = 0; k < NPT; ++k) {
      const int n = tid + k * nt;
      in_t[k] = n < N ? irow[n] : 0.0f;
    }
    float a_rec[NPT];
    gather1<NPT>(wres, coff, offs, *cnt, a_rec);
    uint32_t spn = 0;
#pragma unroll
    for (int k = 0; k < NPT; ++k) {
      const int n = tid + k * nt, widx = n >> 6;
      if (widx < Wd) { // uniform per wave
        float a = net.alpha * v[k];
        if ((sp >> k) & 1u) a = a - net.theta;
        const float it = in_t[k] + a_rec[k];
        const float vn = n < N ? a + it : 0.0f;
        v[k] = vn;
        if (st.cur && t > st.cur_from && n < N)
          st.cur[(size_t)(t - st.cur_from - 1) * st.slot_stride + (size_t)b * SN + off + n] = it;
        const uint64_t word = __ballot(n < N && vn > net.theta);
        if ((word >> lane) & 1ull) spn |= 1u << k;
        if (store_slot >= 0 && n < N)
          st.base[(size_t)store_slot * st.slot_stride + (size_t)b * SN + off + n] = vn;
        if (lane == 0) { // the words are only read by the list expansion, after the barrier
          words[widx] = word;
          mbase[mrow_of(net, l + 1, t) * mstride + widx] = word;
        }
      }
    }
    sp = spn;
    __syncthreads(); // every wave is done with the old list
    expand_offsets(words, Wd, offs, cnt, tid, nt, n4);
    __syncthreads();
  }
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    const int n = tid + k * nt;
    if (n < N) state[(size_t)b * SN + off + n] = v[k];
  }
}

// The same sequential part with the neurons of a layer spread over S workgroups per batch element (one workgroup
// per batch element leaves most of the chip idle and is bound by what one compute unit can load: every active
// weight row passes through its L1).  Workgroup (b, sl) owns the columns [sl N/S, (sl+1) N/S) -- whole 64-bit spike
// words -- and gathers its part of the active rows of W_rec; sums per neuron are the same ascending sums.  After
// the threshold it writes its spike words to the stored bitmask and, as two 8-byte entries per word (32 spike bits
// in the low half, the step count of this launch in the high half), to an exchange buffer in uncached device
// memory that is cleared before every launch and double-buffered by the parity of the step.  There is no barrier:
// every workgroup polls the entries of the whole layer until all carry the tag of the step (bounded number of
// polls; a thread that gives up raises *err and from then on nobody waits), then expands them into its own copy of
// the list of active rows.
template <int NPT>
__global__ void __launch_bounds__(512)
k_layer_seq_gather_sl(NetDev net, SeqJobs jobs, float *__restrict__ state, StoreSpec st, int S, uint64_t *xw,
                      unsigned *err, unsigned spin_limit) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int jq = blockIdx.y;
  const int l = jobs.j[jq].l, t0 = jobs.j[jq].t0, t1 = jobs.j[jq].t1, t_tile = jobs.j[jq].t_tile;
  const float *__restrict__ iin = jobs.j[jq].iin;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, Wd = net.Wd[l + 1];
  const int b = (int)blockIdx.x / S, sl = (int)blockIdx.x % S;
  const int tid = threadIdx.x, nt = blockDim.x, lane = lane_id();
  const int Ns = N / S, c0 = sl * Ns, w0 = c0 >> 6; // own columns and their first word
  uint64_t *words = (uint64_t *)smem;       // [Wd]  whole layer
  int *cnt = (int *)(words + Wd);           // [1] (+3 pad)
  uint32_t *offs = (uint32_t *)(cnt + 4);   // [N + 4] byte offsets of the active rows
  uint64_t *mbase = net.mask[l + 1] + (size_t)b * Wd;
  const size_t mstride = (size_t)B * Wd;
  uint64_t *xb = xw + (size_t)(jq * B + b) * 4 * Wd; // [2][2 Wd] tagged half-words
  const uint32_t n4 = (uint32_t)N * 4u;
  // descriptor over the whole matrix, shifted to this slice's first column
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(net.W_rec[l] + c0), 0, (int)(((size_t)N * N - c0) * sizeof(float)), 0x00027000);
  uint32_t coff[NPT];
#pragma unroll
  for (int k = 0; k < NPT; ++k) coff[k] = (uint32_t)(tid + k * nt) * 4u;
  if (tid == 0) *cnt = 0;
  for (int i = tid; i < Wd; i += nt) words[i] = mbase[mrow_of(net, l + 1, t0) * mstride + i];
  __syncthreads();
  float v[NPT];
  uint32_t sp = 0;
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    const int n = c0 + tid + k * nt;
    v[k] = state[(size_t)b * SN + off + n];
    if ((words[n >> 6] >> lane) & 1ull) sp |= 1u << k;
  }
  expand_offsets(words, Wd, offs, cnt, tid, nt, n4);
  __syncthreads();
  const size_t istride = (size_t)B * N;
  uint32_t *words32 = reinterpret_cast<uint32_t *>(words);
  unsigned step = 0;
  bool dead = false;
  StoreCursor sc;
  sc.init(st, t0 + 1);
  for (int t = t0 + 1; t <= t1; ++t, ++step) {
    const int store_slot = sc.slot(st, t);
    sc.next(st);
    const float *irow = iin + (size_t)(t - 1 - t_tile) * istride + (size_t)b * N + c0;
    float in_t[NPT];
#pragma unroll
    for (int k = 0; k < NPT; ++k) in_t[k] = irow[tid + k * nt];
    float a_rec[NPT];
    gather1<NPT>(wres, coff, offs, *cnt, a_rec);
    uint64_t *xdst = xb + (size_t)(step & 1u) * 2 * Wd;
    const uint64_t tag = (uint64_t)(step + 1u) << 32;
    uint32_t spn = 0;
#pragma unroll
    for (int k = 0; k < NPT; ++k) {
      const int nl = tid + k * nt, widx = w0 + (nl >> 6);
      float a = net.alpha * v[k];
      if ((sp >> k) & 1u) a = a - net.theta;
      const float it = in_t[k] + a_rec[k];
      const float vn = a + it;
      v[k] = vn;
      if (st.cur && t > st.cur_from) st.cur[(size_t)(t - st.cur_from - 1) * st.slot_stride + (size_t)b * SN + off + c0 + nl] = it;
      const uint64_t word = __ballot(vn > net.theta);
      if ((word >> lane) & 1ull) spn |= 1u << k;
      if (store_slot >= 0) st.base[(size_t)store_slot * st.slot_stride + (size_t)b * SN + off + c0 + nl] = vn;
      if (lane == 0) mbase[mrow_of(net, l + 1, t) * mstride + widx] = word;
      if (lane < 2)
        __hip_atomic_store(&xdst[2 * widx + lane], tag | (uint64_t)(uint32_t)(word >> (32 * lane)), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    sp = spn;
    // ---- the whole layer's spike words of this step, from all S workgroups of the batch element ------------
    if (spin_limit == 0u && !dead) { // only ever set by a test of this path: give up at once, arrived or not
      __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      dead = true;
    }
    for (int i = tid; i < 2 * Wd; i += nt) {
      uint64_t e;
      unsigned spins = 0;
      for (;;) {
        e = __hip_atomic_load(&xdst[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(e >> 32) == step + 1u || dead) break;
        if (++spins > spin_limit ||
            ((spins & 63u) == 0u && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
          __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          dead = true; // keep going to the end of the tile, never wait again
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
      words32[i] = (uint32_t)e;
    }
    __syncthreads(); // (every wave was done with the old list before the previous barrier)
    expand_offsets(words, Wd, offs, cnt, tid, nt, n4);
    __syncthreads();
  }
#pragma unroll
  for (int k = 0; k < NPT; ++k) state[(size_t)b * SN + off + c0 + tid + k * nt] = v[k];
}

// ------------------------------------------------------------------------------------------
// A2 for masked recurrent matrices: the rows of active presynaptic neurons in compressed form (only the
// synapses that exist).  A wavefront owns SNN_CSR_SUBW postsynaptic neurons and an accumulator for each in LDS.
// It walks the active rows in ascending order; the lanes take the entries of the row that fall into its range
// (their postsynaptic indices are distinct) and add them to the accumulators (LDS read, vector add, LDS write; a
// wavefront's LDS instructions execute in issue order): every accumulator receives the same addends in the same
// ascending order as in the dense-stored walk, which adds +0.0f wherever no synapse exists -- the same bits.  Only
// the owning wavefront ever touches an accumulator.
// ------------------------------------------------------------------------------------------
#ifndef SNN_CSR_AUX
#define SNN_CSR_AUX 0 // cached like any load: the rows of a step are shared between batch elements (non-temporal: 48 -> 63 ms at configuration 4, T = 512)
#endif
#define SNN_CSR_ACCW (SNN_CSR_SUBW + 64) // floats of LDS per wavefront: its accumulators and 64 spare words behind them
template <int U>
struct CsrGroup { // the entries of U consecutive rows that fall into the wavefront's sub-range, one entry per lane
  uint32_t c[U];
  float v[U];
};
typedef __attribute__((address_space(3))) float lds_float;
typedef unsigned int csr_u32x2 __attribute__((ext_vector_type(2)));
// Requests the entries of rows q .. q + U - 1 of a block (positions and counts one row per lane in p0 / nn; q is a
// constant after unrolling).  One 8-byte load per row from the packed copy (NetDev::csr_pk) through one descriptor
// over the whole array: no scalar descriptor arithmetic per row (the compute unit's one scalar unit is what eight
// gathering wavefronts would otherwise queue for).  A lane past the end of the row's part loads its zero-weight
// entry instead (byte offset `zero`), so the consumer needs neither the count nor a change of the execution mask.
// Straight-line code: the loads of three groups stay in flight.
template <int U>
static __device__ __forceinline__ void csr_issue(CsrGroup<U> &g, int q, uint32_t p0, uint32_t nn,
                                                 __amdgpu_buffer_rsrc_t res, uint32_t lane, uint32_t lane8, uint32_t zero) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t p = (uint32_t)__builtin_amdgcn_readlane(p0, q + u), n = (uint32_t)__builtin_amdgcn_readlane(nn, q + u);
    const csr_u32x2 e = __builtin_amdgcn_raw_buffer_load_b64(res, lane < n ? (p << 3) + lane8 : zero, 0, SNN_CSR_AUX);
    g.v[u] = __builtin_bit_cast(float, e.x);
    g.c[u] = e.y;
  }
}
// Read, add, write back with ordinary LDS instructions: the entries of a row have distinct columns, only this
// wavefront touches its accumulators, and its LDS instructions execute in program order, so the next row's read sees
// this row's write.  (LDS float atomics give the same bits but the counters show the wavefronts waiting two thirds of
// their cycles for them.)  accb: LDS byte address of the accumulator of postsynaptic index 0 (the wavefront's
// first accumulator minus 4 c_base).  OVER: some row of the block has more than 64 entries in this sub-range
// (decided once per block).
template <int U, bool OVER>
static __device__ __forceinline__ void csr_consume(const CsrGroup<U> &g, int q, uint32_t p0, uint32_t nn, uint32_t accb,
                                                   const uint64_t *__restrict__ pk, int lane) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    lds_float *a = (lds_float *)(uintptr_t)((g.c[u] << 2) + accb);
    *a = *a + g.v[u];
    if (OVER) {
      const uint32_t p = (uint32_t)__builtin_amdgcn_readlane(p0, q + u), n = (uint32_t)__builtin_amdgcn_readlane(nn, q + u);
      for (uint32_t o = WAVE; o < n; o += WAVE) // a row with more than 64 entries in this range: finish it first
        if (o + lane < n) {
          const uint64_t e = pk[p + o + lane];
          lds_float *x = (lds_float *)(uintptr_t)(((uint32_t)(e >> 32) << 2) + accb);
          *x = *x + __builtin_bit_cast(float, (uint32_t)e);
        }
    }
  }
}
// The walk of one wavefront over the active rows (list, ascending) for sub-range r.  Rows go in blocks of 48: the
// positions of a block's rows are fetched at once (one row per lane) two blocks ahead of their use, and the entries
// of three groups of 16 rows are in flight while a fourth is added -- a continuous pipeline over the whole list, so
// the wavefront waits for memory once per step and not once per block.  acc_w: SNN_CSR_ACCW floats of LDS.
static __device__ __forceinline__ void csr_gather_wave(const uint16_t *list, int cnt, const uint32_t *__restrict__ sub,
                                                       int nsub1, int r, const uint64_t *__restrict__ pk, uint32_t nnz,
                                                       float *acc_w, int lane) {
  constexpr int U = 16, BL = 3 * U;
  const __amdgpu_buffer_rsrc_t res = __builtin_amdgcn_make_buffer_rsrc(
      (void *)pk, 0, (int)((nnz + (uint32_t)(nsub1 - 1) * 64u) * sizeof(uint64_t)), 0x00027000);
  const uint32_t accb = (uint32_t)(uintptr_t)(lds_float *)acc_w - (uint32_t)r * SNN_CSR_SUBW * 4u;
  const uint32_t lane8 = (uint32_t)lane * 8u, zero = (nnz + (uint32_t)r * 64u + (uint32_t)lane) * 8u;
  auto meta = [&](int base, uint32_t &p0, uint32_t &nn) {
    const int i = base + lane;
    p0 = 0u;
    nn = 0u;
    if (lane < BL && i < cnt) {
      const uint32_t *sp = sub + (size_t)list[i] * nsub1 + r;
      p0 = sp[0];
      nn = sp[1] - p0;
    }
  };
  if (cnt <= 0) return;
  uint32_t p0, nn, p1, n1;
  CsrGroup<U> ga, gb, gc;
  meta(0, p0, nn);
  meta(BL, p1, n1);
  __builtin_amdgcn_sched_barrier(0); // (group by group: the byte offsets of one group at a time in registers)
  csr_issue<U>(ga, 0, p0, nn, res, lane, lane8, zero);
  __builtin_amdgcn_sched_barrier(0);
  csr_issue<U>(gb, U, p0, nn, res, lane, lane8, zero);
  __builtin_amdgcn_sched_barrier(0);
  csr_issue<U>(gc, 2 * U, p0, nn, res, lane, lane8, zero);
  __builtin_amdgcn_sched_barrier(0);
  for (int base = 0; base < cnt; base += BL) {
    const int nr = cnt - base; // rows of this block (>= 1); those past the list's end carry zero entries only
    const bool over = __ballot(nn > (uint32_t)WAVE) != 0ull;
    uint32_t p2, n2;
    meta(base + 2 * BL, p2, n2);
    // The next block's groups are requested as this one's are added -- unconditionally (past the list's end every
    // lane loads its zero entry), so the three register sets have one definition per iteration.
    __builtin_amdgcn_sched_barrier(0); // keep the order: loads of later groups ahead of the adds of earlier ones
    if (over) csr_consume<U, true>(ga, 0, p0, nn, accb, pk, lane);
    else csr_consume<U, false>(ga, 0, p0, nn, accb, pk, lane);
    __builtin_amdgcn_sched_barrier(0);
    csr_issue<U>(ga, 0, p1, n1, res, lane, lane8, zero);
    __builtin_amdgcn_sched_barrier(0);
    if (nr > U) {
      if (over) csr_consume<U, true>(gb, U, p0, nn, accb, pk, lane);
      else csr_consume<U, false>(gb, U, p0, nn, accb, pk, lane);
    }
    __builtin_amdgcn_sched_barrier(0);
    csr_issue<U>(gb, U, p1, n1, res, lane, lane8, zero);
    __builtin_amdgcn_sched_barrier(0);
    if (nr > 2 * U) {
      if (over) csr_consume<U, true>(gc, 2 * U, p0, nn, accb, pk, lane);
      else csr_consume<U, false>(gc, 2 * U, p0, nn, accb, pk, lane);
    }
    __builtin_amdgcn_sched_barrier(0);
    csr_issue<U>(gc, 2 * U, p1, n1, res, lane, lane8, zero);
    __builtin_amdgcn_sched_barrier(0);
    p0 = p1; nn = n1;
    p1 = p2; n1 = n2;
  }
}

// The sliced sequential part for a layer whose recurrent matrix has compressed rows (widths that are multiples
// of 4 SNN_CSR_SUBW).  Workgroup (b, sl) owns 4 SNN_CSR_SUBW columns, wavefront w the sub-range 4 sl + w: it
// walks the compressed rows of the neurons that fired in the previous step (csr_gather_wave, accumulators in LDS,
// cleared by their owner at the start of the step) and moves 1/10 of the bytes of the dense-stored walk when
// 90 % of the synapses do not exist.  Thread (w, lane) then owns the columns 64 k + lane of its wavefront's
// sub-range for the LIF update, so a ballot is a whole spike word.  Exchange of the spike words between the
// workgroups of a batch element, polling and time-out exactly as in k_layer_seq_gather_sl.
static __device__ __forceinline__ void layer_seq_csr_sl_body(const NetDev &net, const SeqJobs &jobs, float *__restrict__ state,
                                                             const StoreSpec &st, int S, uint64_t *xw, unsigned *err,
                                                             unsigned spin_limit, unsigned char *smem, int bx, int jq) {
  constexpr int NPT = SNN_CSR_SUBW / WAVE, NS = 4 * SNN_CSR_SUBW;
  const int l = jobs.j[jq].l, t0 = jobs.j[jq].t0, t1 = jobs.j[jq].t1, t_tile = jobs.j[jq].t_tile;
  const float *__restrict__ iin = jobs.j[jq].iin;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, Wd = net.Wd[l + 1];
  const int b = bx / S, sl = bx % S;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c0 = sl * NS + wave * SNN_CSR_SUBW, w0 = c0 >> 6; // own wavefront's first column and its spike word
  const int nsub1 = N / SNN_CSR_SUBW + 1, r = sl * 4 + wave;
  uint64_t *words = (uint64_t *)smem;                    // [Wd]  whole layer
  int *cnt = (int *)(words + Wd);                        // [1] (+3 pad)
  float *acc = (float *)(cnt + 4);                       // [4][SNN_CSR_ACCW]
  uint16_t *list = (uint16_t *)(acc + 4 * SNN_CSR_ACCW); // [N rounded up to 8] indices of the active rows, ascending
  float *acc_w = acc + wave * SNN_CSR_ACCW;
  uint64_t *mbase = net.mask[l + 1] + (size_t)b * Wd;
  const size_t mstride = (size_t)B * Wd;
  uint64_t *xb = xw + (size_t)(jq * B + b) * 4 * Wd; // [2][2 Wd] tagged half-words
  const uint32_t *__restrict__ sub = net.csr_sub[l];
  if (tid == 0) *cnt = 0;
  for (int i = tid; i < Wd; i += 256) words[i] = mbase[mrow_of(net, l + 1, t0) * mstride + i];
  __syncthreads();
  float v[NPT];
  uint32_t sp = 0;
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    v[k] = state[(size_t)b * SN + off + c0 + 64 * k + lane];
    if ((words[w0 + k] >> lane) & 1ull) sp |= 1u << k;
  }
  expand_all(words, Wd, list, cnt, tid, 256);
  __syncthreads();
  const size_t istride = (size_t)B * N;
  uint32_t *words32 = reinterpret_cast<uint32_t *>(words);
  unsigned step = 0;
  bool dead = false;
  StoreCursor sc;
  sc.init(st, t0 + 1);
  for (int t = t0 + 1; t <= t1; ++t, ++step) {
    const int store_slot = sc.slot(st, t);
    sc.next(st);
    const float *irow = iin + (size_t)(t - 1 - t_tile) * istride + (size_t)b * N + c0;
    float in_t[NPT];
#pragma unroll
    for (int k = 0; k < NPT; ++k) {
      in_t[k] = irow[64 * k + lane];
      acc_w[64 * k + lane] = 0.0f;
    }
    csr_gather_wave(list, *cnt, sub, nsub1, r, net.csr_pk[l], net.csr_nnz[l], acc_w, lane);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup"); // the adds of this wavefront have landed before it reads the sums
    uint64_t *xdst = xb + (size_t)(step & 1u) * 2 * Wd;
    const uint64_t tag = (uint64_t)(step + 1u) << 32;
    uint32_t spn = 0;
#pragma unroll
    for (int k = 0; k < NPT; ++k) {
      const int widx = w0 + k;
      const float a_rec = acc_w[64 * k + lane];
      float a = net.alpha * v[k];
      if ((sp >> k) & 1u) a = a - net.theta;
      const float it = in_t[k] + a_rec;
      const float vn = a + it;
      v[k] = vn;
      if (st.cur && t > st.cur_from) st.cur[(size_t)(t - st.cur_from - 1) * st.slot_stride + (size_t)b * SN + off + c0 + 64 * k + lane] = it;
      const uint64_t word = __ballot(vn > net.theta);
      if ((word >> lane) & 1ull) spn |= 1u << k;
      if (store_slot >= 0) st.base[(size_t)store_slot * st.slot_stride + (size_t)b * SN + off + c0 + 64 * k + lane] = vn;
      if (lane == 0) mbase[mrow_of(net, l + 1, t) * mstride + widx] = word;
      if (lane < 2)
        __hip_atomic_store(&xdst[2 * widx + lane], tag | (uint64_t)(uint32_t)(word >> (32 * lane)), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    sp = spn;
    // ---- the whole layer's spike words of this step, from all S workgroups of the batch element ------------
    if (spin_limit == 0u && !dead) { // only ever set by a test of this path: give up at once, arrived or not
      __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      dead = true;
    }
    __syncthreads(); // every wavefront is done with the list of the previous step (words32 aliases nothing it reads)
    for (int i = tid; i < 2 * Wd; i += 256) {
      uint64_t e;
      unsigned spins = 0;
      for (;;) {
        e = __hip_atomic_load(&xdst[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(e >> 32) == step + 1u || dead) break;
        if (++spins > spin_limit ||
            ((spins & 63u) == 0u && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
          __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          dead = true; // keep going to the end of the tile, never wait again
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
      words32[i] = (uint32_t)e;
    }
    __syncthreads();
    expand_all(words, Wd, list, cnt, tid, 256);
    __syncthreads();
  }
#pragma unroll
  for (int k = 0; k < NPT; ++k) state[(size_t)b * SN + off + c0 + 64 * k + lane] = v[k];
}

__global__ void __launch_bounds__(256)
k_layer_seq_csr_sl(NetDev net, SeqJobs jobs, float *__restrict__ state, StoreSpec st, int S, uint64_t *xw,
                   unsigned *err, unsigned spin_limit) {
  extern __shared__ __align__(16) unsigned char smem[];
  layer_seq_csr_sl_body(net, jobs, state, st, S, xw, err, spin_limit, smem, (int)blockIdx.x, (int)blockIdx.y);
}

// A4: u_t = beta u_{t-1} + I_out,t ; usum += u_t over the steps of a tile (fp64 state: ubar feeds a
// softmax, which turns an absolute error of ubar into a relative error of the loss gradient).
__device__ __forceinline__ void readout_scan_body(const float *__restrict__ iout, double *__restrict__ readout, int B,
                                                  int O, int nsteps, float beta, int init, int vblock) {
  const int i = vblock * blockDim.x + threadIdx.x;
  if (i >= B * O) return;
  const int b = i / O, o = i % O;
  double u = init ? 0.0 : readout[((size_t)b * 2 + 0) * O + o];
  double us = init ? 0.0 : readout[((size_t)b * 2 + 1) * O + o];
  for (int k = 0; k < nsteps; ++k) {
    u = (double)beta * u + (double)iout[(size_t)k * B * O + i];
    us = us + u;
  }
  readout[((size_t)b * 2 + 0) * O + o] = u;
  readout[((size_t)b * 2 + 1) * O + o] = us;
}

__global__ void __launch_bounds__(256)
k_readout_scan(const float *__restrict__ iout, double *__restrict__ readout, int B, int O, int nsteps, float beta,
               int init) {
  readout_scan_body(iout, readout, B, O, nsteps, beta, init, (int)blockIdx.x);
}

// ------------------------------------------------------------------------------------------
// B1 (recompute), part 1: synaptic currents of a whole chunk, parallel over time.
// A recompute pass reads the stored spikes instead of generating them, so nothing in it depends on
// the threshold: the currents I_t = I_in,t + I_rec,t of every (t, b, layer) of a chunk are
// independent gathers.  One workgroup per (t, b, layer) expands the two stored bit rows into index
// lists and runs the same gather as the forward pass; the result lands in the chunk buffer at the
// slot of x_t.  Part 2 (k_scan) then turns currents into states in place.
// ------------------------------------------------------------------------------------------
template <int NPT>
__global__ void __launch_bounds__(512)
k_currents(NetDev net, CurJobs jobs) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, nt = blockDim.x, B = net.B;
  const CurJob &ca = jobs.j[blockIdx.y];
  if ((int)blockIdx.x >= ca.nsteps * B) return; // jobs of one launch may cover different numbers of steps
  const int t0 = ca.t0, t_base = ca.t_base;
  const int t = t0 + 1 + (int)(blockIdx.x / B), b = (int)(blockIdx.x % B);
  // mode 0: recompute, I_in + I_rec of layer ca.lsel into the state slot of x_t
  // mode 1: forward, feed-forward current I_in of layer ca.lsel into a [step][B][N] tile
  // mode 2: forward, readout current sum of W_out rows of the last layer's spikes, [step][B][O] tile
  // mode 3: recompute of a layer whose recurrent matrix is kept as compressed rows: I_in alone into the state slot
  //         of x_t (k_currents_csr then adds I_rec)
  const int l = ca.lsel;
  int N, P, Wi, Wr;
  const float *W;
  const uint64_t *g_in, *g_rec = nullptr;
  if (ca.mode == 2) {
    N = net.n_out; P = net.N[net.L - 1]; Wi = net.Wd[net.L]; Wr = 0; W = net.W_out;
    g_in = net.mask[net.L] + (mrow_of(net, net.L, t) * B + b) * Wi;
  } else {
    N = net.N[l]; P = l == 0 ? net.n_in : net.N[l - 1]; Wi = net.Wd[l]; Wr = ca.mode == 0 ? net.Wd[l + 1] : 0;
    W = net.W_in[l];
    g_in = net.mask[l] + (mrow_of(net, l, t) * B + b) * Wi;
    g_rec = net.mask[l + 1] + (mrow_of(net, l + 1, t - 1) * B + b) * net.Wd[l + 1];
  }
  uint64_t *w_in = (uint64_t *)smem;       // [Wi]
  uint64_t *w_rec = w_in + Wi;             // [Wr]
  int *cnt = (int *)(w_rec + Wr);          // [2] (+2 pad)
  uint16_t *l_in = (uint16_t *)(cnt + 4);  // [P rounded up to 8]
  uint16_t *l_rec = l_in + ((P + 7) & ~7); // [N]
  for (int i = tid; i < Wi; i += nt) w_in[i] = g_in[i];
  for (int i = tid; i < Wr; i += nt) w_rec[i] = g_rec[i];
  if (tid < 2) cnt[tid] = 0;
  __syncthreads();
  expand_all(w_in, Wi, l_in, &cnt[0], tid, nt);
  expand_all(w_rec, Wr, l_rec, &cnt[1], tid, nt);
  __syncthreads();
  float a_in[NPT], a_rec[NPT];
  gather2<NPT>(W, N, (uint32_t)P, tid, nt, l_in, cnt[0], l_rec, cnt[1], a_in, a_rec);
  float *dst = (ca.mode == 0 || ca.mode == 3)
                   ? ca.out + (size_t)(t - t_base - 1) * ca.slot_stride + (size_t)b * net.SN + net.off[l]
                   : ca.out + ((size_t)(t - t_base - 1) * B + b) * N;
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    const int n = tid + k * nt;
    if (n < N) dst[n] = ca.mode == 0 ? a_in[k] + a_rec[k] : a_in[k];
  }
}

// ------------------------------------------------------------------------------------------
// A2 on the matrix cores: currents of 16 (t, b) rows x 64 postsynaptic neurons per wavefront.
// acc[row][col] = fma(s[row][k], W[k][col], acc[row][col]) for k ascending, one K = 1 MFMA
// (v_mfma_f32_16x16x1, four 16x16 blocks sharing the A column) per presynaptic neuron k.  With
// s in {0, 1} every step is either acc + W[k][col] rounded once or acc unchanged, i.e. the ascending
// sum over the active presynaptic neurons -- bit-identical to the gather (checked on the device for
// normal and denormal operands).  A presynaptic neuron that is silent in all 16 rows is skipped
// altogether (no row load, no MFMA): the 64-bit spike words of the 16 rows are OR-ed and the set bits
// of the union expanded into an index list in LDS, so the kernel degrades gracefully from a dense
// contraction (rates of tens of percent: the union is all ones) to a gather shared by 16 rows
// (rates of a few percent).  One coalesced 256-byte row segment is loaded per MFMA.
//   lane layout (verified on the device): A[i] in lane i (< 16, block 0 broadcast: cbsz = 2);
//   B[col] in lane col; D[4*(lane/16) + (r%4)][16*(r/4) + lane%16] in register r.
// mode 0 (recompute): workgroup = 2 row blocks x {feed-forward, recurrent} part, the two partial
// currents are combined through LDS as I_in + I_rec; mode 1 (forward): 4 row blocks, I_in only;
// mode 2 (readout): like mode 1 with W_out and the last layer's spikes.
// ------------------------------------------------------------------------------------------

// Contraction over the presynaptic neurons ent[0..n_pad) (ascending; n_pad a multiple of U*D).  An entry is
// (row index of the weight matrix) | (spikes of the 16 rows, bit r = row r) << 16; the entries past the real
// ones carry an all-zero row mask, so they multiply a valid row by 0 and add +0: no change.  Everything per
// presynaptic neuron happens in the vector unit, with nothing passed through scalar registers (a lane read
// followed by scalar arithmetic costs a wavefront that is alone on its SIMD several issue slots): entries are
// read from LDS four at a time (every lane the same address), the row offset is one multiply-add per lane,
// the row segment (256 B, coalesced) comes through a buffer load with a per-lane offset, and the lane's spike
// is one bit extract and one convert.  Loads stay D - 1 groups of U ahead of the MFMAs that consume them.
template <int U, int D>
static __device__ __forceinline__ void mfma_stream(const uint32_t *ent, int n_pad, __amdgpu_buffer_rsrc_t wres,
                                                   uint32_t col4, int N, int lane, v16f &acc) {
  static_assert(U % 4 == 0, "entries are fetched four at a time");
  if (n_pad <= 0) return;
  const int ng = n_pad / U;
  const uint32_t bitpos = 16u + (uint32_t)(lane & 15), n4 = (uint32_t)N * 4u;
  float w[D][U], a[D][U];
  auto issue = [&](int g, float (&wv)[U], float (&av)[U]) {
    const int gi = g < ng ? g : ng - 1; // groups past the end: loaded again, never consumed
    const uint4 *e4 = reinterpret_cast<const uint4 *>(ent + (size_t)gi * U);
#pragma unroll
    for (int q = 0; q < U / 4; ++q) {
      const uint4 e = e4[q];
      const uint32_t ev[4] = {e.x, e.y, e.z, e.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t off = (ev[i] & 0xFFFFu) * n4 + col4;
        wv[4 * q + i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wres, off, 0, 0));
        av[4 * q + i] = (float)((ev[i] >> bitpos) & 1u);
      }
    }
  };
#pragma unroll
  for (int s = 0; s < D - 1; ++s) issue(s, w[s], a[s]);
  for (int g = 0; g < ng; g += D) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      __builtin_amdgcn_sched_barrier(0); // keep the groups in program order: loads stay D - 1 groups ahead
      issue(g + j + D - 1, w[(j + D - 1) % D], a[(j + D - 1) % D]);
#pragma unroll
      for (int u = 0; u < U; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x1f32(a[j][u], w[j][u], acc, 2, 0, 0);
    }
  }
}

// ws: 64-bit words per row of the LDS copy of the spike words (odd, > the widest presynaptic layer
// of the launch in words: one extra all-zero word); lcap: entries of a wave's list (a multiple of 32).
template <int NWV> // wavefronts per workgroup (4 or 8)
__device__ __forceinline__ void currents_mfma_body(const NetDev &net, const CurJob &ca, int ws, int lcap, int vblock,
                                                   unsigned char *smem) {
  __shared__ float comb[NWV / 2][16][64];
  constexpr int U = 8, D = 4;
  const bool ro = ca.mode == 2; // readout: W_out rows of the last layer's spikes, n_out columns
  const int B = net.B, l = ro ? net.L - 1 : ca.lsel, N = ro ? net.n_out : net.N[l];
  const int rows = ca.nsteps * B, ncb = (N + 63) >> 6;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;
  const int rb_per_wg = ca.mode == 0 ? NWV / 2 : NWV;
  const int n_rbg = (rows + 16 * rb_per_wg - 1) / (16 * rb_per_wg);
  if (vblock >= n_rbg * ncb) return;
  const int cb = vblock % ncb, rbg = vblock / ncb;
  const int part = ca.mode == 0 ? (wave & 1) : 0; // 0 feed-forward, 1 recurrent
  const int rbi = ca.mode == 0 ? (wave >> 1) : wave;
  const int m0 = (rbg * rb_per_wg + rbi) * 16;
  const int m = m0 + (lane & 15);
  const int pl = (part == 0 && !ro) ? l : l + 1;
  const int Wp = net.Wd[pl];
  const int P = ro ? net.N[l] : part == 0 ? (l == 0 ? net.n_in : net.N[l - 1]) : N;
  const float *W = ro ? net.W_out : part == 0 ? net.W_in[l] : net.W_rec[l];
  const uint64_t *g = nullptr;
  if (m < rows) {
    const int t = ca.t0 + 1 + m / B, b = m % B;
    g = net.mask[pl] + (mrow_of(net, pl, part == 0 ? t : t - 1) * B + b) * Wp;
  }
  uint64_t *words = (uint64_t *)smem + (size_t)wave * 16 * ws;              // [16][ws]
  // per wavefront: lcap 32-bit entries for the stream.  The list of indices as it is built (16 bits each) sits in
  // the upper half of the same array: entry i overwrites list[2i - lcap] and its neighbour, both <= i, i.e.
  // indices the wavefront has already turned into entries (it fills them in ascending order).
  uint32_t *ent = (uint32_t *)((uint64_t *)smem + (size_t)NWV * 16 * ws) + (size_t)wave * lcap;
  uint16_t *list = (uint16_t *)(ent + lcap / 2);
  // spike words of the 16 rows -> LDS (rows past the end are silent), plus one all-zero word per row
  for (int wi = lane >> 4; wi < Wp; wi += 4) words[(lane & 15) * ws + wi] = g ? g[wi] : 0ull;
  if (lane < 16) words[lane * ws + Wp] = 0ull;
  __syncthreads();
  // union of the 16 rows, one word per lane, expanded into the ascending list of its set bits
  int n = 0;
  for (int c0 = 0; c0 < Wp; c0 += 64) {
    const int wi = c0 + lane;
    uint64_t un = 0ull;
    if (wi < Wp) {
#pragma unroll
      for (int r = 0; r < 16; ++r) un |= words[r * ws + wi];
      const int rem = P - wi * 64;
      if (rem < 64) un &= rem <= 0 ? 0ull : (1ull << rem) - 1ull;
    }
    const int nq = Wp - c0 < 64 ? Wp - c0 : 64;
    for (int q = 0; q < nq; ++q) {
      const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)un, q);
      const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(un >> 32), q);
      const uint64_t any = ((uint64_t)hi << 32) | lo;
      if (any == 0ull) continue;
      if ((any >> lane) & 1ull) list[n + __popcll(any & lanemask_lt())] = (uint16_t)((c0 + q) * 64 + lane);
      n += __popcll(any);
    }
  }
  // pad to whole rounds with entries that select the all-zero word
  const int n_pad = n > 0 ? (n + U * D - 1) / (U * D) * (U * D) : 0;
  if (n + lane < n_pad) list[n + lane] = (uint16_t)(Wp * 64 + (lane & 31));
  __syncthreads();
  // stream entries: one lane per list entry gathers the entry's bit from the 16 rows (padding entries select
  // the all-zero word) and clamps the row index into the matrix
  for (int i = lane; i < n_pad; i += 64) {
    const int k = list[i], wi = k >> 6, sh = k & 63;
    uint32_t m = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) m |= (uint32_t)((words[r * ws + wi] >> sh) & 1ull) << r;
    ent[i] = (uint32_t)(k < P ? k : P - 1) | (m << 16);
  }
  __syncthreads();
  const int col = cb * 64 + lane;
  v16f acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  const __amdgpu_buffer_rsrc_t wres =
      __builtin_amdgcn_make_buffer_rsrc((void *)W, 0, (int)((size_t)P * N * sizeof(float)), 0x00027000);
  mfma_stream<U, D>(ent, n_pad, wres, (uint32_t)(col < N ? col : 0) * 4u, N, lane, acc);
  if (ca.mode == 0) {
    if (part == 1) {
#pragma unroll
      for (int r = 0; r < 16; ++r) comb[rbi][r][lane] = acc[r];
    }
    __syncthreads();
    if (part == 1) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = acc[r] + comb[rbi][r][lane];
  }
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int mm = m0 + 4 * (lane >> 4) + rr;
    if (mm >= rows) continue;
    const int t = ca.t0 + 1 + mm / B, b = mm % B;
    float *dst = (ca.mode == 0 || ca.mode == 3)
                     ? ca.out + (size_t)(t - ca.t_base - 1) * ca.slot_stride + (size_t)b * net.SN + net.off[l]
                     : ca.out + ((size_t)(t - ca.t_base - 1) * B + b) * N;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = cb * 64 + 16 * q + (lane & 15);
      if (c < N) dst[c] = acc[4 * q + rr];
    }
  }
}

template <int NWV> // 4 wavefronts per workgroup; 2 when the presynaptic layer is so wide that 4 would not fit the LDS
__global__ void __launch_bounds__(64 * NWV)
k_currents_mfma(NetDev net, CurJobs jobs, int ws, int lcap) {
  extern __shared__ __align__(16) unsigned char smem[];
  currents_mfma_body<NWV>(net, jobs.j[blockIdx.y], ws, lcap, (int)blockIdx.x, smem);
}

// The same contraction for matrices far larger than the L2 (a presynaptic x postsynaptic product of tens of MB):
// what bounds the list version there is the weight traffic, every block of 16 rows streaming its own selection
// of weight rows from memory.  Here a workgroup owns 16 MB (t, b) rows x 256 postsynaptic neurons, wavefront w
// the 64 columns 64 w .. 64 w + 63 of all 16 MB rows: it visits EVERY presynaptic neuron k in ascending order
// (at a few percent activity the union over 64 rows is nearly full anyway), loads the 256-byte segment of weight
// row k once (the four wavefronts of the workgroup read 1 KB contiguous per k) and issues one K = 1 MFMA per block of 16 rows with that
// segment as the B operand, on MB independent accumulators (no dependent-issue stall).  The A operand of block
// mb in lane r is bit k of the spike word of row 16 mb + r as 0.0f or 1.0f.  acc + 0 * w leaves acc as it is, so the
// result is bit-identical to the list version and to a gather.
// mode 0 runs the feed-forward and the recurrent part one after the other in the same wavefront and adds the two
// partial currents as I_in + I_rec.
// The A operands are prepared once per workgroup, not once per matrix operation: for every 64 presynaptic
// neurons the 256 threads turn the spike bits of the 64 rows into 0.0f / 1.0f in LDS (thread (row, quarter): 16
// bits of the row's word, which it reads straight from the stored bitmask one word ahead), and a wavefront reads
// the operands of four consecutive k for a block of 16 rows with one 16-byte LDS read.  (Extracting and converting
// the bit in front of every matrix operation cost 3.2 vector instructions per operation, and the counters showed
// matrix and vector pipes busy 69 % + 27 % of the time: one after the other, not side by side.)
// RC only names the instance: 1 for the launches of a recompute pass (modes 0 and 3), 0 for the forward pass's, so
// that a kernel trace lists the two, whose shapes and durations differ, separately.
#define SNN_DENSE_MB_ 4
#define SNN_DENSE_AP 68 // floats per row of the operand buffer (64 + padding)
template <int MB, int RC> // RC = 0: jobs of the forward pass (modes 1 and 2: one matrix per job)
static __device__ __forceinline__ void currents_dense_body(const NetDev &net, const CurJob &ca, int bx,
                                                           float (*Af)[16 * MB][SNN_DENSE_AP]) {
  static_assert(MB == 4, "the staging step maps 256 threads onto 64 rows x 4 quarters of a word");
  constexpr int RW = 16 * MB; // rows per workgroup
  const bool ro = ca.mode == 2;
  const int B = net.B, l = ro ? net.L - 1 : ca.lsel, N = ro ? net.n_out : net.N[l];
  const int rows = ca.nsteps * B, ncg = (N + 255) >> 8, n_rg = (rows + RW - 1) / RW;
  if (bx >= n_rg * ncg) return;
  const int cg = bx % ncg, rg = bx / ncg;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int m0 = rg * RW, cb0 = cg * 256 + wave * 64, col = cb0 + lane;
  const bool active = cb0 < N; // a wavefront past the last column only helps to prepare the operands
  const int srow = tid >> 2, sq = tid & 3; // staging role: row of the tile, quarter of the word
  const int sm = m0 + srow;
  v16f acc0[MB], acc1[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc0[mb][r] = acc1[mb][r] = 0.0f;
  auto run_part = [&](int part, v16f (&acc)[MB]) {
    const int pl = (part == 0 && !ro) ? l : l + 1;
    const int Wp = net.Wd[pl];
    const int P = ro ? net.N[l] : part == 0 ? (l == 0 ? net.n_in : net.N[l - 1]) : N;
    const float *W = ro ? net.W_out : part == 0 ? net.W_in[l] : net.W_rec[l];
    const int Pw = (P + 63) >> 6;
    // the staging thread's row of spike words (a row past the end of the job: no spikes)
    const uint64_t *wrow = nullptr;
    if (sm < rows) {
      const int t = ca.t0 + 1 + sm / B, b = sm % B;
      wrow = net.mask[pl] + (mrow_of(net, pl, part == 0 ? t : t - 1) * B + b) * Wp;
    }
    auto word_at = [&](int kw) -> uint64_t {
      if (!wrow || kw >= Pw) return 0ull;
      uint64_t v = wrow[kw];
      const int rem = P - kw * 64;
      if (rem < 64) v &= (1ull << rem) - 1ull;
      return v;
    };
    auto stage = [&](int buf, uint64_t word) { // bits 16 sq .. 16 sq + 15 of the row's word -> floats
      const uint32_t h = (uint32_t)(word >> (16 * sq)) & 0xFFFFu;
      float4 *dst = reinterpret_cast<float4 *>(&Af[buf][srow][16 * sq]);
#pragma unroll
      for (int q = 0; q < 4; ++q)
        dst[q] = make_float4((float)((h >> (4 * q)) & 1u), (float)((h >> (4 * q + 1)) & 1u), (float)((h >> (4 * q + 2)) & 1u),
                             (float)((h >> (4 * q + 3)) & 1u));
    };
    const __amdgpu_buffer_rsrc_t wres =
        __builtin_amdgcn_make_buffer_rsrc((void *)W, 0, (int)((size_t)P * N * sizeof(float)), 0x00027000);
    const uint32_t col4 = (uint32_t)(col < N ? col : 0) * 4u, n4 = (uint32_t)N * 4u;
    constexpr int U = 4, D = 4, G = 64 / U; // G groups of U presynaptic neurons per 64-bit spike word
    float w[D][U];
    auto issue = [&](int g, float (&wv)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = g * U + u, kc = k < P ? k : P - 1; // past the end: the last row again, multiplied by 0
        wv[u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wres, col4, (uint32_t)kc * n4, 0));
      }
    };
    if (part) __syncthreads(); // everybody is done with the operand buffers of the first part
    uint64_t wnext = word_at(0);
    stage(0, wnext);
    wnext = word_at(1);
    if (active) {
#pragma unroll
      for (int g = 0; g < D - 1; ++g) issue(g, w[g]);
    }
    for (int kw = 0; kw < Pw; ++kw) {
      const int buf = kw & 1;
      __syncthreads(); // operands of word kw are in place; everybody has left word kw - 1's
      if (kw + 1 < Pw) stage(buf ^ 1, wnext);
      wnext = word_at(kw + 2);
      if (active) {
#pragma unroll
        for (int g8 = 0; g8 < G; ++g8) {
          __builtin_amdgcn_sched_barrier(0); // keep the groups in program order: loads stay D - 1 groups ahead
          issue(kw * G + g8 + D - 1, w[(g8 + D - 1) % D]);
          float4 a4[MB];
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) a4[mb] = *reinterpret_cast<const float4 *>(&Af[buf][16 * mb + (lane & 15)][U * g8]);
#pragma unroll
          for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
              const float a = u == 0 ? a4[mb].x : u == 1 ? a4[mb].y : u == 2 ? a4[mb].z : a4[mb].w;
              acc[mb] = __builtin_amdgcn_mfma_f32_16x16x1f32(a, w[g8 % D][u], acc[mb], 2, 0, 0);
            }
        }
      }
    }
  };
  run_part(0, acc0);
  if (RC && ca.mode == 0) run_part(1, acc1);
  if (!active) return;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    if (RC && ca.mode == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc0[mb][r] = acc0[mb][r] + acc1[mb][r];
    }
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int mm = m0 + 16 * mb + 4 * (lane >> 4) + rr;
      if (mm >= rows) continue;
      const int t = ca.t0 + 1 + mm / B, b = mm % B;
      float *dst = (ca.mode == 0 || ca.mode == 3)
                       ? ca.out + (size_t)(t - ca.t_base - 1) * ca.slot_stride + (size_t)b * net.SN + net.off[l]
                       : ca.out + ((size_t)(t - ca.t_base - 1) * B + b) * N;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = cb0 + 16 * q + (lane & 15);
        if (c < N) dst[c] = acc0[mb][4 * q + rr];
      }
    }
  }
}

template <int MB, int RC>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_currents_dense(NetDev net, CurJobs jobs, int ws) {
  (void)ws;
  __shared__ __align__(16) float Af[2][16 * MB][SNN_DENSE_AP];
  currents_dense_body<MB, RC>(net, jobs.j[blockIdx.y], (int)blockIdx.x, Af);
}

// One stage of the pipelined forward pass of wide layers with compressed recurrent rows in a single launch: the
// first n_seq workgroups run the sequential parts of the stage's tiles (k_layer_seq_csr_sl: a chain of gathers
// that leaves the matrix cores idle and most issue slots empty), the others the dense feed-forward currents that
// the NEXT stage's sequential parts will consume (k_currents_dense; the two are independent).  Three wavefronts
// per SIMD: two of sequential workgroups -- they come first in the grid, so all of them are resident before any
// current workgroup, which their exchange of spike words needs -- and one of the current kernel, which keeps the
// matrix cores as busy with one wavefront per SIMD as with two.
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
k_fwd_stage_csr(NetDev net, SeqJobs sj, float *__restrict__ state, StoreSpec st, int S, uint64_t *xw, unsigned *err,
                unsigned spin_limit, CurJobs cj, int n_seq_x, int cur_gx) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int n_seq = n_seq_x * sj.count;
  if ((int)blockIdx.x < n_seq) {
    __builtin_amdgcn_s_setprio(3); // the chain goes first wherever both have an instruction ready
    layer_seq_csr_sl_body(net, sj, state, st, S, xw, err, spin_limit, smem, (int)blockIdx.x % n_seq_x, (int)blockIdx.x / n_seq_x);
  } else {
    const int i = (int)blockIdx.x - n_seq;
    currents_dense_body<SNN_DENSE_MB_, 0>(net, cj.j[i / cur_gx], i % cur_gx,
                                          reinterpret_cast<float (*)[16 * SNN_DENSE_MB_][SNN_DENSE_AP]>(smem));
  }
}

// Recompute, recurrent part of layers with compressed rows: workgroup = one (t, b) row of the chunk and a span of
// 4 sub-ranges (one per wavefront).  The state slot of x_t holds I_in on entry (a mode-3 job wrote it) and
// I_in + I_rec on return: two separate sums, added once, as everywhere.
__global__ void __launch_bounds__(256) k_currents_csr(NetDev net, CurJobs jobs) {
  extern __shared__ __align__(16) unsigned char smem[];
  const CurJob &ca = jobs.j[blockIdx.y];
  const int B = net.B, l = ca.lsel, N = net.N[l], Wd = net.Wd[l + 1];
  const int nsub = (N + SNN_CSR_SUBW - 1) / SNN_CSR_SUBW, nspan = (nsub + 3) >> 2;
  if ((int)blockIdx.x >= ca.nsteps * B * nspan) return;
  const int span = (int)blockIdx.x % nspan, m = (int)blockIdx.x / nspan;
  const int t = ca.t0 + 1 + m / B, b = m % B;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint64_t *words = (uint64_t *)smem;                 // [Wd]
  int *cnt = (int *)(words + Wd);                     // [1] (+3 pad)
  float *acc = (float *)(cnt + 4);                    // [4][SNN_CSR_ACCW]
  uint16_t *list = (uint16_t *)(acc + 4 * SNN_CSR_ACCW); // [N rounded up to 8]
  const uint64_t *g_rec = net.mask[l + 1] + (mrow_of(net, l + 1, t - 1) * B + b) * Wd;
  for (int i = tid; i < Wd; i += 256) words[i] = g_rec[i];
  for (int i = tid; i < 4 * SNN_CSR_ACCW; i += 256) acc[i] = 0.0f;
  if (tid == 0) *cnt = 0;
  __syncthreads();
  expand_all(words, Wd, list, cnt, tid, 256);
  __syncthreads();
  const int r = span * 4 + wave;
  if (r < nsub)
    csr_gather_wave(list, *cnt, net.csr_sub[l], nsub + 1, r, net.csr_pk[l], net.csr_nnz[l], acc + wave * SNN_CSR_ACCW, lane);
  __syncthreads();
  float *dst = ca.out + (size_t)(t - ca.t_base - 1) * ca.slot_stride + (size_t)b * net.SN + net.off[l];
  for (int i = tid; i < 4 * SNN_CSR_SUBW; i += 256) {
    const int n = span * 4 * SNN_CSR_SUBW + i;
    if (n < N) dst[n] = dst[n] + acc[(i / SNN_CSR_SUBW) * SNN_CSR_ACCW + i % SNN_CSR_SUBW];
  }
}

// One stage of the pipelined forward pass in a single launch: the first n_seq_blocks workgroups run the
// sequential part of every layer's current tile (job = block / B, batch element = block % B), the others
// compute the synaptic currents that the NEXT stage's sequential parts will consume (virtual grid cur_gx x
// jobs) and run the leaky readout over the tile whose readout currents are ready.  The two are independent; the launcher asks for enough LDS that every workgroup gets a compute unit
// of its own, so the current kernels fill the compute units the sequential part leaves idle without
// competing with it for issue slots.
__global__ void __launch_bounds__(256)
k_fwd_stage(NetDev net, SeqJobs sj, float *__restrict__ state, StoreSpec st, CurJobs cj, int ws, int lcap,
            int n_seq_blocks, int cur_gx, RoJob ro, double *__restrict__ readout) {
  extern __shared__ __align__(16) unsigned char smem[];
  int v = (int)blockIdx.x; // every branch below is uniform per workgroup
  if (v < n_seq_blocks) {
    layer_seq_rs_body<256>(net, sj.j[v / net.B], state, st, v % net.B);
    return;
  }
  v -= n_seq_blocks;
  if (v < ro.n) { // leaky readout over the tile whose readout currents the previous stage computed
    readout_scan_body(ro.iout, readout, net.B, net.n_out, ro.nsteps, net.beta, ro.init, v);
    return;
  }
  v -= ro.n;
  currents_mfma_body<4>(net, cj.j[v / cur_gx], ws, lcap, v % cur_gx, smem);
}

// B1, part 2: v_t = (alpha v_{t-1} - theta s_{t-1}) + I_t along a chunk, one thread per (b, neuron).
// buf holds I_t at the slot of x_t on entry; with store_all the states replace the currents in
// place, otherwise only the final state is written (state_out).  Same operations, in the same
// order, as the forward pass, so the recomputed states are bit-identical to the original ones.
// cur_src != NULL: the currents are read from there (slot of step t = t - src_base - 1) instead of from buf, which
// then only receives the states.
__device__ __forceinline__ void scan_body(const NetDev &net, int t0, int t1, const float *__restrict__ state_in,
                                          float *buf, int t_base, size_t slot_stride, int store_all,
                                          float *__restrict__ state_out, int vblock, const float *cur_src = nullptr,
                                          int src_base = 0) {
  const size_t i = (size_t)vblock * blockDim.x + threadIdx.x;
  const int B = net.B, SN = net.SN;
  if (i >= (size_t)B * SN) return;
  const int b = (int)(i / SN), idx = (int)(i % SN);
  int l = 0;
  while (l + 1 < net.L && idx >= net.off[l + 1]) ++l;
  const int n = idx - net.off[l], Wd = net.Wd[l + 1];
  const uint64_t *mcol = net.mask[l + 1] + (size_t)b * Wd + (n >> 6);
  const size_t mstride = (size_t)B * Wd;
  const int sh = n & 63;
  float v = state_in[i];
  float *col = buf + i;
  const float *ccol = cur_src ? cur_src + i - (size_t)(src_base - t_base) * slot_stride : col; // indexed like col
  constexpr int U = 8;
  int t = t0 + 1;
  for (; t + U - 1 <= t1; t += U) {
    float cur[U];
    uint64_t wd[U];
#pragma unroll
    for (int r = 0; r < U; ++r) {
      cur[r] = ccol[(size_t)(t + r - t_base - 1) * slot_stride];
      wd[r] = mcol[mrow_of(net, l + 1, t + r - 1) * mstride];
    }
#pragma unroll
    for (int r = 0; r < U; ++r) {
      float a = net.alpha * v;
      if ((wd[r] >> sh) & 1ull) a = a - net.theta;
      v = a + cur[r];
      if (store_all) col[(size_t)(t + r - t_base - 1) * slot_stride] = v;
    }
  }
  for (; t <= t1; ++t) {
    const float cur = ccol[(size_t)(t - t_base - 1) * slot_stride];
    const uint64_t wd = mcol[mrow_of(net, l + 1, t - 1) * mstride];
    float a = net.alpha * v;
    if ((wd >> sh) & 1ull) a = a - net.theta;
    v = a + cur;
    if (store_all) col[(size_t)(t - t_base - 1) * slot_stride] = v;
  }
  if (state_out) state_out[i] = v;
}

__global__ void __launch_bounds__(256)
k_scan(NetDev net, int t0, int t1, const float *__restrict__ state_in, float *buf, int t_base, size_t slot_stride,
       int store_all, float *__restrict__ state_out, const float *cur_src, int src_base) {
  scan_body(net, t0, t1, state_in, buf, t_base, slot_stride, store_all, state_out, (int)blockIdx.x, cur_src, src_base);
}

// ------------------------------------------------------------------------------------------
// A5: loss and its gradient with respect to every u_t (constant over t).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_loss(const double *__restrict__ readout, const int32_t *__restrict__ labels,
                                              int B, int O, int T, float *__restrict__ ubar, float *__restrict__ g,
                                              float *__restrict__ loss) {
  // The readout state is fp64, and so is everything here: with a confident (saturated) softmax the gradient
  // softmax - onehot of the labelled class is a difference of nearly equal numbers.  It is formed as minus the
  // sum of the other classes' probabilities, which has no cancellation, and rounded to fp32 once.
  extern __shared__ double lossb[]; // [B]
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    const double *us = readout + ((size_t)b * 2 + 1) * O;
    float *ub = ubar + (size_t)b * O;
    double m = -INFINITY;
    for (int o = 0; o < O; ++o) {
      const double x = us[o] / (double)T;
      ub[o] = (float)x;
      m = fmax(m, x);
    }
    double z = 0.0;
    for (int o = 0; o < O; ++o) z = z + exp(us[o] / (double)T - m);
    const int y = labels[b];
    lossb[b] = (m + log(z)) - us[y] / (double)T;
    double others = 0.0;
    for (int o = 0; o < O; ++o)
      if (o != y) others = others + exp(us[o] / (double)T - m) / z;
    const double scale = (double)B * (double)T;
    for (int o = 0; o < O; ++o) {
      const double p = exp(us[o] / (double)T - m) / z;
      g[(size_t)b * O + o] = (float)((o == y ? -others : p) / scale);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int b = 0; b < B; ++b) s = s + lossb[b];
    *loss = (float)(s / (double)B);
  }
}

// ------------------------------------------------------------------------------------------
// B2-B4: adjoint pass over one chunk of time steps, layer by layer (top layer first):
//   du_t   = beta du_{t+1} + g                                             (k_du_scan)
//   up^l_t = (l==L ? W_out du_t : W_in^{l+1} dv^{l+1}_t)                   (k_up_gemm, all t of the chunk at once)
//   ds^l_t = up^l_t + W_rec^l dv^l_{t+1} - theta dv^l_{t+1}                (k_adj_rec_*: the only sequential part)
//   dv^l_t = alpha dv^l_{t+1} + ds^l_t / (1 + k |v^l_t - theta|)^2
// dv^l_t needs dv^{l+1}_t of the same step and dv^l_{t+1}; running a whole chunk of layer l+1 before
// layer l keeps both available and turns the inter-layer product into one dense GEMM per chunk that
// fills the chip, leaving only the recurrent product in the per-batch-element time loop.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void du_scan_body(const float *__restrict__ g, float *__restrict__ carry,
                                             float *__restrict__ dubuf, int B, int O, int SN, int t0, int t1,
                                             int t_base, float beta, int carry_init, int vblock) {
  const int i = vblock * blockDim.x + threadIdx.x;
  if (i >= B * O) return;
  const int b = i / O, o = i % O;
  float *cb = carry + (size_t)b * (SN + O) + SN + o;
  float d = carry_init ? 0.0f : *cb;
  const float gg = g[i];
  for (int t = t1; t > t0; --t) {
    d = beta * d + gg;
    dubuf[((size_t)(t - t_base - 1) * B + b) * O + o] = d;
  }
  *cb = d;
}

__global__ void __launch_bounds__(256)
k_du_scan(const float *__restrict__ g, float *__restrict__ carry, float *__restrict__ dubuf, int B, int O, int SN,
          int t0, int t1, int t_base, float beta, int carry_init) {
  du_scan_body(g, carry, dubuf, B, O, SN, t0, t1, t_base, beta, carry_init, (int)blockIdx.x);
}

// C[m][j] = sum_k A[m*lda + k] * W[j*K + k]   (m < M rows = (slot, b) pairs, j < N)
// fp32 matrix cores (v_mfma_f32_32x32x2): a workgroup of WM x WN wavefronts owns a (32 WM) x (32 WN)
// tile of C, each wavefront a 32 x 32 block.  K runs in tiles of 32 through LDS; the next tile's
// global loads are in flight while the current one is multiplied.  The order of the additions per
// element (k ascending in pairs) is fixed and independent of M, i.e. of how time is cut into chunks.
//   lane layout (verified on the device): A[i][k] in lane i + 32k, B[k][j] in lane j + 32k,
//   D[8*(r/4) + 4*(lane/32) + r%4][lane%32] in register r.
template <int WM, int WN, int BM = 1, int BN = 1>
__device__ __forceinline__ void up_gemm_body(const float *__restrict__ A, int lda, const float *__restrict__ W, int K,
                                             int N, float *__restrict__ C, int ldc, int M, int bx, int by) {
  // (BM x BN blocks of 32 x 32 per wavefront: every LDS value read feeds BN or BM matrix instructions, and a
  // tile of 32 WM BM x 32 WN BN needs proportionally fewer operand bytes from the L2 per flop -- what bounds the
  // 64 x 64 tiles once the matrices are far beyond it.  The operations per element of C are the same.)
  constexpr int NT = 64 * WM * WN, TM = 32 * WM * BM, TN = 32 * WN * BN, KT = 32;
  constexpr int LA = TM * KT / NT, LW = TN * KT / NT;
  __shared__ float As[TM][KT + 1], Ws[TN][KT + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;
  const int m0 = bx * TM, j0 = by * TN;
  v16f acc[BM][BN];
#pragma unroll
  for (int p = 0; p < BM; ++p)
#pragma unroll
    for (int q = 0; q < BN; ++q)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[p][q][r] = 0.0f;
  float ra[LA], rw[LW];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int e = tid + i * NT, r = e / KT, kk = e % KT;
      ra[i] = (m0 + r < M && k0 + kk < K) ? A[(size_t)(m0 + r) * lda + k0 + kk] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < LW; ++i) {
      const int e = tid + i * NT, r = e / KT, kk = e % KT;
      rw[i] = (j0 + r < N && k0 + kk < K) ? W[(size_t)(j0 + r) * K + k0 + kk] : 0.0f;
    }
  };
  gload(0);
  for (int k0 = 0; k0 < K; k0 += KT) {
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const int e = tid + i * NT;
      As[e / KT][e % KT] = ra[i];
    }
#pragma unroll
    for (int i = 0; i < LW; ++i) {
      const int e = tid + i * NT;
      Ws[e / KT][e % KT] = rw[i];
    }
    __syncthreads();
    if (k0 + KT < K) gload(k0 + KT);
#pragma unroll
    for (int kk = 0; kk < KT; kk += 2) {
      float a[BM], b[BN];
#pragma unroll
      for (int p = 0; p < BM; ++p) a[p] = As[(wm * BM + p) * 32 + (lane & 31)][kk + (lane >> 5)];
#pragma unroll
      for (int q = 0; q < BN; ++q) b[q] = Ws[(wn * BN + q) * 32 + (lane & 31)][kk + (lane >> 5)];
#pragma unroll
      for (int p = 0; p < BM; ++p)
#pragma unroll
        for (int q = 0; q < BN; ++q) acc[p][q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[p], b[q], acc[p][q], 0, 0, 0);
    }
    __syncthreads();
  }
#pragma unroll
  for (int p = 0; p < BM; ++p)
#pragma unroll
    for (int q = 0; q < BN; ++q) {
      const int j = j0 + (wn * BN + q) * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + (wm * BM + p) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < M && j < N) C[(size_t)m * ldc + j] = acc[p][q][r];
      }
    }
}

// The same product for small weight matrices (N * K <= 65536, K a multiple of 16, 16-byte aligned rows):
// one wavefront per 16 x 16 block of C, operands straight from memory as float4 (no LDS, no barrier),
// v_mfma_f32_16x16x4.  Lane (i, kk) loads columns k0 + 4kk .. 4kk+3 of row i of its 16 rows; MFMA e of
// a 16-column chunk takes element e of every lane, i.e. columns k0 + 4kk + e -- the same assignment
// for both operands, a fixed order of additions that does not depend on M.  A chunk of time steps is
// only a few thousand rows: blocks this small put a wavefront on every SIMD of the chip, where the
// LDS-tiled kernel would occupy a quarter of them.  Which of the two kernels runs depends on the
// layer shapes only, never on M, so every storage strategy sees the same arithmetic.
//   lane layout (verified on the device): A[i][k] in lane i + 16k, B[k][j] in lane j + 16k,
//   D[4*(lane/16) + r][lane%16] in register r.
typedef float v4f __attribute__((ext_vector_type(4)));
template <int WM, int WN, int BM = 1, int BN = 1>
__global__ void __launch_bounds__(64 * WM * WN)
k_up_gemm(const float *__restrict__ A, int lda, const float *__restrict__ W, int K, int N, float *__restrict__ C,
          int ldc, int M) {
  up_gemm_body<WM, WN, BM, BN>(A, lda, W, K, N, C, ldc, M, (int)blockIdx.x, (int)blockIdx.y);
}
// Matrices from 2048 x 2048: 128 x 128 tiles (a rule on the layer's shape only, like the one for small matrices).
static __host__ __device__ __forceinline__ bool up_gemm_big(int N, int K) { return N >= 2048 && K >= 2048; }

__device__ __forceinline__ void up_gemm16_body(const float *__restrict__ A, int lda, const float *__restrict__ W, int K,
                                               int N, float *__restrict__ C, int ldc, int M, int vblock) {
  const int lane = threadIdx.x & 63, i = lane & 15, kk = lane >> 4;
  const int tiles_n = (N + 15) >> 4;
  const int tile = vblock * 4 + (threadIdx.x >> 6);
  const int m0 = (tile / tiles_n) * 16, j0 = (tile % tiles_n) * 16;
  if (m0 >= M) return;
  const int ra = m0 + i < M ? m0 + i : M - 1, rw = j0 + i < N ? j0 + i : N - 1; // rows past the end: loaded, not stored
  const float4 *pa = reinterpret_cast<const float4 *>(A + (size_t)ra * lda) + kk;
  const float4 *pw = reinterpret_cast<const float4 *>(W + (size_t)rw * K) + kk;
  v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
  const int nch = K >> 4; // chunks of 16 columns
  for (int c0 = 0; c0 < nch; c0 += 8) {
    float4 a[8], b[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int cc = c0 + c < nch ? c0 + c : nch - 1;
      a[c] = pa[cc * 4];
      b[c] = pw[cc * 4];
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      if (c0 + c < nch) {
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[c].x, b[c].x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[c].y, b[c].y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[c].z, b[c].z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[c].w, b[c].w, acc, 0, 0, 0);
      }
    }
  }
  const int j = j0 + i;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int m = m0 + 4 * kk + r;
    if (m < M && j < N) C[(size_t)m * ldc + j] = acc[r];
  }
}

__global__ void __launch_bounds__(256)
k_up_gemm16(const float *__restrict__ A, int lda, const float *__restrict__ W, int K, int N, float *__restrict__ C,
            int ldc, int M) {
  up_gemm16_body(A, lda, W, K, N, C, ldc, M, (int)blockIdx.x);
}

// Surrogate derivative of the threshold at membrane potential v: 1/(1 + k|v - theta|)^2, and 0
// outside the window |v - theta| < win when a window is set (win > 0).
__device__ __forceinline__ float surrogate(const NetDev &net, float v) {
  const float x = fabsf(v - net.theta);
  const float d = 1.0f + net.k * x;
  const float g = 1.0f / (d * d);
  return (net.win > 0.0f && !(x < net.win)) ? 0.0f : g;
}

// Recurrent part, layers of up to H*KH neurons: the recurrent matrix stays in registers for the
// whole chunk.  Thread (jj, h) keeps W_rec[j][h*KH .. h*KH+KH) for the R postsynaptic rows
// j = jj, jj + NJR, ..., jj + (R-1)*NJR (H threads per row, each a slice of the reduction; partial sums
// combined in a fixed order).  dv_{t+1} is broadcast from LDS; every value read feeds R FMAs: the LDS
// traffic that bounds this kernel (every thread re-reading its slice of dv) shrinks by R, while the
// weights per thread stay R*KH.  No weight traffic and no waiting on global memory in the time loop
// (operands staged G steps ahead), two barriers per step.  One workgroup per batch element,
// H*NJR threads.
template <int KH, int H, int R>
__device__ __forceinline__ void adj_rec_rs_body(const NetDev &net, const AdjJob &jb, float *__restrict__ carry, int b) {
  __shared__ __align__(16) float x[2][H * KH];
  __shared__ float part[H][256];
  __shared__ float ring[2 * SNN_SEQ_GROUP][256];
  const int l = jb.l, t0 = jb.t0, t1 = jb.t1, t_base = jb.t_base, carry_init = jb.carry_init;
  float *__restrict__ vbuf = jb.vbuf;
  const float *__restrict__ up = jb.up;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, ldu = N;
  const int NJR = blockDim.x / H, tid = threadIdx.x;
  const int jj = tid % NJR, h = tid / NJR;
  const int j = tid;                 // finalising role: the first R*NJR threads own one row each
  const bool own = tid < R * NJR && j < N;
  float *cb = carry + (size_t)b * (SN + net.n_out) + off;

  float w[R][KH];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int q = 0; q < KH; ++q) {
      const int n = h * KH + q, jr = jj + r * NJR;
      w[r][q] = (jr < N && n < N) ? net.W_recT[l][(size_t)n * N + jr] : 0.0f; // = W_rec[jr][n], coalesced over jj
    }
  for (int i = tid; i < H * KH; i += blockDim.x) {
    x[0][i] = (i < N && !carry_init) ? cb[i] : 0.0f;
    x[1][i] = 0.0f;
  }
  __syncthreads();
  int cur = 0;
  const size_t slot_stride = (size_t)B * SN;
  // Operand staging.  A global load issued in one step and used in the next would put most of a
  // memory round trip into every step.  Instead the v_t and up_t of G steps are loaded into
  // registers one group ahead (stage_issue), parked in a thread-private column of an LDS ring when
  // their group starts (stage_park: the only point that waits for them, G steps after the issue),
  // and read from there step by step.
  constexpr int G = SNN_SEQ_GROUP;
  float rv[G], ru[G];
  auto stage_issue = [&](int t_hi) { // steps t_hi, t_hi - 1, ... (steps past the end re-read the last one)
#pragma unroll
    for (int k = 0; k < G; ++k) {
      const int t = t_hi - k > t0 ? t_hi - k : t0 + 1;
      rv[k] = vbuf[(size_t)(t - t_base - 1) * slot_stride + (size_t)b * SN + off + j];
      ru[k] = up[((size_t)(t - t_base - 1) * B + b) * ldu + j];
    }
  };
  auto stage_park = [&]() {
#pragma unroll
    for (int k = 0; k < G; ++k) {
      ring[2 * k][j] = rv[k];
      ring[2 * k + 1][j] = ru[k];
    }
  };
  if (own) stage_issue(t1);
  for (int tg = t1; tg > t0; tg -= G) {
    if (own) {
      stage_park();
      if (tg - G > t0) stage_issue(tg - G);
    }
    const int tlo = tg - G > t0 ? tg - G : t0;
    for (int t = tg; t > tlo; --t) {
      const float4 *xs = reinterpret_cast<const float4 *>(&x[cur][h * KH]);
      float a[R][4];
#pragma unroll
      for (int r = 0; r < R; ++r) a[r][0] = a[r][1] = a[r][2] = a[r][3] = 0.0f;
#pragma unroll
      for (int q = 0; q < KH / 4; ++q) {
        const float4 xv = xs[q];
#pragma unroll
        for (int r = 0; r < R; ++r) {
          a[r][0] = fmaf(w[r][4 * q + 0], xv.x, a[r][0]);
          a[r][1] = fmaf(w[r][4 * q + 1], xv.y, a[r][1]);
          a[r][2] = fmaf(w[r][4 * q + 2], xv.z, a[r][2]);
          a[r][3] = fmaf(w[r][4 * q + 3], xv.w, a[r][3]);
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r) part[h][jj + r * NJR] = (a[r][0] + a[r][1]) + (a[r][2] + a[r][3]);
      __syncthreads();
      if (own) {
        const float vt = ring[2 * (tg - t)][j], upv = ring[2 * (tg - t) + 1][j];
        float sacc = part[0][j];
#pragma unroll
        for (int q = 1; q < H; ++q) sacc = sacc + part[q][j];
        const float dn = x[cur][j];
        const float ds = (sacc + upv) - net.theta * dn;
        const float dvt = fmaf(ds, surrogate(net, vt), net.alpha * dn);
        x[cur ^ 1][j] = dvt;
        vbuf[(size_t)(t - t_base - 1) * slot_stride + (size_t)b * SN + off + j] = dvt;
      }
      __syncthreads();
      cur ^= 1;
    }
  }
  if (own) cb[j] = x[cur][j];
}

// blockIdx.y selects the job: layers that are one tile apart in the layer pipeline share a launch
template <int KH, int H, int R>
__global__ void __launch_bounds__(512)
k_adj_rec_rs(NetDev net, AdjJobs jobs, float *__restrict__ carry) {
  adj_rec_rs_body<KH, H, R>(net, jobs.j[blockIdx.y], carry, blockIdx.x);
}

// Recurrent part, wide layers (N/8 weights per thread fit in registers, N <= 1024): the recurrent
// matrix is spread over the chip and stays in registers for the whole chunk.  Workgroup (js, bg)
// owns 32 postsynaptic rows x 8 batch elements: thread (jl, kp) keeps W_rec[j][kp*NR .. +NR) and
// forms partial products for the 8 batch elements against dv_{t+1} broadcast from LDS; the 8
// partial sums are combined in a fixed order.  The N/32 workgroups that share a batch group
// exchange their slices of dv_t through a double-buffered array in device memory and a counting
// barrier (one atomic per workgroup and step).  The barrier spins a bounded number of times: if a
// workgroup never arrives the kernel raises *err and every workgroup runs to completion.
template <int NR>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) // one wave per SIMD: the weights must stay in registers
k_adj_rec_ws(NetDev net, AdjJobs jobs, float *__restrict__ carry, float *xg, unsigned *bar, unsigned *err, int G_b,
             unsigned spin_limit, int blocks_per_job, int xg_stride) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_dead; // set by thread 0 when a barrier gave up
  // Several jobs (layers of equal width that are one tile apart in the layer pipeline) share a launch: each
  // has its own range of workgroups, exchange buffer and barrier counters; they never wait for each other.
  const int jq = blockIdx.x / blocks_per_job, vb = blockIdx.x % blocks_per_job;
  const AdjJob &jb = jobs.j[jq];
  const int l = jb.l, t0 = jb.t0, t1 = jb.t1, t_base = jb.t_base, carry_init = jb.carry_init;
  float *__restrict__ vbuf = jb.vbuf;
  const float *__restrict__ up = jb.up;
  xg += (size_t)jq * xg_stride;
  bar += jq * 64;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, O = net.n_out, ldu = N;
  const int tid = threadIdx.x;
  if (tid == 0) s_dead = 0;
  const int bg = vb % G_b, js = vb / G_b, n_slices = blocks_per_job / G_b;
  const int b0 = bg * 8, j0 = js * 32;
  const int NP = NR * 8;                       // padded reduction length (>= N)
  float *xs = (float *)smem;                   // [NP][8]  dv_{t+1}, batch-minor
  float *part = xs + (size_t)NP * 8;           // [8][32][8]
  const int jl = tid & 31, kp = tid >> 5;

  // every load unconditional, from a clamped address, zeroed with an integer mask afterwards: a select
  // lets the compiler put each load under its condition, one memory round trip after the other
  float w[NR];
  {
    const int jc = j0 + jl < N ? j0 + jl : N - 1;
#pragma unroll
    for (int q = 0; q < NR; ++q) {
      const int n = kp * NR + q, nc = n < N ? n : N - 1;
      w[q] = net.W_recT[l][(size_t)nc * N + jc]; // = W_rec[j][n]
    }
#pragma unroll
    for (int q = 0; q < NR; ++q)
      w[q] = __uint_as_float(__float_as_uint(w[q]) & (0u - (uint32_t)(j0 + jl < N && kp * NR + q < N)));
  }
  // dv_{t1+1} of this batch group (loads unconditional and clamped, zeroed afterwards: see above)
  {
    float cv[NR / 4];
#pragma unroll
    for (int r = 0; r < NR / 4; ++r) {
      const int i = tid + 256 * r, n = i >> 3, bb = i & 7;
      cv[r] = carry[(size_t)(b0 + bb < B ? b0 + bb : B - 1) * (SN + O) + off + (n < N ? n : N - 1)];
    }
#pragma unroll
    for (int r = 0; r < NR / 4; ++r) {
      const int i = tid + 256 * r, n = i >> 3, bb = i & 7;
      xs[i] = __uint_as_float(__float_as_uint(cv[r]) & (0u - (uint32_t)(!carry_init && n < N && b0 + bb < B)));
    }
  }
  __syncthreads();
  // finalising role of this thread: row fj, batch element fb
  const int fj = j0 + (tid & 31), fbb = tid >> 5, fb = b0 + fbb;
  const bool fin = fj < N && fb < B;
  const size_t slot_stride = (size_t)B * SN;
  unsigned step = 0;
  bool dead = false;
  for (int t = t1; t > t0; --t, ++step) {
    const size_t slot = (size_t)(t - t_base - 1);
    float vt = 0.0f, upv = 0.0f;
    if (fin) {
      vt = vbuf[slot * slot_stride + (size_t)fb * SN + off + fj];
      upv = up[(slot * B + fb) * ldu + fj];
    }
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.0f;
    const float4 *x4 = reinterpret_cast<const float4 *>(xs + (size_t)kp * NR * 8);
#pragma unroll
    for (int q = 0; q < NR; ++q) {
      const float4 xa = x4[2 * q], xb = x4[2 * q + 1];
      acc[0] = fmaf(w[q], xa.x, acc[0]); acc[1] = fmaf(w[q], xa.y, acc[1]);
      acc[2] = fmaf(w[q], xa.z, acc[2]); acc[3] = fmaf(w[q], xa.w, acc[3]);
      acc[4] = fmaf(w[q], xb.x, acc[4]); acc[5] = fmaf(w[q], xb.y, acc[5]);
      acc[6] = fmaf(w[q], xb.z, acc[6]); acc[7] = fmaf(w[q], xb.w, acc[7]);
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) part[((size_t)kp * 32 + jl) * 8 + c] = acc[c];
    __syncthreads();
    const int par = step & 1;
    if (fin) {
      float sacc = part[((size_t)0 * 32 + (tid & 31)) * 8 + fbb];
#pragma unroll
      for (int k = 1; k < 8; ++k) sacc = sacc + part[((size_t)k * 32 + (tid & 31)) * 8 + fbb];
      const float dn = xs[(size_t)fj * 8 + fbb];
      const float ds = (sacc + upv) - net.theta * dn;
      const float dvt = fmaf(ds, surrogate(net, vt), net.alpha * dn);
      vbuf[slot * slot_stride + (size_t)fb * SN + off + fj] = dvt;
      xg[((size_t)par * B + fb) * N + fj] = dvt;
    }
    // ---- counting barrier over the workgroups of this batch group -------------------------
    // xg and bar live in uncached device memory: stores to them are visible to every other
    // workgroup as soon as they are acknowledged, so each wave waiting for its own stores
    // (s_waitcnt vmcnt(0), written out: a workgroup-scope fence does not emit it) before the
    // workgroup barrier is all the release that is needed -- the arrival below is only counted
    // once every wave of this workgroup has its slice of dv_t in memory.  No L2 write-back or
    // invalidate per step.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
    __syncthreads();
    if (tid == 0 && !dead) {
      __hip_atomic_fetch_add(&bar[bg], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned target = (step + 1u) * (unsigned)n_slices;
      unsigned spins = 0;
      // spin_limit == 0 (only ever set by a test of this path): give up at once, arrived or not
      while (spin_limit == 0u || __hip_atomic_load(&bar[bg], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
        // give up after spin_limit polls, or (looked at now and then: every poll is a memory round
        // trip) when another workgroup already has
        if (++spins > spin_limit ||
            ((spins & 63u) == 0u && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
          __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          s_dead = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
    }
    __syncthreads();
    if (s_dead) dead = true; // keep going to the end of the chunk, never wait again
    // ---- dv_t of the whole layer for this batch group -> LDS --------------------------------
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    {
      // thread -> batch element tid/32, columns (tid%32) + 32*i: all loads issued before the first use
      const int bb = tid >> 5, nb = tid & 31;
      const float *src = xg + ((size_t)par * B + b0 + bb) * N + nb;
      float r[NR / 4];
#pragma unroll
      for (int i = 0; i < NR / 4; ++i) // agent-scope loads: never served from this compute unit's L1
        r[i] = (b0 + bb < B && nb + 32 * i < N)
                   ? __hip_atomic_load(&src[32 * i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                   : 0.0f;
#pragma unroll
      for (int i = 0; i < NR / 4; ++i)
        if (nb + 32 * i < N) xs[(size_t)(nb + 32 * i) * 8 + bb] = r[i];
    }
    __syncthreads();
  }
  // carry out dv_{t0+1}: every workgroup writes its own rows
  if (fin) carry[(size_t)fb * (SN + O) + off + fj] = xs[(size_t)fj * 8 + fbb];
}

// The same chip-wide recurrence on the matrix cores.  Workgroup (js, bg) owns 32 postsynaptic rows x 16 batch
// elements; wavefront q takes a quarter of the reduction range and, for each of the two 16-row blocks, keeps its
// part of W_rec in registers as the A operands of NK K-steps (v_mfma_f32_16x16x4: A[i][k] in lane i + 16k).  The
// B operand of a K-step is dv_{t+1} of 4 presynaptic neurons x 16 batch elements, read from LDS (batch-minor, so
// the 64 lanes read 64 consecutive floats).  Per step a wavefront issues 2 NK MFMAs on two independent
// accumulators and one LDS read per K-step, where the VALU version reads every dv value of 8 batch elements
// once per thread and is bound by the LDS (about twice the time).  The four partial sums are combined in a
// fixed order; exchange and barrier are those of k_adj_rec_ws.
// With NG = 2 a workgroup serves two batch groups of 16 with the same registers of W_rec, half a step apart: while
// the values one group has just stored travel through the exchange buffer, the matrix cores work on the other
// group, and the two round trips of a step no longer add to its products.  Half as many workgroups per layer also
// lets more layers of a pipeline stage share a launch.  The operations per element are those of NG = 1.
// With RH = 2 a workgroup has eight wavefronts and owns 64 rows (wavefront w: rows 32 (w / 4) .., quarter w % 4 of
// the reduction range; two wavefronts per SIMD, 256 registers each): half as many workgroups read a batch group's
// dv_t from the exchange buffer, which is what a step costs.
template <int NK, int NG, int RH> // K-steps per wavefront and row block (padded width 16 NK); batch groups and 32-row halves per workgroup
__global__ void __launch_bounds__(256 * RH) __attribute__((amdgpu_waves_per_eu(RH, RH))) // the weights must stay in registers
k_adj_rec_wsm(NetDev net, AdjJobs jobs, float *__restrict__ carry, float *xg, unsigned *bar, unsigned *err, int G_w,
              unsigned spin_limit, int blocks_per_job, int xg_stride) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int jq = blockIdx.x / blocks_per_job, vb = blockIdx.x % blocks_per_job;
  const AdjJob &jb = jobs.j[jq];
  const int l = jb.l, t0 = jb.t0, t1 = jb.t1, t_base = jb.t_base, carry_init = jb.carry_init;
  float *__restrict__ vbuf = jb.vbuf;
  const float *__restrict__ up = jb.up;
  // exchange entries: dv_t in the low half, the step count (from 1; the buffer is cleared before every launch)
  // in the high half -- a reader polls the values it needs until they all carry the tag of the step
  uint64_t *xq = reinterpret_cast<uint64_t *>(xg + (size_t)jq * xg_stride); // [2][B][N]
  (void)bar;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, O = net.n_out, ldu = N;
  constexpr int NT = 256 * RH;
  const int tid = threadIdx.x, lane = tid & 63, wv = (tid >> 6) & 3, rh = tid >> 8, li = lane & 15, lk = lane >> 4;
  const int bg = vb % G_w, js = vb / G_w; // G_w workgroups of NG batch groups each per 32 RH rows
  const int j0 = js * 32 * RH, jw = j0 + 32 * rh; // first row of the workgroup, of the wavefront
  constexpr int NP = 16 * NK;                          // padded reduction length (>= N)
  float *xs_all = (float *)smem;                       // [NG][NP][16]  dv_{t+1}, batch-minor
  float *part_all = xs_all + (size_t)NG * NP * 16;     // [NG][RH][4][32][16]

  // A operands: a[rb][s] = W_rec[j0 + 16 rb + li][4 NK wv + 4 s + lk].  Every load unconditional, from a clamped
  // address, zeroed with an integer mask afterwards (a select lets the compiler put each load under its condition).
  float a[2][NK];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int j = jw + 16 * rb + li, jc = j < N ? j : N - 1;
#pragma unroll
    for (int q = 0; q < NK; ++q) {
      const int n = 4 * NK * wv + 4 * q + lk, nc = n < N ? n : N - 1;
      a[rb][q] = net.W_recT[l][(size_t)nc * N + jc]; // = W_rec[j][n]
    }
#pragma unroll
    for (int q = 0; q < NK; ++q)
      a[rb][q] = __uint_as_float(__float_as_uint(a[rb][q]) & (0u - (uint32_t)(j < N && 4 * NK * wv + 4 * q + lk < N)));
  }
  // dv_{t1+1} of the batch groups
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int b0 = (bg * NG + g) * 16;
    float cv[NK / RH];
#pragma unroll
    for (int r = 0; r < NK / RH; ++r) {
      const int i = tid + NT * r, n = i >> 4, bb = i & 15;
      cv[r] = carry[(size_t)(b0 + bb < B ? b0 + bb : B - 1) * (SN + O) + off + (n < N ? n : N - 1)];
    }
#pragma unroll
    for (int r = 0; r < NK / RH; ++r) {
      const int i = tid + NT * r, n = i >> 4, bb = i & 15;
      xs_all[(size_t)g * NP * 16 + i] =
          __uint_as_float(__float_as_uint(cv[r]) & (0u - (uint32_t)(!carry_init && n < N && b0 + bb < B)));
    }
  }
  __syncthreads();
  // finalising role: 32 RH x 16 (row, batch element) pairs per group, two per thread
  int fj[2], fbb[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int pidx = tid + NT * e;
    fj[e] = j0 + (pidx >> 4);
    fbb[e] = pidx & 15;
  }
  const size_t slot_stride = (size_t)B * SN;
  bool dead = false;
  // one step of one batch group: products, the sum of the four partial results, the recurrence, the exchange stores
  auto compute = [&](int g, unsigned step, int t) {
    const int b0 = (bg * NG + g) * 16;
    float *xs = xs_all + (size_t)g * NP * 16, *part = part_all + (size_t)g * RH * 4 * 32 * 16;
    const size_t slot = (size_t)(t - t_base - 1);
    float vt[2] = {0.0f, 0.0f}, upv[2] = {0.0f, 0.0f};
#pragma unroll
    for (int e = 0; e < 2; ++e)
      if (fj[e] < N && b0 + fbb[e] < B) {
        vt[e] = vbuf[slot * slot_stride + (size_t)(b0 + fbb[e]) * SN + off + fj[e]];
        upv[e] = up[(slot * B + b0 + fbb[e]) * ldu + fj[e]];
      }
    v4f acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
    const float *xb = xs + (size_t)(4 * NK * wv + lk) * 16 + li;
#pragma unroll
    for (int q = 0; q < NK; ++q) {
      const float x = xb[64 * q];
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0][q], x, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1][q], x, acc1, 0, 0, 0);
    }
    // D[4 lk + r][li]: row 4 lk + r of the block, batch element li
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      part[((size_t)(4 * rh + wv) * 32 + 4 * lk + r) * 16 + li] = acc0[r];
      part[((size_t)(4 * rh + wv) * 32 + 16 + 4 * lk + r) * 16 + li] = acc1[r];
    }
    __syncthreads();
    const int par = step & 1;
#pragma unroll
    for (int e = 0; e < 2; ++e)
      if (fj[e] < N && b0 + fbb[e] < B) {
        const int fr = (fj[e] - j0) & 31, fh = (fj[e] - j0) >> 5, fb = b0 + fbb[e];
        float sacc = part[((size_t)(4 * fh) * 32 + fr) * 16 + fbb[e]];
#pragma unroll
        for (int k = 1; k < 4; ++k) sacc = sacc + part[((size_t)(4 * fh + k) * 32 + fr) * 16 + fbb[e]];
        const float dn = xs[(size_t)fj[e] * 16 + fbb[e]];
        const float ds = (sacc + upv[e]) - net.theta * dn;
        const float dvt = fmaf(ds, surrogate(net, vt[e]), net.alpha * dn);
        vbuf[slot * slot_stride + (size_t)fb * SN + off + fj[e]] = dvt;
        __hip_atomic_store(&xq[((size_t)par * B + fb) * N + fj[e]],
                           ((uint64_t)(step + 1u) << 32) | (uint64_t)__float_as_uint(dvt), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
  };
  // dv_t of the whole layer for one batch group -> LDS.  No barrier: the values themselves say when they have
  // arrived.  One store and one load round trip per step instead of store, wait, atomic, poll, load.  The polling
  // is bounded like the barrier of k_adj_rec_ws: a thread that gives up raises *err, and from then on nobody waits.
  auto poll = [&](int g, unsigned step) {
    const int b0 = (bg * NG + g) * 16, par = step & 1;
    float *xs = xs_all + (size_t)g * NP * 16;
    // thread -> batch element tid / (16 RH), columns tid % (16 RH) + 16 RH i: all loads of a round issued before
    // the first use.  One base address for all of them, the column in the constant offset: entries past the layer's
    // width read whatever follows (the buffer has 16 KB of slack behind its last row) and are neither waited for
    // nor used.
    constexpr int NB = 16 * RH, NE = NK / RH; // lanes along the row, entries per thread
    const int bb = tid / NB, nb = tid % NB;
    const uint64_t *src = xq + ((size_t)par * B + (b0 + bb < B ? b0 + bb : B - 1)) * N + nb;
    const uint32_t want = step + 1u;
    if (spin_limit == 0u && !dead) { // only ever set by a test of this path: give up at once, arrived or not
      __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      dead = true;
    }
    constexpr int CH = RH == 2 ? NE / 2 : (NE < 32 ? NE : 32); // values polled at a time: a round that comes too early is read again
#pragma unroll
    for (int c = 0; c < NE; c += CH) {
      uint64_t r[CH];
      unsigned spins = 0;
      for (;;) {
        uint32_t bad = 0;
#pragma unroll
        for (int i = 0; i < CH; ++i) // agent-scope loads: never served from this compute unit's L1
          r[i] = __hip_atomic_load(&src[NB * (c + i)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int i = 0; i < CH; ++i) bad |= ((uint32_t)(r[i] >> 32) ^ want) & (0u - (uint32_t)(nb + NB * (c + i) < N));
        if (bad == 0u || dead) break;
        if (++spins > spin_limit / 8u ||
            ((spins & 15u) == 0u && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
          __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          dead = true; // keep going to the end of the chunk, never wait again
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        const int n = nb + NB * (c + i);
        xs[(size_t)n * 16 + bb] = __uint_as_float((uint32_t)r[i] & (0u - (uint32_t)(n < N && b0 + bb < B)));
      }
    }
  };
  unsigned step = 0;
  for (int t = t1; t > t0; --t, ++step) {
    compute(0, step, t);
    if (NG == 2) {
      // the second group runs half a step behind: its values of the previous step have had the first group's
      // products to arrive
      if (step > 0u) poll(1, step - 1u);
      __syncthreads();
      compute(1, step, t);
    }
    __syncthreads(); // every thread has read its dv_{t+1} of the first group from LDS
    poll(0, step);
    __syncthreads();
  }
  if (NG == 2) {
    poll(1, step - 1u);
    __syncthreads();
  }
  // carry out dv_{t0+1}: every workgroup writes its own rows
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int b0 = (bg * NG + g) * 16;
#pragma unroll
    for (int e = 0; e < 2; ++e)
      if (fj[e] < N && b0 + fbb[e] < B)
        carry[(size_t)(b0 + fbb[e]) * (SN + O) + off + fj[e]] = xs_all[(size_t)g * NP * 16 + (size_t)fj[e] * 16 + fbb[e]];
  }
}

// The chip-wide recurrence for layers whose recurrent matrix does not fit the registers of the chip (N > 1024,
// N a multiple of 64, batch <= 64).  Per step the whole batch shares ONE pass over W_rec: workgroup js owns
// R = 16 RB postsynaptic rows and every batch element, its four wavefronts each take a quarter of the reduction
// range.  A operand of a K-step group (v_mfma_f32_16x16x4, four K-steps per 16 presynaptic neurons): lane
// (i, k) loads the 16 bytes W_rec[j0 + i][n .. n+4) with n = nb + 16 q + 4 k, so the four lanes of a row read 64
// contiguous bytes and the stream over q walks each row front to back; component s of the load is the A value
// of K-step s.  The B operand needs dv_{t+1}[n + s][b] in the same lane positions: the exchange buffer holds
// dv as [batch block][n / 4][16 batch][4], one 16-byte load per lane and 1 KB contiguous per wavefront.  The
// order of the sum (which neuron meets which K-step) is fixed by this layout and the same in every launch.
// Loads of W_rec run D groups ahead of the MFMAs in a register ring that continues into the next step (the
// matrix is the same), loads of dv start after the step's barrier.  Exchange, counting barrier and its bounded
// spin are those of k_adj_rec_ws with one counter for the whole grid; dv is read with loads that bypass the
// non-coherent cache levels (the exchange buffer is uncached device memory).
template <int RB, int NBB>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
k_adj_rec_wide(NetDev net, AdjJob jb, float *__restrict__ carry, float *xg, unsigned *bar, unsigned *err,
               unsigned spin_limit) {
  constexpr int D = 8, R = 16 * RB, BP = 16 * NBB, ITEMS = (R / 4) * BP, NIT = (ITEMS + 255) / 256;
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_dead;
  float *part = (float *)smem; // [4][R][BP]
  const int l = jb.l, t0 = jb.t0, t1 = jb.t1, t_base = jb.t_base, carry_init = jb.carry_init;
  float *__restrict__ vbuf = jb.vbuf;
  const float *__restrict__ up = jb.up;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, O = net.n_out, ldu = N;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, li = lane & 15, lk = lane >> 4;
  if (tid == 0) s_dead = 0;
  const int j0 = blockIdx.x * R;
  const unsigned n_wg = gridDim.x;
  const int NQ = N / 64, NQp = (NQ + D - 1) / D * D; // K-step groups per wavefront and step; padded to the ring
  const int nb = wv * (N / 4);
  const size_t xpar = (size_t)BP * N; // floats per parity of the exchange buffer
  const __amdgpu_buffer_rsrc_t xres =
      __builtin_amdgcn_make_buffer_rsrc((void *)xg, 0, (int)(2 * xpar * sizeof(float)), 0x00027000);
  const float4 *ap[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
    ap[rb] = reinterpret_cast<const float4 *>(net.W_rec[l] + (size_t)(j0 + 16 * rb + li) * N + nb) + lk;
  // groups past the end of the range (ring padding) load the last group and are zeroed: they add 0 * dv
  auto load_a = [&](int q, float4 (&dst)[RB]) {
    const int qc = q < NQ ? q : NQ - 1;
    const uint32_t m = 0u - (uint32_t)(q < NQ);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float4 v = ap[rb][4 * qc];
      dst[rb].x = __uint_as_float(__float_as_uint(v.x) & m);
      dst[rb].y = __uint_as_float(__float_as_uint(v.y) & m);
      dst[rb].z = __uint_as_float(__float_as_uint(v.z) & m);
      dst[rb].w = __uint_as_float(__float_as_uint(v.w) & m);
    }
  };
  auto load_x = [&](int par, int q, float4 (&dst)[NBB]) {
    const int qc = q < NQ ? q : NQ - 1;
#pragma unroll
    for (int bk = 0; bk < NBB; ++bk) {
      const uint32_t idx = (uint32_t)(((bk * (N / 4) + nb / 4 + 4 * qc + lk) * 16 + li) * 4);
      const uint32_t byte = (uint32_t)(((size_t)par * xpar + idx) * sizeof(float));
      dst[bk] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(xres, byte, 0, 17)); // sc0 sc1
    }
  };
  bool dead = false;
  unsigned arrivals = 0;
  auto grid_barrier = [&]() {
    // see k_adj_rec_ws: every wave waits for its own stores, then one arrival per workgroup
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
    __syncthreads();
    arrivals += n_wg;
    if (tid == 0 && !dead) {
      __hip_atomic_fetch_add(&bar[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      unsigned spins = 0;
      while (spin_limit == 0u || __hip_atomic_load(&bar[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < arrivals) {
        if (++spins > spin_limit ||
            ((spins & 63u) == 0u && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
          __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          s_dead = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
    }
    __syncthreads();
    if (s_dead) dead = true; // keep going to the end of the chunk, never wait again
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  };
  // finalising role: item = 4 consecutive rows x one batch element
  int fj[NIT], fbb[NIT];
  bool fit[NIT], fin[NIT];
  float dprev[NIT][4];
#pragma unroll
  for (int i = 0; i < NIT; ++i) {
    const int it = tid + 256 * i;
    fit[i] = it < ITEMS;
    fj[i] = j0 + 4 * ((it / BP) % (R / 4));
    fbb[i] = it % BP;
    fin[i] = fit[i] && fbb[i] < B;
#pragma unroll
    for (int c = 0; c < 4; ++c)
      dprev[i][c] = (fin[i] && !carry_init) ? carry[(size_t)fbb[i] * (SN + O) + off + fj[i] + c] : 0.0f;
  }
  auto x_slot = [&](int par, int i) { // this item's four values in the exchange buffer
    return xg + (size_t)par * xpar + ((size_t)((fbb[i] >> 4) * (N / 4) + fj[i] / 4) * 16 + (fbb[i] & 15)) * 4;
  };
  // dv_{t1+1} of the own rows into parity 1, which step 0 reads
#pragma unroll
  for (int i = 0; i < NIT; ++i)
    if (fit[i]) *reinterpret_cast<float4 *>(x_slot(1, i)) = make_float4(dprev[i][0], dprev[i][1], dprev[i][2], dprev[i][3]);
  float4 a[D][RB], x[D][NBB];
#pragma unroll
  for (int d = 0; d < D; ++d) load_a(d, a[d]);
  grid_barrier();
  const size_t slot_stride = (size_t)B * SN;
  unsigned step = 0;
  for (int t = t1; t > t0; --t, ++step) {
    const int rd = (int)((step & 1u) ^ 1u);
    const size_t slot = (size_t)(t - t_base - 1);
#pragma unroll
    for (int d = 0; d < D; ++d) load_x(rd, d, x[d]);
    float vt[NIT][4], upv[NIT][4];
#pragma unroll
    for (int i = 0; i < NIT; ++i)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        vt[i][c] = fin[i] ? vbuf[slot * slot_stride + (size_t)fbb[i] * SN + off + fj[i] + c] : 0.0f;
        upv[i][c] = fin[i] ? up[(slot * B + fbb[i]) * ldu + fj[i] + c] : 0.0f;
      }
    v4f acc[RB][NBB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int bk = 0; bk < NBB; ++bk) acc[rb][bk] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    for (int q0 = 0; q0 < NQp; q0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int bk = 0; bk < NBB; ++bk) {
            acc[rb][bk] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[d][rb].x, x[d][bk].x, acc[rb][bk], 0, 0, 0);
            acc[rb][bk] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[d][rb].y, x[d][bk].y, acc[rb][bk], 0, 0, 0);
            acc[rb][bk] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[d][rb].z, x[d][bk].z, acc[rb][bk], 0, 0, 0);
            acc[rb][bk] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[d][rb].w, x[d][bk].w, acc[rb][bk], 0, 0, 0);
          }
        const int qn = q0 + d + D;
        load_x(rd, qn, x[d]);                        // past the end: a repeat of the last group, never used
        load_a(qn >= NQp ? qn - NQp : qn, a[d]);     // past the end: the first groups of the next step
      }
    }
    // D[4 lk + r][li] of block (rb, bk): row 16 rb + 4 lk + r, batch element 16 bk + li
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int bk = 0; bk < NBB; ++bk)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[((size_t)wv * R + 16 * rb + 4 * lk + r) * BP + 16 * bk + li] = acc[rb][bk][r];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NIT; ++i)
      if (fit[i]) {
        float dv[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int fr = fj[i] - j0 + c;
          float sacc = part[((size_t)0 * R + fr) * BP + fbb[i]];
#pragma unroll
          for (int k = 1; k < 4; ++k) sacc = sacc + part[((size_t)k * R + fr) * BP + fbb[i]];
          const float dn = dprev[i][c];
          const float ds = (sacc + upv[i][c]) - net.theta * dn;
          dv[c] = fin[i] ? fmaf(ds, surrogate(net, vt[i][c]), net.alpha * dn) : 0.0f;
          if (fin[i]) vbuf[slot * slot_stride + (size_t)fbb[i] * SN + off + fj[i] + c] = dv[c];
          dprev[i][c] = dv[c];
        }
        *reinterpret_cast<float4 *>(x_slot(rd ^ 1, i)) = make_float4(dv[0], dv[1], dv[2], dv[3]);
      }
    if (t > t0 + 1) grid_barrier(); // nobody reads the exchange buffer after the last step
  }
  // carry out dv_{t0+1}: every workgroup writes its own rows
#pragma unroll
  for (int i = 0; i < NIT; ++i)
    if (fin[i])
#pragma unroll
      for (int c = 0; c < 4; ++c) carry[(size_t)fbb[i] * (SN + O) + off + fj[i] + c] = dprev[i][c];
}

// Recurrent part, any layer width: the transposed recurrent matrix is streamed from L2 every step
// (coalesced over the output index), the reduction split over KG thread groups with a fixed
// combination order.
static __device__ __forceinline__ float dot_T(const float *__restrict__ WT, int ld, int j, const float *x, int n0,
                                              int n1) {
  float a0 = 0.0f, a1 = 0.0f;
  int n = n0;
  for (; n + 8 <= n1; n += 8) {
    float w[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) w[q] = WT[(size_t)(n + q) * ld + j];
#pragma unroll
    for (int q = 0; q < 8; q += 2) {
      a0 = fmaf(w[q], x[n + q], a0);
      a1 = fmaf(w[q + 1], x[n + q + 1], a1);
    }
  }
  for (; n < n1; ++n) a0 = fmaf(WT[(size_t)n * ld + j], x[n], a0);
  return a0 + a1;
}

__global__ void __launch_bounds__(1024)
k_adj_rec_stream(NetDev net, int l, int t0, int t1, float *__restrict__ vbuf, int t_base,
                 const float *__restrict__ up, int ldu, float *__restrict__ carry, int carry_init) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, NT = blockDim.x, b = blockIdx.x;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN;
  float *xa = (float *)smem; // [N]
  float *xb = xa + N;        // [N]
  float *part = xb + N;      // [NT]
  float *cb = carry + (size_t)b * (SN + net.n_out) + off;
  for (int i = tid; i < N; i += NT) { xa[i] = carry_init ? 0.0f : cb[i]; xb[i] = 0.0f; }
  __syncthreads();
  float *x_next = xa, *x_cur = xb;
  const int NJ = (N + WAVE - 1) & ~(WAVE - 1);
  const int tile = NJ < NT ? NJ : NT;
  const int KG = NT / tile;
  const int kg = tid / tile, jt = tid % tile;
  const int r0 = (int)((long long)N * kg / KG), r1 = (int)((long long)N * (kg + 1) / KG);
  for (int t = t1; t > t0; --t) {
    const size_t slot = (size_t)(t - t_base - 1);
    float *vrow = vbuf + slot * ((size_t)B * SN) + (size_t)b * SN + off;
    const float *urow = up + (slot * B + b) * ldu;
    for (int jb = 0; jb < NJ; jb += tile) {
      const int j = jb + jt;
      const bool act = kg < KG && j < N;
      float vt = 0.0f, upv = 0.0f;
      if (act && kg == 0) { vt = vrow[j]; upv = urow[j]; }
      float p = 0.0f;
      if (act) p = dot_T(net.W_recT[l], N, j, x_next, r0, r1);
      if (kg < KG) part[kg * tile + jt] = p;
      __syncthreads();
      if (act && kg == 0) {
        float s = part[jt];
        for (int q = 1; q < KG; ++q) s = s + part[q * tile + jt];
        const float dn = x_next[j];
        const float ds = (s + upv) - net.theta * dn;
        const float dvt = fmaf(ds, surrogate(net, vt), net.alpha * dn);
        x_cur[j] = dvt;
        vrow[j] = dvt;
      }
      __syncthreads();
    }
    float *tmp = x_next; x_next = x_cur; x_cur = tmp;
  }
  for (int i = tid; i < N; i += NT) cb[i] = x_next[i];
}

// B3/B4 under a surrogate window, event-driven (layers wider than 256 neurons; one workgroup per batch element).
// With a window w > 0 the surrogate derivative is zero for every neuron whose potential is at least w away from
// the threshold; for those dv_t = fma(ds, 0, alpha dv_{t+1}) = alpha dv_{t+1} whatever ds is, so the row of
// W_rec . dv_{t+1} that would give ds is never evaluated.  Per step the workgroup (a) classifies its neurons from
// the stored v_t, finishes the ones outside the window at once and compacts the others into an ascending list
// (ballot, popcount prefix: the spike compaction of the forward pass applied to |v - theta| < w), (b) evaluates the
// listed rows only, one wavefront per row: lane-strided products accumulated in index order, then a fixed-order sum
// over the lanes (wave_sum) -- an order that depends on the row alone, so listing every row (list_all, the dense form of the
// very same kernel) gives the same bits for the rows inside the window.  A masked recurrent matrix is read through
// its compressed rows: only the synapses that exist.  dv_{t+1} of the batch element stays in LDS.
__global__ void __launch_bounds__(1024)
k_adj_rec_rows(NetDev net, AdjJobs jobs, float *__restrict__ carry, int list_all) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int wcnt[16];
  const AdjJob &jb = jobs.j[blockIdx.y];
  const int l = jb.l, t0 = jb.t0, t1 = jb.t1, t_base = jb.t_base;
  float *__restrict__ vbuf = jb.vbuf;
  const float *__restrict__ up = jb.up;
  const int tid = threadIdx.x, NT = blockDim.x, b = blockIdx.x, lane = tid & 63, wave = tid >> 6, NW = NT >> 6;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, ldu = N;
  float *xa = (float *)smem;                 // [N]
  float *xb = xa + N;                        // [N]
  uint16_t *list = (uint16_t *)(xb + N);     // [N]
  float *cb = carry + (size_t)b * (SN + net.n_out) + off;
  for (int i = tid; i < N; i += NT) { xa[i] = jb.carry_init ? 0.0f : cb[i]; xb[i] = 0.0f; }
  __syncthreads();
  float *x_next = xa, *x_cur = xb;
  const float *__restrict__ Wl = net.W_rec[l];
  const uint32_t *__restrict__ sub = net.csr_sub[l];
  const uint16_t *__restrict__ col = net.csr_col[l];
  const float *__restrict__ val = net.csr_val[l];
  const int nsub1 = (N + SNN_CSR_SUBW - 1) / SNN_CSR_SUBW + 1;
  const bool vec4 = (N & 3) == 0;
  for (int t = t1; t > t0; --t) {
    const size_t slot = (size_t)(t - t_base - 1);
    float *vrow = vbuf + slot * ((size_t)B * SN) + (size_t)b * SN + off;
    const float *urow = up + (slot * B + b) * ldu;
    // (a) classify, finish the neurons outside the window, list the others in ascending order
    int cnt = 0;
    for (int j0 = 0; j0 < N; j0 += NT) {
      const int j = j0 + tid;
      bool inside = false;
      if (j < N) {
        const float vt = vrow[j];
        inside = list_all || !(net.win > 0.0f) || fabsf(vt - net.theta) < net.win;
        if (!inside) {
          const float dvt = net.alpha * x_next[j];
          x_cur[j] = dvt;
          vrow[j] = dvt;
        }
      }
      const uint64_t m = __ballot(inside);
      if (lane == 0) wcnt[wave] = __popcll(m);
      __syncthreads();
      int before = 0, total = 0;
      for (int q = 0; q < NW; ++q) {
        const int c = wcnt[q];
        before += q < wave ? c : 0;
        total += c;
      }
      if (inside) list[cnt + before + __popcll(m & lanemask_lt())] = (uint16_t)j;
      cnt += total;
      __syncthreads();
    }
    // (b) the listed rows, one wavefront per row (rows wave, wave + NW, ... of the list)
    auto finish = [&](int j, float a0, float a1) {
      const float sacc = wave_sum(a0 + a1);
      if (lane == 0) {
        const float dn = x_next[j];
        const float ds = (sacc + urow[j]) - net.theta * dn;
        const float dvt = fmaf(ds, surrogate(net, vrow[j]), net.alpha * dn);
        x_cur[j] = dvt;
        vrow[j] = dvt;
      }
    };
    if (sub) {
      // compressed rows: the positions of this wavefront's next 64 rows are fetched at once (one row per lane); the
      // entries of a row (up to CH x 64 per pass) are all in flight before the first product, and the next row's
      // are requested before this row's products start
      constexpr int CH = 16;
      const int mine = cnt > wave ? (cnt - wave + NW - 1) / NW : 0; // rows of this wavefront
      struct Row { float w[CH]; uint32_t c[CH]; };
      auto fetch = [&](Row &r, uint32_t eb, uint32_t e1) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
          const uint32_t e = eb + (uint32_t)(WAVE * i + lane);
          const bool ok = e < e1;
          r.w[i] = ok ? val[e] : 0.0f;
          r.c[i] = ok ? (uint32_t)col[e] : 0u;
        }
      };
      auto mac = [&](const Row &r, float &a0, float &a1) {
#pragma unroll
        for (int i = 0; i < CH; i += 2) {
          a0 = fmaf(r.w[i], x_next[r.c[i]], a0);
          a1 = fmaf(r.w[i + 1], x_next[r.c[i + 1]], a1);
        }
      };
      for (int rb = 0; rb < mine; rb += WAVE) {
        uint32_t m0 = 0u, m1 = 0u;
        int mj = 0;
        if (rb + lane < mine) {
          mj = list[wave + NW * (rb + lane)];
          m0 = sub[(size_t)mj * nsub1];
          m1 = sub[(size_t)mj * nsub1 + nsub1 - 1];
        }
        const int nr = mine - rb < WAVE ? mine - rb : WAVE;
        Row ra, rbuf;
        fetch(ra, __builtin_amdgcn_readlane(m0, 0), __builtin_amdgcn_readlane(m1, 0));
        for (int q = 0; q < nr; ++q) {
          const uint32_t e0 = __builtin_amdgcn_readlane(m0, q), e1 = __builtin_amdgcn_readlane(m1, q);
          const int j = __builtin_amdgcn_readlane(mj, q);
          const int qn = q + 1 < nr ? q + 1 : q; // past the end: the same row again, never used
          __builtin_amdgcn_sched_barrier(0);
          fetch(rbuf, __builtin_amdgcn_readlane(m0, qn), __builtin_amdgcn_readlane(m1, qn));
          __builtin_amdgcn_sched_barrier(0);
          float a0 = 0.0f, a1 = 0.0f;
          mac(ra, a0, a1);
          for (uint32_t eb = e0 + CH * WAVE; eb < e1; eb += CH * WAVE) { // rows longer than one pass
            Row more;
            fetch(more, eb, e1);
            mac(more, a0, a1);
          }
          finish(j, a0, a1);
          ra = rbuf;
        }
      }
    } else {
      for (int idx = wave; idx < cnt; idx += NW) {
        const int j = list[idx];
        float a0 = 0.0f, a1 = 0.0f;
        if (vec4) {
          const float4 *wr = reinterpret_cast<const float4 *>(Wl + (size_t)j * N);
          const float4 *xr = reinterpret_cast<const float4 *>(x_next);
          const int n4 = N >> 2;
          for (int i0 = 0; i0 < n4; i0 += 8 * WAVE) { // 8 loads of 16 bytes in flight per lane
            float4 wv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              const int i = i0 + u * WAVE + lane;
              wv[u] = i < n4 ? wr[i] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              const int i = i0 + u * WAVE + lane;
              const float4 xv = xr[i < n4 ? i : 0];
              float &a = (u & 1) ? a1 : a0;
              a = fmaf(wv[u].x, xv.x, a); a = fmaf(wv[u].y, xv.y, a); a = fmaf(wv[u].z, xv.z, a); a = fmaf(wv[u].w, xv.w, a);
            }
          }
        } else {
          const float *wr = Wl + (size_t)j * N;
          int n = lane;
          for (; n + WAVE < N; n += 2 * WAVE) {
            a0 = fmaf(wr[n], x_next[n], a0);
            a1 = fmaf(wr[n + WAVE], x_next[n + WAVE], a1);
          }
          if (n < N) a0 = fmaf(wr[n], x_next[n], a0);
        }
        finish(j, a0, a1);
      }
    }
    __syncthreads();
    float *tmp = x_next; x_next = x_cur; x_cur = tmp;
  }
  for (int i = tid; i < N; i += NT) cb[i] = x_next[i];
}

// B3/B4 for wide layers whose recurrent matrix is masked: the chip-wide recurrence over the compressed rows.
// Streaming the dense-stored matrix costs 4 N^2 bytes per step whatever the mask; the compressed rows hold 6 bytes
// per synapse that exists.  Workgroup (job, row block rb, batch group bg) owns R = ceil(N / n_rb) postsynaptic rows
// and four batch elements: dv_{t+1} of those four, all N neurons, sits in LDS as float4 per neuron (16 N bytes), so
// one 16-byte LDS read per synapse feeds four FMAs and a row of the matrix is fetched once for four batch elements.
// The eight (or ceil(B / 4)) workgroups that share a row block are placed on the same die: they stream the same
// rows at about the same time, so the die's L2 serves seven of the eight reads.  Rows are dealt to the sixteen
// wavefronts in contiguous runs; a wavefront evaluates a row like k_adj_rec_rows does -- entries lane-strided, two
// accumulators taking alternate groups of 64 entries, then wave_sum over the lanes: the same order, so the
// same bits as that kernel listing every row -- with all entries of the next row requested before the products of
// the current one (the first row of the next step before the step's barrier: the matrix does not change).  Lane r
// then finishes row r for the four batch elements and writes dv_t as one float4 into the exchange buffer
// [parity][batch group][N][4]; a counting barrier per (job, batch group) -- the batch groups never wait for each
// other -- and every workgroup reloads its group's slice into LDS.  Bounded spin and error flag as in k_adj_rec_ws.
__global__ void __launch_bounds__(1024)
k_adj_rec_csrw(NetDev net, AdjJobs jobs, float *__restrict__ carry, float *xg, unsigned *bar, unsigned *err,
               unsigned spin_limit, int n_rb, int n_bg, int xg_stride, int lds_n) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_dead;
  float4 *xs = reinterpret_cast<float4 *>(smem); // [N]: dv_{t+1} of the group's four batch elements
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  float4 *sums = xs + lds_n + 64 * wave; // [16][64] behind the widest layer's slice: the row sums of a step, per wavefront
  if (tid == 0) s_dead = 0;
  // workgroups are dealt to the eight dies in turn: all batch groups of a (job, row block) onto one die
  const int G = jobs.count * n_rb;
  int g, bg;
  if ((G & 7) == 0) {
    const int die = (int)blockIdx.x & 7, k = (int)blockIdx.x >> 3;
    g = die + 8 * (k / n_bg);
    bg = k % n_bg;
  } else {
    g = (int)blockIdx.x / n_bg;
    bg = (int)blockIdx.x % n_bg;
  }
  const int jq = g / n_rb, rb = g % n_rb;
  const AdjJob &jb = jobs.j[jq];
  const int l = jb.l, t0 = jb.t0, t1 = jb.t1, t_base = jb.t_base;
  float *__restrict__ vbuf = jb.vbuf;
  const float *__restrict__ up = jb.up;
  const int N = net.N[l], off = net.off[l], B = net.B, SN = net.SN, O = net.n_out, ldu = N;
  const uint32_t *__restrict__ sub = net.csr_sub[l];
  const uint16_t *__restrict__ col = net.csr_col[l];
  const float *__restrict__ val = net.csr_val[l];
  const uint64_t *__restrict__ pk = net.csr_pk[l];
  const int nsub1 = (N + SNN_CSR_SUBW - 1) / SNN_CSR_SUBW + 1;
  // rows: the workgroup's [rb R, rb R + R), the wavefront's nr <= 64 consecutive ones from jw0; lane r keeps the
  // position of row jw0 + r
  const int R = (N + n_rb - 1) / n_rb, nrw = (R + 15) / 16;
  const int row_end = (rb + 1) * R < N ? (rb + 1) * R : N;
  const int jw0 = rb * R + wave * nrw;
  const int jw1 = jw0 + nrw < row_end ? jw0 + nrw : row_end;
  const int nr = jw1 > jw0 ? jw1 - jw0 : 0;
  const int j = jw0 + lane;
  uint32_t m0 = 0u, m1 = 0u;
  if (lane < nr) {
    m0 = sub[(size_t)j * nsub1];
    m1 = sub[(size_t)j * nsub1 + nsub1 - 1];
  }
  float *xq = xg + (size_t)jq * xg_stride; // [2][n_bg][N][4]
  const __amdgpu_buffer_rsrc_t xres =
      __builtin_amdgcn_make_buffer_rsrc((void *)xq, 0, (int)((size_t)2 * n_bg * N * 4 * sizeof(float)), 0x00027000);
  unsigned *cnt = bar + 64 * jq + bg;
  bool dead = false;
  unsigned arrivals = 0;
  auto group_barrier = [&]() {
    // see k_adj_rec_ws: every wave waits for its own stores, then one arrival per workgroup
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
    __syncthreads();
    arrivals += (unsigned)n_rb;
    if (tid == 0 && !dead) {
      __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      unsigned spins = 0;
      while (spin_limit == 0u || __hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < arrivals) {
        if (++spins > spin_limit ||
            ((spins & 63u) == 0u && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
          __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          s_dead = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
    }
    __syncthreads();
    if (s_dead) dead = true; // keep going to the end of the chunk, never wait again
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  };
  // dv_{t1+1} of the group's batch elements; nobody writes the carry before every workgroup has read it
  for (int i = tid; i < N; i += 1024) {
    float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (!jb.carry_init) {
      const float *cp = carry + (size_t)(4 * bg) * (SN + O) + off + i;
      if (4 * bg + 0 < B) v.x = cp[0];
      if (4 * bg + 1 < B) v.y = cp[(size_t)1 * (SN + O)];
      if (4 * bg + 2 < B) v.z = cp[(size_t)2 * (SN + O)];
      if (4 * bg + 3 < B) v.w = cp[(size_t)3 * (SN + O)];
    }
    xs[i] = v;
  }
  group_barrier();
  // Entries of a row through buffer loads whose range is the row: lane + 64 i past the end reads 0 (weight 0, column
  // 0) with no address arithmetic or compare in the vector unit.
  constexpr int CH = 14, CH2 = 2; // groups of 64 entries per pass (both even: group k always meets accumulator k & 1)
  struct Row { float w[CH]; uint32_t c[CH]; };
  // (weight and index of an entry come as one 8-byte load from the packed copy of the rows, NetDev::csr_pk)
  auto fetch = [&](Row &r, uint32_t e0, uint32_t e1) {
    const __amdgpu_buffer_rsrc_t rp =
        __builtin_amdgcn_make_buffer_rsrc((void *)(pk + e0), 0, (int)((e1 - e0) * sizeof(uint64_t)), 0x00027000);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const csr_u32x2 e = __builtin_amdgcn_raw_buffer_load_b64(rp, (uint32_t)(lane * 8), 512 * i, 0);
      r.w[i] = __builtin_bit_cast(float, e.x);
      r.c[i] = e.y;
    }
  };
  // one row: its entries sit in `r` (requested a row ago); each pair of registers is reloaded with the next row's
  // entries right after its products, so one row buffer serves both rows
  Row r;
  auto do_row = [&](int q) {
    const uint32_t e0 = __builtin_amdgcn_readlane(m0, q), e1 = __builtin_amdgcn_readlane(m1, q);
    const int qn = q + 1 < nr ? q + 1 : 0; // after the last row: the first row of the next step
    const uint32_t n0 = __builtin_amdgcn_readlane(m0, qn), n1 = __builtin_amdgcn_readlane(m1, qn);
    const __amdgpu_buffer_rsrc_t np =
        __builtin_amdgcn_make_buffer_rsrc((void *)(pk + n0), 0, (int)((n1 - n0) * sizeof(uint64_t)), 0x00027000);
    float a0[4] = {0.0f, 0.0f, 0.0f, 0.0f}, a1[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    auto fma2 = [&](float w0, const float4 &x0, float w1, const float4 &x1) {
      a0[0] = fmaf(w0, x0.x, a0[0]); a0[1] = fmaf(w0, x0.y, a0[1]);
      a0[2] = fmaf(w0, x0.z, a0[2]); a0[3] = fmaf(w0, x0.w, a0[3]);
      a1[0] = fmaf(w1, x1.x, a1[0]); a1[1] = fmaf(w1, x1.y, a1[1]);
      a1[2] = fmaf(w1, x1.z, a1[2]); a1[3] = fmaf(w1, x1.w, a1[3]);
    };
    auto mac2 = [&](float w0, uint32_t c0, float w1, uint32_t c1) { fma2(w0, xs[c0], w1, xs[c1]); };
    // the LDS reads of a pair of groups are issued before the products of the pair before it
    float4 xa = xs[r.c[0]], xb = xs[r.c[1]];
#pragma unroll
    for (int i = 0; i < CH; i += 2) {
      float4 na = xa, nb = xb;
      if (i + 2 < CH) {
        na = xs[r.c[i + 2]];
        nb = xs[r.c[i + 3]];
      }
      fma2(r.w[i], xa, r.w[i + 1], xb);
#pragma unroll
      for (int h = i; h < i + 2; ++h) { // the next row's entries into the registers just used
        const csr_u32x2 e = __builtin_amdgcn_raw_buffer_load_b64(np, (uint32_t)(lane * 8), 512 * h, 0);
        r.w[h] = __builtin_bit_cast(float, e.x);
        r.c[h] = e.y;
      }
      xa = na;
      xb = nb;
    }
    if (e1 - e0 > (uint32_t)(CH * WAVE)) { // rows longer than one pass
      const __amdgpu_buffer_rsrc_t rv =
          __builtin_amdgcn_make_buffer_rsrc((void *)(val + e0), 0, (int)((e1 - e0) * sizeof(float)), 0x00027000);
      const __amdgpu_buffer_rsrc_t rc =
          __builtin_amdgcn_make_buffer_rsrc((void *)(col + e0), 0, (int)((e1 - e0) * sizeof(uint16_t)), 0x00027000);
      for (uint32_t eb = CH * WAVE; eb < e1 - e0; eb += CH2 * WAVE) {
        const uint32_t o = eb + (uint32_t)lane;
        const float w0 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rv, o * 4u, 0, 0));
        const float w1 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rv, (o + WAVE) * 4u, 0, 0));
        const uint32_t c0 = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rc, o * 2u, 0, 0);
        const uint32_t c1 = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rc, (o + WAVE) * 2u, 0, 0);
        mac2(w0, c0, w1, c1);
      }
    }
    const float4 sum4 = make_float4(wave_sum_lane63(a0[0] + a1[0]), wave_sum_lane63(a0[1] + a1[1]),
                                    wave_sum_lane63(a0[2] + a1[2]), wave_sum_lane63(a0[3] + a1[3]));
    if (lane == 63) sums[q] = sum4; // read back by lane q of this wavefront when the step's rows are done
  };
  if (nr > 0) fetch(r, __builtin_amdgcn_readlane(m0, 0), __builtin_amdgcn_readlane(m1, 0));
  const size_t slot_stride = (size_t)B * SN;
  unsigned step = 0;
  for (int t = t1; t > t0; --t, ++step) {
    const int wr = (int)(step & 1u);
    const size_t slot = (size_t)(t - t_base - 1);
    float vt[4] = {0.0f, 0.0f, 0.0f, 0.0f}, upv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (lane < nr) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (4 * bg + c < B) {
          vt[c] = vbuf[slot * slot_stride + (size_t)(4 * bg + c) * SN + off + j];
          upv[c] = up[(slot * B + 4 * bg + c) * ldu + j];
        }
    }
    for (int q = 0; q < nr; ++q) do_row(q);
    const bool last = t == t0 + 1;
    if (lane < nr) {
      const float4 dn4 = xs[j], my4 = sums[lane];
      const float dn[4] = {dn4.x, dn4.y, dn4.z, dn4.w}, mys[4] = {my4.x, my4.y, my4.z, my4.w};
      float dv[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool ok = 4 * bg + c < B;
        const float ds = (mys[c] + upv[c]) - net.theta * dn[c];
        const float dvt = fmaf(ds, surrogate(net, vt[c]), net.alpha * dn[c]);
        dv[c] = ok ? dvt : 0.0f;
        if (ok) {
          vbuf[slot * slot_stride + (size_t)(4 * bg + c) * SN + off + j] = dvt;
          if (last) carry[(size_t)(4 * bg + c) * (SN + O) + off + j] = dvt; // dv_{t0+1}: every workgroup its own rows
        }
      }
      if (!last)
        *reinterpret_cast<float4 *>(xq + (((size_t)wr * n_bg + bg) * N + j) * 4) = make_float4(dv[0], dv[1], dv[2], dv[3]);
    }
    if (last) break; // nobody reads the exchange buffer after the last step
    group_barrier();
    const uint32_t xbase = (uint32_t)((((size_t)wr * n_bg + bg) * N) * 4 * sizeof(float));
    for (int i0 = 0; i0 < N; i0 += 8 * 1024) {
      float4 r[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * 1024 + tid, ic = i < N ? i : N - 1;
        r[u] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(xres, xbase + (uint32_t)ic * 16u, 0, 17)); // sc0 sc1
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * 1024 + tid;
        if (i < N) xs[i] = r[u];
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// B5: weight gradient over active spikes.  One workgroup per presynaptic row j (x column tile);
// dW[j][:] += sum_{t = t1..t0+1 desc} sum_{b asc} [spike(t - lag, b, j)] * post(t, b, :)
// Sequential per-element accumulation continued from the value already in dW, so the result
// does not depend on how the time axis is cut into launches.  The accumulators are fp64 (tens of
// thousands of same-sign fp32 terms per element would otherwise lose ~1e-4 of the result); the
// gradient is rounded to fp32 once, at the end of the training step.
// ------------------------------------------------------------------------------------------
#define DW_NPT 4
__global__ void __launch_bounds__(256)
k_dw(const uint64_t *__restrict__ pre_mask, int pre_words, int lag, const float *__restrict__ postbuf,
     size_t slot_stride, int post_stride, int post_off, int n_post, int B, int t0, int t1, int t_base,
     double *__restrict__ dW, int pre_ring) {
  const int j = blockIdx.x;
  const int c0 = blockIdx.y * (256 * DW_NPT) + threadIdx.x;
  double acc[DW_NPT];
#pragma unroll
  for (int k = 0; k < DW_NPT; ++k) {
    const int n = c0 + k * 256;
    acc[k] = n < n_post ? dW[(size_t)j * n_post + n] : 0.0;
  }
  const int wj = j >> 6;
  const uint64_t bit = 1ull << (j & 63);
  for (int t = t1; t > t0; --t) {
    const int tp = t - lag; // step 0 of the mask is all zero
    const uint64_t *mrow = pre_mask + (size_t)(pre_ring > 0 ? tp % pre_ring : tp) * B * pre_words + wj;
    const float *prow = postbuf + (size_t)(t - t_base - 1) * slot_stride + post_off;
    for (int b = 0; b < B; ++b) {
      if (mrow[(size_t)b * pre_words] & bit) {
        const float *p = prow + (size_t)b * post_stride;
#pragma unroll
        for (int k = 0; k < DW_NPT; ++k) {
          const int n = c0 + k * 256;
          if (n < n_post) acc[k] = acc[k] + (double)p[n];
        }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < DW_NPT; ++k) {
    const int n = c0 + k * 256;
    if (n < n_post) dW[(size_t)j * n_post + n] = acc[k];
  }
}

// ------------------------------------------------------------------------------------------
// B5, dense path: dW += S^T . P on the matrix cores, where S[(t,b)][j] are the presynaptic spikes (0/1)
// and P[(t,b)][n] the postsynaptic adjoints dv_t (or du_t).  At the activity levels the benchmark
// networks run at, adding rows event by event moves more bytes than this contraction costs in flops.
// v_mfma_f32_16x16x4: one K-step covers 4 consecutive batch elements of one time step.  The products of
// ONE time step (b ascending) are summed in an fp32 accumulator that starts from zero; at the end of the
// time step it is added to the fp64 accumulator that persists in HBM between launches (a sum of at most
// a few hundred exact terms in fp32, then tens of thousands of time steps in fp64).  Time steps run in
// descending order and a chunk boundary is always a time-step boundary, so the sequence of operations
// applied to an element does not depend on how the time axis is cut into chunks: every storage strategy
// gets bit-identical gradients.  A K-step whose 16x4 spike block is empty is skipped (it would add exact
// zeros).  Why not the fp64 matrix instruction: on this chip it runs at the rate of, and instead of, the
// fp64 vector unit (the counters show no cycle in which a VALU instruction and an fp64 MFMA overlap), so
// the ten VALU instructions that prepare each K-step cost as much again as the MFMA itself; the fp32
// matrix core is twice as fast and runs beside the VALU.
// Lane layouts (checked on gfx950): A[i][k] in lane i + 16k, B[k][j] in lane j + 16k,
// D[4*(lane/16) + r][lane%16] in register r of the lane.
// One launch covers every weight matrix of the network: blockIdx.x -> (matrix, 64 x 16*NT*CW tile).
// ------------------------------------------------------------------------------------------
#define DW_STAGE_ELEMS 4096 // elements of P per stage of the contraction (rows x columns of a tile)
typedef double dvec4 __attribute__((ext_vector_type(4)));

template <int NT, int CW>
__device__ __forceinline__ void dw_mfma_body(const DwBatch &batch, int B, int vblock, unsigned char *smem) {
  int di = 0;
  while (di + 1 < batch.count && vblock >= batch.d[di + 1].tile0) ++di;
  const DwDesc &d = batch.d[di];
  const int t0 = d.t0, t1 = d.t1, t_base = d.t_base;
  const int tile = vblock - d.tile0;
  constexpr int COLS = 16 * NT * CW;
  const int j0 = (tile / d.tiles_n) * 64, n0 = (tile % d.tiles_n) * COLS;
  // wavefront (w, cg): presynaptic rows 16w .. 16w+15 of the tile, column blocks NT*cg .. NT*cg+NT-1.
  // With CW > 1 two (or four) wavefronts share a SIMD, so that the operand preparation of one overlaps
  // the MFMAs of the other.
  const int tid = threadIdx.x, lane = tid & 63, w = (tid >> 6) & 3, cb0 = NT * (tid >> 8);
  const int Bp = (B + 3) & ~3;
  constexpr int STRIDE = COLS + 16; // rows 16 banks apart: conflict-free operand reads
  // staging: thread -> (row, 4 columns) of the P tile; the threads cover RPP rows per pass, NPASS passes.
  // A stage holds TS consecutive time steps (row = ts*Bp + b, step t_hi - ts): several steps of
  // MFMAs per barrier, so that the global loads of the next stage (issued before the MFMAs of the
  // current one) have time to arrive.
  constexpr int TPR = COLS / 4;          // threads per row
  constexpr int RPP = 256 * CW / TPR;    // rows per pass
  constexpr int NPASS = DW_STAGE_ELEMS / 1024 / CW;
  constexpr int ROWS = NPASS * RPP;      // rows per stage (= DW_STAGE_ELEMS / COLS)
  const int TS = ROWS / Bp;              // time steps per stage (>= 1: the launcher checks Bp <= ROWS)
  float *Pt = (float *)smem;                                   // [2][ROWS][STRIDE]
  uint64_t *Sw = (uint64_t *)(Pt + (size_t)2 * ROWS * STRIDE); // [2][ROWS]
  const int li = lane & 15, lk = lane >> 4;

  dvec4 acc[NT];
  v4f part[NT]; // fp32 sum of the current time step
  const int kpt = Bp >> 2;
  const bool galign = (kpt & 3) == 0; // a time step is a whole number of K-step groups
  int kin = 0;
#pragma unroll
  for (int q = 0; q < NT; ++q) part[q] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int q = 0; q < NT; ++q)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int j = j0 + 16 * w + 4 * lk + r, n = n0 + 16 * (cb0 + q) + li;
      acc[q][r] = (j < d.n_pre && n < d.n_post) ? d.acc[(size_t)j * d.n_post + n] : 0.0;
    }

  const int srow = tid / TPR, scol = (tid % TPR) * 4;
  // rows of the stage that starts at step t_hi and covers nts steps.  stage_load only issues the
  // loads -- unconditionally, from clamped (valid) addresses, so that all of them are in flight
  // together while the MFMAs of the current stage run; stage_store zeroes what lies outside the
  // stage (integer masks: a select would let the compiler move a load back under its condition)
  // and writes the tile to LDS.
  auto stage_load = [&](int t_hi, int nts, float (&reg)[NPASS][4], uint64_t &wreg) {
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
      const int r = srow + ps * RPP, ts = r / Bp, b = r - ts * Bp;
      const bool ok = ts < nts && b < B;
      const float *prow = d.post + (size_t)(t_hi - (ok ? ts : 0) - t_base - 1) * d.slot_stride + d.post_off +
                          (size_t)(ok ? b : 0) * d.post_stride;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int n = n0 + scol + c;
        reg[ps][c] = prow[n < d.n_post ? n : d.n_post - 1];
      }
    }
    {
      const int ts = tid / Bp, b = tid - ts * Bp;
      const bool ok = tid < ROWS && ts < nts && b < B;
      const int tt = t_hi - (ok ? ts : 0) - d.lag; // its row of the stored spike words (a ring in time if d.pre_ring > 0)
      wreg = d.pre_mask[((size_t)(d.pre_ring > 0 ? tt % d.pre_ring : tt) * B + (ok ? b : 0)) * d.pre_words + (j0 >> 6)];
    }
  };
  auto stage_store = [&](int buf, int nts, const float (&reg)[NPASS][4], uint64_t wreg) {
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
      const int r = srow + ps * RPP, ts = r / Bp, b = r - ts * Bp;
      const bool ok = ts < nts && b < B;
      float *dst = Pt + ((size_t)buf * ROWS + r) * STRIDE + scol;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        dst[c] = __uint_as_float(__float_as_uint(reg[ps][c]) & (0u - (uint32_t)(ok && n0 + scol + c < d.n_post)));
    }
    if (tid < ROWS) {
      const int ts = tid / Bp, b = tid - ts * Bp;
      Sw[(size_t)buf * ROWS + tid] = wreg & (0ull - (uint64_t)(ts < nts && b < B));
    }
  };

  // Stage s covers steps t1 - s*TS, ... (TS of them, fewer in the last).  The loads of PF stages are in
  // flight while a stage is multiplied.  Register sets are indexed statically (the stage loop is unrolled
  // PF times); loads for stages past the end are still issued (clamped to the last stage) so that the
  // number of loads in flight is the same on every path and the compiler can wait for exactly the oldest
  // set.  Measured: a depth beyond 1 buys nothing (37.5 us per 32-step launch at PF = 4, 34.8 at PF = 1):
  // the stage loop is bound by the matrix cores and the operand preparation, not by memory latency.
  constexpr int PF = 1;
  const int nstages = (t1 - t0 + TS - 1) / TS;
  float reg[PF][NPASS][4];
  uint64_t wreg[PF];
  auto t_of = [&](int sidx) { return t1 - (sidx < nstages ? sidx : nstages - 1) * TS; };
  auto n_of = [&](int sidx) { const int th = t_of(sidx); return th - t0 < TS ? th - t0 : TS; };
#pragma unroll
  for (int pf = 0; pf < PF; ++pf) stage_load(t_of(pf), n_of(pf), reg[pf], wreg[pf]);
  stage_store(0, n_of(0), reg[0], wreg[0]);
  __syncthreads();
  int buf = 0;
  for (int s0 = 0; s0 < nstages; s0 += PF) {
#pragma unroll
    for (int pf = 0; pf < PF; ++pf) {
      const int sidx = s0 + pf;
      if (sidx >= nstages) break;
      const int nts = n_of(sidx);
      stage_load(t_of(sidx + PF), n_of(sidx + PF), reg[pf], wreg[pf]); // set pf went to LDS one stage ago
      const float *P = Pt + (size_t)buf * ROWS * STRIDE;
      const uint64_t *S = Sw + (size_t)buf * ROWS;
      // (t descending, b ascending), 4 batch elements per K-step.  The operands of KU K-steps are read
      // from LDS one group ahead of the MFMAs that use them (rows past the stage's last one hold zeros,
      // and the buffer has a whole group of them to spare only when the stage is not full: the read
      // of the group after the last is clamped to the last one and discarded).
      constexpr int KU = 4;
      const int nrows = nts * Bp;
      uint32_t word[2][KU]; // the 32-bit half of the spike word that holds this wavefront's 16 presynaptic rows
      float pv[2][KU][NT];
      const uint32_t *S32 = reinterpret_cast<const uint32_t *>(S) + (w >> 1);
      const int sh = 16 * (w & 1) + li;
      auto fetch = [&](int r0, uint32_t (&wd)[KU], float (&p)[KU][NT]) {
        const int rr = r0 < nrows ? r0 : nrows - 4 * KU < 0 ? 0 : ((nrows - 1) / (4 * KU)) * (4 * KU);
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          wd[u] = S32[2 * (rr + 4 * u + lk)];
          const float *prow = P + (size_t)(rr + 4 * u + lk) * STRIDE + 16 * cb0 + li;
#pragma unroll
          for (int q = 0; q < NT; ++q) p[u][q] = prow[16 * q];
        }
      };
      auto flush = [&]() {
#pragma unroll
        for (int q = 0; q < NT; ++q)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            acc[q][r] = acc[q][r] + (double)part[q][r];
            part[q][r] = 0.0f;
          }
      };
      // One group of KU K-steps.  SKIP (sparse presynaptic layers only): a K-step whose 16 x 4 spike block is
      // empty is skipped (it would add exact zeros); for dense layers the test costs more than it saves, and
      // the group is straight-line code.
      auto group = [&](auto skip, const uint32_t (&wd)[KU], const float (&p)[KU][NT]) {
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          const uint32_t bit = (wd[u] >> sh) & 1u;
          if (decltype(skip)::value && __ballot(bit != 0u) == 0ull) continue;
          const float a = (float)bit;
#pragma unroll
          for (int q = 0; q < NT; ++q) part[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, p[u][q], part[q], 0, 0, 0);
        }
      };
      // After the last K-step of a time step (Bp / 4 of them) the fp32 sum of the time step goes into the
      // fp64 accumulator.  When a time step is a whole number of groups (gpt), the stage is a plain loop over
      // groups; otherwise K-steps are counted one by one and those past the stage's last row left out.
      auto run_aligned = [&](auto skip) {
        const int ng = nrows / (4 * KU), gpt = kpt / KU;
        int gin = 0;
        fetch(0, word[0], pv[0]);
        for (int g = 0; g < ng; g += 2) {
          fetch((g + 1) * 4 * KU, word[1], pv[1]);
          group(skip, word[0], pv[0]);
          if (++gin == gpt) { gin = 0; flush(); }
          if (g + 1 >= ng) break;
          fetch((g + 2) * 4 * KU, word[0], pv[0]);
          group(skip, word[1], pv[1]);
          if (++gin == gpt) { gin = 0; flush(); }
        }
      };
      auto mma_counted = [&](int rbase, const uint32_t (&wd)[KU], const float (&p)[KU][NT]) {
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          if (rbase + 4 * u >= nrows) break; // uniform
          const uint32_t bit = (wd[u] >> sh) & 1u;
          if (__ballot(bit != 0u) != 0ull) {
            const float a = (float)bit;
#pragma unroll
            for (int q = 0; q < NT; ++q) part[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, p[u][q], part[q], 0, 0, 0);
          }
          if (++kin == kpt) { kin = 0; flush(); }
        }
      };
      if (galign) {
        if (d.skip_empty) run_aligned(std::true_type{});
        else run_aligned(std::false_type{});
      } else {
        fetch(0, word[0], pv[0]);
        for (int r0 = 0; r0 < nrows; r0 += 8 * KU) {
          fetch(r0 + 4 * KU, word[1], pv[1]);
          mma_counted(r0, word[0], pv[0]);
          if (r0 + 4 * KU >= nrows) break;
          fetch(r0 + 8 * KU, word[0], pv[0]);
          mma_counted(r0 + 4 * KU, word[1], pv[1]);
        }
      }
      if (sidx + 1 < nstages) stage_store(buf ^ 1, n_of(sidx + 1), reg[(pf + 1) % PF], wreg[(pf + 1) % PF]);
      __syncthreads();
      buf ^= 1;
    }
  }
#pragma unroll
  for (int q = 0; q < NT; ++q)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int j = j0 + 16 * w + 4 * lk + r, n = n0 + 16 * (cb0 + q) + li;
      if (j < d.n_pre && n < d.n_post) d.acc[(size_t)j * d.n_post + n] = acc[q][r];
    }
}

template <int NT, int CW>
__global__ void __launch_bounds__(256 * CW)
k_dw_mfma(DwBatch batch, int B) {
  extern __shared__ __align__(16) unsigned char smem[];
  dw_mfma_body<NT, CW>(batch, B, (int)blockIdx.x, smem);
}

// B5, event-driven and tiled (networks with very large matrices at a few percent activity, where the dense
// contraction above spends nineteen of twenty matrix-core operations on zero spikes).  Workgroup = 128 presynaptic
// rows x 256 postsynaptic columns of one matrix, 16 wavefronts: wavefront w owns rows 8w .. 8w+7, lane q the
// columns 4q .. 4q+3, and keeps the 32 fp64 accumulators of its (row, column) pairs in registers for the whole
// launch (loaded from and stored back to the accumulators in HBM, so the sequence of operations per element is
// the one of the dense version: per time step, descending, an fp32 sum over the batch elements that spiked,
// ascending, started from zero, then one fp64 add).  The time axis runs in tiles of floor(64 / B) steps: the tile's
// adjoint rows P[(t, b)][256 columns] go to LDS (64 KB, two such buffers in turn; the next tile's are in flight in registers meanwhile) and so
// do the spike words of its rows for the workgroup's 128 presynaptic neurons; a ballot over the rows turns the
// words into, per presynaptic neuron, the 64-bit set of rows in which it spiked (wavefront-uniform), and only
// those rows are read from LDS and added: one 16-byte LDS read and four adds per (spike, four columns).
// (Sixteen wavefronts of 8 rows rather than eight of 16: what bounds the kernel is the round trip LDS read -> add of
// consecutive events, and four wavefronts per SIMD hide twice as much of it as two.)
#define DWT_WAVES 16
template <int BS> // BS = 32 / 64: the batch is 32 (a tile is two whole time steps: the halves of a 64-bit set of rows) or 64
                   // (one time step: the whole set); 0: any batch up to 64
__global__ void __launch_bounds__(64 * DWT_WAVES)
k_dw_tile(DwBatch batch, int B) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int PJ = 128, PC = 256, RT = 64, NWV = DWT_WAVES, RW = PJ / NWV, SK = RT / NWV; // rows per wavefront, staging loads per thread
  // two tile buffers in turn: a tile is written while slower wavefronts still read the one before it, so a tile
  // costs one barrier, not two
  float *const Pb = (float *)smem;                       // [2][RT][PC]
  uint64_t *const Wb = (uint64_t *)(Pb + 2 * RT * PC);   // [2][2][RT] spike words of the tile's rows
  float *P = Pb;
  uint64_t *Wv = Wb;
  int di = 0;
  while (di + 1 < batch.count && (int)blockIdx.x >= batch.d[di + 1].tile0) ++di;
  const DwDesc &d = batch.d[di];
  const int tile = (int)blockIdx.x - d.tile0;
  const int j0 = (tile / d.tiles_n) * PJ, n0 = (tile % d.tiles_n) * PC;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = d.t0, t1 = d.t1, t_base = d.t_base;
  const int TS = RT / B;                                  // time steps per tile (B <= 64)
  const int jw = j0 + RW * wave;                          // first presynaptic row of this wavefront
  const int wsel = (RW * wave) >> 6, bitbase = (RW * wave) & 63;
  const int c0 = n0 + 4 * lane;
  // accumulators: continued from HBM
  double acc[RW][4];
#pragma unroll
  for (int i = 0; i < RW; ++i)
#pragma unroll
    for (int c = 0; c < 4; ++c)
      acc[i][c] = (jw + i < d.n_pre && c0 + c < d.n_post) ? d.acc[(size_t)(jw + i) * d.n_post + c0 + c] : 0.0;
  // staging of a tile: thread -> SK x (row, 4 columns); 64 threads cover one row's 256 columns
  const bool al = ((d.post_off + n0) & 3) == 0 && (d.post_stride & 3) == 0 && (d.slot_stride & 3) == 0 &&
                  (((uintptr_t)d.post) & 15) == 0 && n0 + PC <= d.n_post;
  float4 stg[SK];
  auto tile_load = [&](int t_hi, int nts) {
#pragma unroll
    for (int k = 0; k < SK; ++k) {
      const int r = NWV * k + wave, ts = r / B, b = r - ts * B; // row r of the tile: step t_hi - ts, batch element b
      const bool ok = ts < nts;
      const float *prow = d.post + (size_t)(t_hi - (ok ? ts : 0) - t_base - 1) * d.slot_stride + d.post_off +
                          (size_t)(ok ? b : 0) * d.post_stride;
      float4 v;
      if (al) {
        v = *reinterpret_cast<const float4 *>(prow + c0);
      } else {
        v.x = c0 + 0 < d.n_post ? prow[c0 + 0] : 0.0f;
        v.y = c0 + 1 < d.n_post ? prow[c0 + 1] : 0.0f;
        v.z = c0 + 2 < d.n_post ? prow[c0 + 2] : 0.0f;
        v.w = c0 + 3 < d.n_post ? prow[c0 + 3] : 0.0f;
      }
      stg[k] = ok ? v : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
  };
  auto tile_store = [&](int t_hi, int nts) {
#pragma unroll
    for (int k = 0; k < SK; ++k) *reinterpret_cast<float4 *>(P + (size_t)(NWV * k + wave) * PC + 4 * lane) = stg[k];
    if (tid < 2 * RT) { // spike words of the tile's rows for presynaptic neurons j0 .. j0+127
      const int r = tid & (RT - 1), ws = tid >> 6, ts = r / B, b = r - ts * B;
      uint64_t wv = 0ull;
      if (ts < nts && (j0 >> 6) + ws < d.pre_words) {
        const int tt = t_hi - ts - d.lag;
        wv = d.pre_mask[((size_t)(d.pre_ring > 0 ? tt % d.pre_ring : tt) * B + b) * d.pre_words + (j0 >> 6) + ws];
      }
      Wv[ws * RT + r] = wv;
    }
  };
  const uint64_t bmask = B >= 64 ? ~0ull : ((1ull << B) - 1ull);
  int t_hi = t1;
  tile_load(t_hi, t_hi - t0 < TS ? t_hi - t0 : TS);
  for (int it = 0; t_hi > t0; ++it) {
    const int nts = t_hi - t0 < TS ? t_hi - t0 : TS;
    // the buffer read two tiles ago: every wavefront has left it, or it would not have passed the barrier of the tile between
    P = Pb + (it & 1) * RT * PC;
    Wv = Wb + (it & 1) * 2 * RT;
    tile_store(t_hi, nts);
    __syncthreads();
    const int t_next = t_hi - nts;
    if (t_next > t0) tile_load(t_next, t_next - t0 < TS ? t_next - t0 : TS); // in flight during the adds below
    const uint64_t wv = Wv[wsel * RT + lane];
    if constexpr (BS == 64) { // one time step of 64 rows: the row set as it is
#pragma unroll
      for (int i = 0; i < RW; ++i) {
        uint64_t mt = __ballot((wv >> (bitbase + i)) & 1ull); // rows of the tile in which neuron jw + i spiked
        if (mt == 0ull) continue;
        const int k0 = (int)__builtin_ctzll(mt); // the first row starts the sum (see below)
        asm("s_bitset0_b64 %0, %1" : "+s"(mt) : "s"(k0));
        float4 part = *reinterpret_cast<const float4 *>(P + (size_t)k0 * PC + 4 * lane);
        while (mt) {
          const int kb = (int)__builtin_ctzll(mt);
          asm("s_bitset0_b64 %0, %1" : "+s"(mt) : "s"(kb));
          const float4 pv = *reinterpret_cast<const float4 *>(P + (size_t)kb * PC + 4 * lane);
          part.x = part.x + pv.x; part.y = part.y + pv.y; part.z = part.z + pv.z; part.w = part.w + pv.w;
        }
        acc[i][0] = acc[i][0] + (double)part.x;
        acc[i][1] = acc[i][1] + (double)part.y;
        acc[i][2] = acc[i][2] + (double)part.z;
        acc[i][3] = acc[i][3] + (double)part.w;
      }
    } else if constexpr (BS == 32) { // two time steps of 32 rows: the halves of the row set, no shifts, masks or loop counter (rows past nts hold no spikes)
#pragma unroll
      for (int i = 0; i < RW; ++i) {
        const uint64_t m = __ballot((wv >> (bitbase + i)) & 1ull); // rows of the tile in which neuron jw + i spiked
        auto half = [&](uint32_t mt, const float *Ph) {
          // the first row starts the sum (0.0f + x and x differ only for x = -0.0f, and a sum that is -0.0f or +0.0f
          // leaves the fp64 accumulator, which never is -0.0, the same)
          const int k0 = (int)__builtin_ctz(mt);
          asm("s_bitset0_b32 %0, %1" : "+s"(mt) : "s"(k0)); // mt &= ~(1 << k0) as one scalar instruction
          float4 part = *reinterpret_cast<const float4 *>(Ph + (size_t)k0 * PC);
          while (mt) {
            const int kb = (int)__builtin_ctz(mt);
            asm("s_bitset0_b32 %0, %1" : "+s"(mt) : "s"(kb));
            const float4 pv = *reinterpret_cast<const float4 *>(Ph + (size_t)kb * PC);
            part.x = part.x + pv.x; part.y = part.y + pv.y; part.z = part.z + pv.z; part.w = part.w + pv.w;
          }
          acc[i][0] = acc[i][0] + (double)part.x;
          acc[i][1] = acc[i][1] + (double)part.y;
          acc[i][2] = acc[i][2] + (double)part.z;
          acc[i][3] = acc[i][3] + (double)part.w;
        };
        const uint32_t m0 = (uint32_t)m, m1 = (uint32_t)(m >> 32);
        if (m0) half(m0, P + 4 * lane);
        if (m1) half(m1, P + (size_t)32 * PC + 4 * lane);
      }
    } else {
#pragma unroll
      for (int i = 0; i < RW; ++i) {
        const uint64_t m = __ballot((wv >> (bitbase + i)) & 1ull);
        if (m == 0ull) continue;
        for (int ts = 0; ts < nts; ++ts) {
          uint64_t mt = (m >> (ts * B)) & bmask;
          if (mt == 0ull) continue;
          const int k0 = (int)__builtin_ctzll(mt);
          asm("s_bitset0_b64 %0, %1" : "+s"(mt) : "s"(k0));
          float4 part = *reinterpret_cast<const float4 *>(P + (size_t)(ts * B + k0) * PC + 4 * lane);
          while (mt) {
            const int kb = (int)__builtin_ctzll(mt), r = ts * B + kb;
            asm("s_bitset0_b64 %0, %1" : "+s"(mt) : "s"(kb));
            const float4 pv = *reinterpret_cast<const float4 *>(P + (size_t)r * PC + 4 * lane);
            part.x = part.x + pv.x; part.y = part.y + pv.y; part.z = part.z + pv.z; part.w = part.w + pv.w;
          }
          acc[i][0] = acc[i][0] + (double)part.x;
          acc[i][1] = acc[i][1] + (double)part.y;
          acc[i][2] = acc[i][2] + (double)part.z;
          acc[i][3] = acc[i][3] + (double)part.w;
        }
      }
    }
    t_hi = t_next;
  }
#pragma unroll
  for (int i = 0; i < RW; ++i)
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (jw + i < d.n_pre && c0 + c < d.n_post) d.acc[(size_t)(jw + i) * d.n_post + c0 + c] = acc[i][c];
}

// B5 for a masked recurrent matrix, over its compressed rows: the gradient of a synapse that does not exist is
// zero by definition, so only the existing ones (a tenth at configuration 4) get an accumulator and an add.
// Workgroup = 256 presynaptic rows x one sub-range of SNN_CSR_SUBW postsynaptic columns, 16 wavefronts of 16 rows.
// For each of its rows a wavefront keeps the first 64 entries of the row's part of the sub-range one per lane: the
// fp64 accumulator in a register for the whole launch and the column as an offset into a row of the adjoint tile
// (the few entries beyond 64 -- 3 % of the rows have any at 10 % density -- keep theirs in LDS, up to 64 per wavefront;
// the host checks that this is enough, else the matrix keeps dense accumulators).
// The time axis runs in tiles of floor(32 / B) steps whose adjoint rows P[(t, b)][512 columns] go through LDS
// (64 KB, two such buffers in turn, the next tile's loads in flight meanwhile) with the spike words of the 256 presynaptic neurons; a ballot
// gives the rows in which a neuron spiked, and each such row costs one LDS gather and one add per lane.
// Per synapse the sequence of operations is the one of k_dw_tile and of the dense contraction: per time step,
// descending, an fp32 sum over the batch elements that spiked, ascending, from zero, then one fp64 add.
#define DWC_WAVES 16
template <bool B32> // B32: the batch is 32 -- a tile is exactly one time step, the set of rows needs no shift or mask
__global__ void __launch_bounds__(64 * DWC_WAVES)
k_dw_csr(DwBatch batch, int B) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int PJ = 256, PC = SNN_CSR_SUBW, RT = 32, NWV = DWC_WAVES, RW = PJ / NWV, WPB = PJ / 64;
  constexpr int SK = RT * (PC / 4) / (64 * NWV); // staging loads (float4) per thread
  float *const Pb = (float *)smem;                       // [2][RT][PC]: two tile buffers in turn, one barrier per tile (see k_dw_tile)
  uint64_t *const Wb = (uint64_t *)(Pb + 2 * RT * PC);   // [2][WPB][RT] spike words of the tile's rows
  float *P = Pb;
  uint64_t *Wv = Wb;
  double *xacc_all = (double *)(Wb + 2 * WPB * RT);      // [NWV][64] accumulators of the entries beyond a row's 64th
  uint32_t *xoff_all = (uint32_t *)(xacc_all + NWV * 64); // [NWV][64] their column offsets
  int di = 0;
  while (di + 1 < batch.count && (int)blockIdx.x >= batch.d[di + 1].tile0) ++di;
  const DwDesc &d = batch.d[di];
  const int tile = (int)blockIdx.x - d.tile0;
  const int nsub = d.tiles_n, r = tile % nsub, j0 = (tile / nsub) * PJ, n0 = r * PC;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  double *xacc = xacc_all + 64 * wave;
  uint32_t *xoff = xoff_all + 64 * wave;
  const int t0 = d.t0, t1 = d.t1, t_base = d.t_base;
  const int TS = RT / B; // time steps per tile (B <= 32)
  const int jw = j0 + RW * wave;
  const int wsel = (RW * wave) >> 6, bitbase = (RW * wave) & 63;
  // the wavefront's synapses: entry `lane` of every row's part of the sub-range
  double acc[RW];
  uint32_t offs[RW / 2]; // byte offsets of the entries' columns inside a row of the tile, two rows per register
  auto entries = [&](int i, uint32_t &e0, uint32_t &n) { // first entry and number of entries of row jw + i here
    e0 = 0u;
    uint32_t e1 = 0u;
    if (jw + i < d.n_pre) {
      e0 = d.csr_sub[(size_t)(jw + i) * (nsub + 1) + r];
      e1 = d.csr_sub[(size_t)(jw + i) * (nsub + 1) + r + 1];
    }
    e0 = __builtin_amdgcn_readfirstlane(e0);
    n = __builtin_amdgcn_readfirstlane(e1) - e0;
  };
  // entries beyond the 64th of row i: their number (wavefront-uniform, a byte each); they sit one row after the
  // other in xacc / xoff
  uint32_t xpack[RW / 4] = {};
  auto xn_of = [&](int i) { return (xpack[i >> 2] >> (8 * (i & 3))) & 0xFFu; };
  uint32_t xtot = 0u, xmask = 0u; // xmask: bit i = row i has such entries (3 % of the rows at 10 % density)
#pragma unroll
  for (int i = 0; i < RW; ++i) {
    uint32_t e0, n;
    entries(i, e0, n);
    const bool has = (uint32_t)lane < n;
    const uint32_t o = has ? ((uint32_t)d.csr_col[e0 + lane] - (uint32_t)n0) * 4u : 0u; // < 2048
    if (i & 1) offs[i >> 1] |= o << 16;
    else offs[i >> 1] = o;
    acc[i] = has ? d.acc[e0 + lane] : 0.0;
    const uint32_t xn = n > 64u ? n - 64u : 0u;
    xpack[i >> 2] |= xn << (8 * (i & 3));
    if (xn) xmask |= 1u << i;
    if ((uint32_t)lane < xn) { // (the host has checked: at most 64 per row and per wavefront)
      xacc[xtot + lane] = d.acc[e0 + 64 + lane];
      xoff[xtot + lane] = ((uint32_t)d.csr_col[e0 + 64 + lane] - (uint32_t)n0) * 4u;
    }
    xtot += xn;
  }
  // staging of a tile: 128 threads cover one row's 512 columns; thread -> SK x (row, 4 columns)
  const int c4 = 4 * (tid & 127), srow = tid >> 7;
  const bool al = ((d.post_off + n0) & 3) == 0 && (d.post_stride & 3) == 0 && (d.slot_stride & 3) == 0 &&
                  (((uintptr_t)d.post) & 15) == 0 && n0 + PC <= d.n_post;
  float4 stg[SK];
  auto tile_load = [&](int t_hi, int nts) {
#pragma unroll
    for (int k = 0; k < SK; ++k) {
      const int rr = 8 * k + srow, ts = rr / B, b = rr - ts * B; // row rr of the tile: step t_hi - ts, batch element b
      const bool ok = ts < nts;
      const float *prow = d.post + (size_t)(t_hi - (ok ? ts : 0) - t_base - 1) * d.slot_stride + d.post_off +
                          (size_t)(ok ? b : 0) * d.post_stride + n0;
      float4 v;
      if (al) {
        v = *reinterpret_cast<const float4 *>(prow + c4);
      } else {
        v.x = n0 + c4 + 0 < d.n_post ? prow[c4 + 0] : 0.0f;
        v.y = n0 + c4 + 1 < d.n_post ? prow[c4 + 1] : 0.0f;
        v.z = n0 + c4 + 2 < d.n_post ? prow[c4 + 2] : 0.0f;
        v.w = n0 + c4 + 3 < d.n_post ? prow[c4 + 3] : 0.0f;
      }
      stg[k] = ok ? v : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
  };
  auto tile_store = [&](int t_hi, int nts) {
#pragma unroll
    for (int k = 0; k < SK; ++k) *reinterpret_cast<float4 *>(P + (size_t)(8 * k + srow) * PC + c4) = stg[k];
    if (tid < WPB * RT) { // spike words of the tile's rows for presynaptic neurons j0 .. j0 + 255
      const int rr = tid & (RT - 1), ws = tid / RT, ts = rr / B, b = rr - ts * B;
      uint64_t wv = 0ull;
      if (ts < nts && (j0 >> 6) + ws < d.pre_words) {
        const int tt = t_hi - ts - d.lag;
        wv = d.pre_mask[((size_t)(d.pre_ring > 0 ? tt % d.pre_ring : tt) * B + b) * d.pre_words + (j0 >> 6) + ws];
      }
      Wv[ws * RT + rr] = wv;
    }
  };
  const uint32_t bmask = B >= 32 ? ~0u : ((1u << B) - 1u);
  int t_hi = t1;
  tile_load(t_hi, t_hi - t0 < TS ? t_hi - t0 : TS);
  for (int it = 0; t_hi > t0; ++it) {
    const int nts = t_hi - t0 < TS ? t_hi - t0 : TS;
    P = Pb + (it & 1) * RT * PC;
    Wv = Wb + (it & 1) * WPB * RT;
    tile_store(t_hi, nts);
    __syncthreads();
    const int t_next = t_hi - nts;
    if (t_next > t0) tile_load(t_next, t_next - t0 < TS ? t_next - t0 : TS); // in flight during the adds below
    const uint64_t wv = lane < RT ? Wv[wsel * RT + lane] : 0ull;
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      const uint32_t m = (uint32_t)__ballot((wv >> (bitbase + i)) & 1ull); // rows of the tile in which neuron jw + i spiked
      if (m == 0u) continue;
      const uint32_t o = (i & 1) ? offs[i >> 1] >> 16 : offs[i >> 1] & 0xFFFFu;
      for (int ts = 0; ts < (B32 ? 1 : nts); ++ts) {
        uint32_t mt = B32 ? m : (m >> (ts * B)) & bmask;
        if (mt == 0u) continue;
        const unsigned char *Pts = reinterpret_cast<const unsigned char *>(P) + (size_t)ts * B * PC * sizeof(float) + o;
        const int k0 = (int)__builtin_ctz(mt); // the first row starts the sum (see k_dw_tile)
        asm("s_bitset0_b32 %0, %1" : "+s"(mt) : "s"(k0));
        float part = *reinterpret_cast<const float *>(Pts + (size_t)k0 * PC * sizeof(float));
        while (mt) {
          const int k = (int)__builtin_ctz(mt);
          asm("s_bitset0_b32 %0, %1" : "+s"(mt) : "s"(k)); // mt &= ~(1 << k) as one scalar instruction
          part = part + *reinterpret_cast<const float *>(Pts + (size_t)k * PC * sizeof(float));
        }
        acc[i] = acc[i] + (double)part;
      }
      if ((xmask >> i) & 1u) { // the row's entries beyond the 64th: the same walk, accumulators in LDS
        const uint32_t xn = xn_of(i);
        uint32_t xb = 0u; // they sit behind those of the rows before it
#pragma unroll
        for (int k = 0; k < i; ++k) xb += xn_of(k);
        const bool mine = (uint32_t)lane < xn;
        const uint32_t ox = mine ? xoff[xb + lane] : 0u;
        for (int ts = 0; ts < (B32 ? 1 : nts); ++ts) {
          uint32_t mt = B32 ? m : (m >> (ts * B)) & bmask;
          if (mt == 0u) continue;
          float part = 0.0f;
          const unsigned char *Pts = reinterpret_cast<const unsigned char *>(P) + (size_t)ts * B * PC * sizeof(float) + ox;
          while (mt) {
            const int k = (int)__builtin_ctz(mt);
            asm("s_bitset0_b32 %0, %1" : "+s"(mt) : "s"(k));
            part = part + *reinterpret_cast<const float *>(Pts + (size_t)k * PC * sizeof(float));
          }
          if (mine) xacc[xb + lane] = xacc[xb + lane] + (double)part;
        }
      }
    }
    t_hi = t_next;
  }
  uint32_t xbase = 0u;
#pragma unroll
  for (int i = 0; i < RW; ++i) {
    uint32_t e0, n;
    entries(i, e0, n);
    const uint32_t xn = xn_of(i);
    if ((uint32_t)lane < n) d.acc[e0 + lane] = acc[i];
    if ((uint32_t)lane < xn) d.acc[e0 + 64 + lane] = xacc[xbase + lane];
    xbase += xn;
  }
}

// Gradient of a masked matrix from the accumulators of its existing synapses: one workgroup per presynaptic row.
__global__ void __launch_bounds__(256)
k_finish_grad_csr(const double *__restrict__ acc, const uint32_t *__restrict__ sub, const uint16_t *__restrict__ col, int N,
                  int nsub, float *__restrict__ dW) {
  const int j = blockIdx.x;
  float *row = dW + (size_t)j * N;
  for (int n = threadIdx.x; n < N; n += 256) row[n] = 0.0f;
  __syncthreads();
  const uint32_t e0 = sub[(size_t)j * (nsub + 1)], e1 = sub[(size_t)j * (nsub + 1) + nsub];
  for (uint32_t e = e0 + threadIdx.x; e < e1; e += 256) row[col[e]] = (float)acc[e];
}

// One stage of the layer-pipelined backward pass takes two launches.
// k_bwd_stage (512 threads), workgroup ranges in this order:
//   [0, n_adj)        adjoint recurrences of the stage (job = block / B, batch element = block % B)
//   [.., + du.n)      du_t of the NEXT tile (a scan over its steps; needs only the carried du)
//   [.., + n_dw)      weight-gradient contraction of what the previous stage finished
//   the rest          (optional) recompute work for later chunks, see k_bwd_inter
// All of them are independent of each other, and the recurrences (a chain of dependent steps on a few dozen
// compute units) leave most of the chip idle: the contraction fills it.  The register footprint of the
// recurrence part keeps two workgroups from sharing a compute unit, so nothing competes with a recurrence
// for issue slots.
template <int KH, int H, int R>
__global__ void __launch_bounds__(512)
k_bwd_stage(NetDev net, AdjJobs jobs, float *__restrict__ carry, DwBatch batch, DuJob du, const float *__restrict__ g,
            PreJobs pre, int n_adj_blocks, int n_dw_blocks) {
  extern __shared__ __align__(16) unsigned char smem[];
  int v = (int)blockIdx.x; // every branch below is uniform per workgroup
  if (v < n_adj_blocks) {
    adj_rec_rs_body<KH, H, R>(net, jobs.j[v / net.B], carry, v % net.B);
    return;
  }
  v -= n_adj_blocks;
  if (v < du.n) {
    du_scan_body(g, carry, du.dubuf, net.B, net.n_out, net.SN, du.t0, du.t1, du.t_base, net.beta, du.carry_init, v);
    return;
  }
  v -= du.n;
  if (v < n_dw_blocks) {
    dw_mfma_body<1, 2>(batch, net.B, v, smem);
    return;
  }
  v -= n_dw_blocks;
  // recompute work for later chunks, on the compute units the contraction has left
  const int n_cur = pre.cur_gx * pre.cur.count;
  if (v < n_cur) {
    currents_mfma_body<8>(net, pre.cur.j[v / pre.cur_gx], pre.ws, pre.lcap, v % pre.cur_gx, smem);
    return;
  }
  v -= n_cur;
  if (v < pre.n_scan)
    scan_body(net, pre.t0, pre.t1, pre.state_in, pre.buf, pre.t_base, pre.slot_stride, pre.store_all, pre.state_out, v);
}

// k_bwd_inter (256 threads) runs between two stage launches, workgroup ranges in this order:
//   the inter-layer products that the next stage's recurrences need (of the layers just finished, and the top
//   layer's product of the next tile), then the recompute work that rides along: part 1 (currents) of the chunk
//   two stages ahead, part 2 (scan) of the chunk one stage ahead.  All short and independent of each other.
__global__ void __launch_bounds__(256)
k_bwd_inter(NetDev net, InterJobs ij) {
  extern __shared__ __align__(16) unsigned char smem[];
  int v = (int)blockIdx.x; // every branch below is uniform per workgroup
  for (int q = 0; q < ij.n_gemm; ++q) {
    const GemmJob &gj = ij.g[q];
    if (v < gj.n_blocks) {
      if (gj.kind == 0) up_gemm16_body(gj.A, gj.lda, gj.W, gj.K, gj.N, gj.C, gj.N, gj.M, v);
      else up_gemm_body<2, 2>(gj.A, gj.lda, gj.W, gj.K, gj.N, gj.C, gj.N, gj.M, v % gj.tiles_m, v / gj.tiles_m);
      return;
    }
    v -= gj.n_blocks;
  }
  const PreJobs &pre = ij.pre;
  const int n_cur = pre.cur_gx * pre.cur.count;
  if (v < n_cur) {
    currents_mfma_body<4>(net, pre.cur.j[v / pre.cur_gx], pre.ws, pre.lcap, v % pre.cur_gx, smem);
    return;
  }
  v -= n_cur;
  if (v < pre.n_scan)
    scan_body(net, pre.t0, pre.t1, pre.state_in, pre.buf, pre.t_base, pre.slot_stride, pre.store_all, pre.state_out, v);
}

// ------------------------------------------------------------------------------------------
// small utilities
// ------------------------------------------------------------------------------------------
__global__ void k_transpose(const float *__restrict__ src, float *__restrict__ dst, int rows, int cols) {
  __shared__ float tile[32][33];
  int x = blockIdx.x * 32 + threadIdx.x, y = blockIdx.y * 32 + threadIdx.y;
  for (int i = 0; i < 32; i += 8)
    if (x < cols && y + i < rows) tile[threadIdx.y + i][threadIdx.x] = src[(size_t)(y + i) * cols + x];
  __syncthreads();
  x = blockIdx.y * 32 + threadIdx.x;
  y = blockIdx.x * 32 + threadIdx.y;
  for (int i = 0; i < 32; i += 8)
    if (x < rows && y + i < cols) dst[(size_t)(y + i) * rows + x] = tile[threadIdx.x][threadIdx.y + i];
}

// fp64 accumulator -> fp32 gradient; a masked matrix has a gradient only where a synapse exists
__global__ void k_finish_grad(const double *__restrict__ acc, const uint8_t *__restrict__ mask, float *__restrict__ dW,
                              size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dW[i] = (mask && !mask[i]) ? 0.0f : (float)acc[i];
}

__global__ void k_unpack(const uint64_t *__restrict__ mask, int words, int N, size_t TB, uint8_t *__restrict__ dst) {
  // mask rows 1..T -> dst[T][B][N]
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= TB * (size_t)N) return;
  const size_t tb = i / N;
  const int n = (int)(i % N);
  const uint64_t w = mask[tb * words + (n >> 6)];
  dst[i] = (uint8_t)((w >> (n & 63)) & 1ull);
}

__global__ void k_count(const uint64_t *__restrict__ mask, size_t n_words, unsigned long long *count) {
  unsigned long long c = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += (size_t)gridDim.x * blockDim.x)
    c += __popcll(mask[i]);
  for (int s = 32; s > 0; s >>= 1) c += __shfl_down(c, s);
  if (lane_id() == 0 && c) atomicAdd(count, c); // integer atomic: order-independent
}

// plain streaming copy of known size (reference for scaling hardware byte counters)
__global__ void __launch_bounds__(256) k_copy(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

__global__ void k_zero(uint32_t *p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
static LaunchCfg forward_cfg(const NetDev &net) {
  int nmax = 64;
  for (int l = 0; l < net.L; ++l) nmax = net.N[l] > nmax ? net.N[l] : nmax;
  LaunchCfg c;
  c.npt = 1;
  while (((nmax + c.npt - 1) / c.npt + 63) / 64 * 64 > 512 && c.npt < 16) c.npt *= 2;
  c.nt_neuron = ((nmax + c.npt - 1) / c.npt + 63) / 64 * 64;
  int wdmax = 1;
  size_t lists = (size_t)((net.n_in + 7) & ~7);
  for (int l = 0; l < net.L; ++l) {
    wdmax = net.Wd[l + 1] > wdmax ? net.Wd[l + 1] : wdmax;
    lists += (size_t)((net.N[l] + 7) & ~7);
  }
  c.lds_bytes = (size_t)wdmax * 8 + 16 + lists * 2;
  return c;
}

static size_t adjoint_lds(const NetDev &net, int nt) {
  int nmax = 0;
  for (int l = 0; l < net.L; ++l) nmax = net.N[l] > nmax ? net.N[l] : nmax;
  return nmax <= 256 ? 0 : ((size_t)2 * nmax + nt) * sizeof(float);
}

static size_t seq_gather_lds(const NetDev &net) {
  size_t mx = 0;
  for (int l = 0; l < net.L; ++l) {
    const size_t b = (size_t)net.Wd[l + 1] * 8 + 16 + (size_t)(((net.N[l] + 7) & ~7) + 8) * 4; // words, count, row offsets
    mx = b > mx ? b : mx;
  }
  return mx;
}

static size_t currents_lds(const NetDev &net) {
  size_t mx = 0;
  for (int l = 0; l < net.L; ++l) {
    const int P = l == 0 ? net.n_in : net.N[l - 1];
    const size_t b = (size_t)(net.Wd[l] + net.Wd[l + 1]) * 8 + 16 + (size_t)(((P + 7) & ~7) + ((net.N[l] + 7) & ~7)) * 2;
    mx = b > mx ? b : mx;
  }
  return mx;
}

bool snn_kernel_shape_ok(const NetDev &net, char *why, size_t why_len) {
  const LaunchCfg c = forward_cfg(net);
  const size_t lds_max = 64 * 1024; // per-workgroup limit without opting in to more
  if (c.nt_neuron > 512 || c.nt_neuron * c.npt < 1) { snprintf(why, why_len, "layer too wide for the forward kernel"); return false; }
  for (int l = 0; l < net.L; ++l)
    if ((net.N[l] + c.npt - 1) / c.npt > c.nt_neuron) { snprintf(why, why_len, "layer too wide for the forward kernel (max %d neurons)", 512 * 16); return false; }
  if (net.Wd[0] > WAVE) { snprintf(why, why_len, "n_in > 4096 not supported"); return false; }
  if (seq_gather_lds(net) > lds_max) { snprintf(why, why_len, "forward kernel needs %zu B of LDS (> %zu)", seq_gather_lds(net), lds_max); return false; }
  if (currents_lds(net) > lds_max) { snprintf(why, why_len, "recompute kernel needs %zu B of LDS (> %zu)", currents_lds(net), lds_max); return false; }
  // the streamed adjoint kernel may opt in to the full 160 KB of LDS of a gfx950 compute unit
  if (adjoint_lds(net, 1024) > 160 * 1024) { snprintf(why, why_len, "adjoint kernel needs %zu B of LDS (> %zu)", adjoint_lds(net, 1024), lds_max); return false; }
  return true;
}

hipError_t launch_pack_inputs(const uint8_t *in_spikes, uint64_t *mask0, int T, int B, int n_in, int Wd0,
                              hipStream_t s) {
  if (T <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_pack_inputs, dim3((unsigned)((size_t)T * B)), dim3(WAVE), 0, s, in_spikes, mask0, B, n_in, Wd0);
  return hipGetLastError();
}

template <int NPT>
static void launch_currents_t(const NetDev &net, dim3 grid, int nt, size_t lds, const CurJobs &jobs, hipStream_t s) {
  hipLaunchKernelGGL((k_currents<NPT>), grid, dim3(nt), lds, s, net, jobs);
}
// SNN_CURRENTS=gather selects the event-by-event gather kernel for every current (the default runs
// the feed-forward and recurrent currents on the matrix cores and only the narrow readout as a gather); the
// context turns it into net.sel_currents.
static bool currents_use_mfma(const NetDev &net) { return net.sel_currents != 1; }
static hipError_t launch_currents_gather(const NetDev &net, const CurJobs &jobs, hipStream_t s);
static void currents_geometry(const NetDev &net, const CurJobs &jobs, unsigned *gx, int *ws, int *lcap, int nwv);
static size_t currents_lds(int nwv, int ws, int lcap) {
  return (size_t)nwv * 16 * ws * sizeof(uint64_t) + (size_t)nwv * lcap * sizeof(uint32_t);
}
#define SNN_LDS_PER_CU (160 * 1024)
// Matrices of a job: presynaptic widths and the larger product with the postsynaptic width, in bytes.
static void currents_job_shape(const NetDev &net, const CurJob &j, int *pmax, size_t *wbytes) {
  const bool ro = j.mode == 2;
  const int l = ro ? net.L - 1 : j.lsel, N = ro ? net.n_out : net.N[l];
  int p = ro ? net.N[l] : (l == 0 ? net.n_in : net.N[l - 1]);
  if (j.mode == 0 && N > p) p = N;
  *pmax = p;
  *wbytes = (size_t)p * N * sizeof(float);
}
// Which kernel runs a job: 0 list version, 1 dense version, 2 event-by-event gather.  Weights that fit the L2
// many times over: always the list version.  Weights far beyond it: what the context chose from the firing rates
// of its last step (the gather below about 3.5 % presynaptic activity, the dense version above, and before any
// rate is known).  SNN_CURRENTS=dense / mfma / gather forces one of them for every job.
#define SNN_DENSE_MB 4
static int currents_job_kernel(const NetDev &net, const CurJob &j) {
  int p;
  size_t wb;
  currents_job_shape(net, j, &p, &wb);
  const bool dense_ok = wb < ((size_t)1 << 32); // one buffer descriptor
  if (net.sel_currents == 3) return dense_ok ? 1 : 0;
  if (net.sel_currents == 2) return 0;
  if (wb < ((size_t)32 << 20) || j.mode == 2) return 0;
  const int pol = net.cur_pol[j.mode == 0 ? 1 : 0][j.lsel];
  if (pol == 1) return 2;
  return dense_ok ? 1 : 0;
}
static hipError_t launch_currents_dense(const NetDev &net, const CurJobs &jobs, hipStream_t s) {
  unsigned gx = 0;
  int ws = 1;
  for (int i = 0; i < jobs.count; ++i) {
    const CurJob &j = jobs.j[i];
    int p;
    size_t wb;
    currents_job_shape(net, j, &p, &wb);
    const int N = j.mode == 2 ? net.n_out : net.N[j.lsel], rows = j.nsteps * net.B;
    const unsigned g = (unsigned)(((rows + 16 * SNN_DENSE_MB - 1) / (16 * SNN_DENSE_MB)) * ((N + 255) >> 8));
    gx = g > gx ? g : gx;
    const int w1 = ((p + 63) >> 6) | 1;
    ws = w1 > ws ? w1 : ws;
  }
  const size_t lds = 0; // the operand buffers are static
  const bool rc = jobs.j[0].mode == 0 || jobs.j[0].mode == 3;
  if (rc) hipLaunchKernelGGL((k_currents_dense<SNN_DENSE_MB, 1>), dim3(gx, jobs.count), dim3(256), lds, s, net, jobs, ws);
  else hipLaunchKernelGGL((k_currents_dense<SNN_DENSE_MB, 0>), dim3(gx, jobs.count), dim3(256), lds, s, net, jobs, ws);
  return hipGetLastError();
}
static hipError_t launch_currents_csr(const NetDev &net, const CurJobs &jobs, hipStream_t s) {
  if (jobs.count <= 0) return hipSuccess;
  unsigned gx = 0;
  size_t lds = 0;
  for (int i = 0; i < jobs.count; ++i) {
    const int l = jobs.j[i].lsel, N = net.N[l], nsub = (N + SNN_CSR_SUBW - 1) / SNN_CSR_SUBW;
    const unsigned g = (unsigned)((size_t)jobs.j[i].nsteps * net.B * ((nsub + 3) >> 2));
    gx = g > gx ? g : gx;
    const size_t b = (size_t)net.Wd[l + 1] * 8 + 16 + (size_t)4 * SNN_CSR_SUBW * 4 + (size_t)((N + 7) & ~7) * 2 + (size_t)4 * 64 * 4;
    lds = b > lds ? b : lds;
  }
  hipLaunchKernelGGL(k_currents_csr, dim3(gx, jobs.count), dim3(256), lds, s, net, jobs);
  return hipGetLastError();
}
static hipError_t launch_currents_plain(const NetDev &net, const CurJobs &jobs, hipStream_t s);
// Does the recurrent part of a recompute job walk compressed rows?  Like the event-by-event gather it pays per
// presynaptic spike (with a tenth of the bytes per spike at 10 % density), the dense matrix-core version per
// presynaptic neuron: it takes over where the context's firing-rate policy picks the gather, i.e. for matrices far
// beyond the L2 at low activity.  net.sel_csr == 2 forces it wherever compressed rows exist.
static bool currents_job_csr(const NetDev &net, const CurJob &j) {
  const int l = j.lsel;
  if (!net.csr_sub[l]) return false;
  if (net.sel_csr == 2) return true;
  return (size_t)net.N[l] * net.N[l] * sizeof(float) >= ((size_t)32 << 20) && (net.cur_pol[1][l] == 1 || net.cur_pol[1][l] == 3);
}
// Recompute jobs (mode 0) of layers whose recurrent matrix has compressed rows are split: the feed-forward part
// goes through the usual kernels (mode 3), the recurrent part through k_currents_csr behind them.
static hipError_t launch_currents(const NetDev &net, const CurJobs &jobs, hipStream_t s) {
  CurJobs plain = jobs, cs{};
  for (int i = 0; i < plain.count; ++i)
    if (plain.j[i].mode == 0 && plain.j[i].nsteps > 0 && currents_job_csr(net, plain.j[i])) {
      cs.j[cs.count++] = plain.j[i];
      plain.j[i].mode = 3;
    }
  const hipError_t e = launch_currents_plain(net, plain, s);
  if (e != hipSuccess) return e;
  return launch_currents_csr(net, cs, s);
}
static hipError_t launch_currents_plain(const NetDev &net, const CurJobs &jobs, hipStream_t s) {
  if (!currents_use_mfma(net)) return launch_currents_gather(net, jobs, s);
  CurJobs mf{}, dn{}, ga{};
  for (int i = 0; i < jobs.count; ++i)
    if (jobs.j[i].nsteps > 0) {
      const int k = currents_job_kernel(net, jobs.j[i]);
      CurJobs &dst = k == 1 ? dn : k == 2 ? ga : mf;
      dst.j[dst.count++] = jobs.j[i];
    }
  if (dn.count) {
    const hipError_t e = launch_currents_dense(net, dn, s);
    if (e != hipSuccess) return e;
  }
  if (ga.count) {
    const hipError_t e = launch_currents_gather(net, ga, s);
    if (e != hipSuccess) return e;
  }
  if (!mf.count) return hipSuccess;
  unsigned gx;
  int ws, lcap;
  currents_geometry(net, mf, &gx, &ws, &lcap, 4);
  // 8 KB of static LDS (the combine buffer of recompute mode) beside the dynamic part
  const int nwv = currents_lds(4, ws, lcap) + 8192 <= SNN_LDS_PER_CU ? 4 : 2;
  if (nwv == 2) currents_geometry(net, mf, &gx, &ws, &lcap, 2);
  const size_t lds = currents_lds(nwv, ws, lcap);
  if (lds + 8192 > SNN_LDS_PER_CU) return launch_currents_gather(net, jobs, s); // same sums, event by event
  if (lds > 48 * 1024) {
    const hipError_t ea = hipFuncSetAttribute(nwv == 4 ? reinterpret_cast<const void *>(k_currents_mfma<4>)
                                                       : reinterpret_cast<const void *>(k_currents_mfma<2>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (ea != hipSuccess) return ea;
  }
  if (nwv == 4) hipLaunchKernelGGL(k_currents_mfma<4>, dim3(gx, mf.count), dim3(256), lds, s, net, mf, ws, lcap);
  else hipLaunchKernelGGL(k_currents_mfma<2>, dim3(gx, mf.count), dim3(128), lds, s, net, mf, ws, lcap);
  return hipGetLastError();
}
static hipError_t launch_currents_gather(const NetDev &net, const CurJobs &jobs, hipStream_t s) {
  if (jobs.count <= 0) return hipSuccess;
  const LaunchCfg c = forward_cfg(net);
  int max_steps = 0;
  for (int i = 0; i < jobs.count; ++i) max_steps = jobs.j[i].nsteps > max_steps ? jobs.j[i].nsteps : max_steps;
  if (max_steps <= 0) return hipSuccess;
  const dim3 grid((unsigned)((size_t)max_steps * net.B), jobs.count);
  const size_t lds = currents_lds(net);
  switch (c.npt) {
    case 1: launch_currents_t<1>(net, grid, c.nt_neuron, lds, jobs, s); break;
    case 2: launch_currents_t<2>(net, grid, c.nt_neuron, lds, jobs, s); break;
    case 4: launch_currents_t<4>(net, grid, c.nt_neuron, lds, jobs, s); break;
    case 8: launch_currents_t<8>(net, grid, c.nt_neuron, lds, jobs, s); break;
    case 16: launch_currents_t<16>(net, grid, c.nt_neuron, lds, jobs, s); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Currents jobs of a launch: virtual grid width and LDS geometry of the matrix-core current kernel.
static void currents_geometry(const NetDev &net, const CurJobs &jobs, unsigned *gx, int *ws, int *lcap, int nwv = 4) {
  unsigned g = 0;
  int pmax = 1;
  for (int i = 0; i < jobs.count; ++i) {
    const CurJob &j = jobs.j[i];
    const int rows = j.nsteps * net.B, per = 16 * (j.mode == 0 ? nwv / 2 : nwv);
    const int ncols = j.mode == 2 ? net.n_out : net.N[j.lsel];
    const unsigned n = (unsigned)((rows + per - 1) / per) * (unsigned)((ncols + 63) / 64);
    g = n > g ? n : g;
    if (j.mode == 2) { pmax = net.N[net.L - 1] > pmax ? net.N[net.L - 1] : pmax; continue; }
    const int l = j.lsel, p_in = l == 0 ? net.n_in : net.N[l - 1];
    pmax = p_in > pmax ? p_in : pmax;
    if (j.mode == 0) pmax = net.N[l] > pmax ? net.N[l] : pmax;
  }
  *gx = g;
  *ws = ((pmax + 63) / 64 + 1) | 1;
  *lcap = ((pmax + 31) & ~31) + 32;
}

// does the matrix-core current kernel of a fused forward stage fit the LDS beside the sequential part?
static bool fwd_stage_fits(const NetDev &net) {
  int pmax = net.n_in;
  for (int l = 0; l < net.L; ++l) pmax = net.N[l] > pmax ? net.N[l] : pmax;
  const int ws = ((pmax + 63) / 64 + 1) | 1, lcap = ((pmax + 31) & ~31) + 32;
  return currents_lds(4, ws, lcap) + 17 * 1024 <= SNN_LDS_PER_CU;
}

static hipError_t launch_fwd_stage(const NetDev &net, const SeqJobs &sj, float *state, const StoreSpec &st,
                                   const CurJobs &cj, RoJob ro, double *readout, hipStream_t s) {
  for (int i = 0; i < cj.count; ++i)
    if (cj.j[i].nsteps <= 0) return hipErrorInvalidValue;
  unsigned gx;
  int ws, lcap;
  currents_geometry(net, cj, &gx, &ws, &lcap);
  // the sequential part holds ~8 KB of static LDS, the current part 8 KB; asking for 72 KB more puts the
  // total above half of a compute unit's 160 KB, so every workgroup gets a compute unit of its own
  size_t lds = currents_lds(4, ws, lcap);
  if (lds + 17 * 1024 > SNN_LDS_PER_CU) return hipErrorInvalidValue; // the caller checks fwd_stage_fits first
  if (lds < 72 * 1024) lds = 72 * 1024;
  const hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void *>(k_fwd_stage),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (ea != hipSuccess) return ea;
  const int n_seq = net.B * sj.count;
  if (ro.n != 0) {
    if (ro.nsteps <= 0 || !ro.iout) return hipErrorInvalidValue;
    ro.n = (net.B * net.n_out + 255) / 256;
  }
  hipLaunchKernelGGL(k_fwd_stage, dim3(n_seq + ro.n + gx * cj.count), dim3(256), lds, s, net, sj, state, st, cj, ws, lcap,
                     n_seq, (int)gx, ro, readout);
  return hipGetLastError();
}

// Forward pass over the tiles bounds[0] < bounds[1] < ... < bounds[n_tiles] (each at most
// SNN_FWD_TILE steps).  The layers are pipelined two stages apart: the feed-forward currents of layer l for
// tile k are computed in stage k + 2l (the layer below finished that tile in stage k + 2l - 1), its
// sequential part runs in stage k + 2l + 1, the readout currents of tile k in stage k + 2L.  Everything a
// stage does is independent of everything else in it, so a stage is one launch (k_fwd_stage) when all
// layers are register-stationary, and otherwise one launch per kernel flavour.  The current tiles are
// double-buffered by tile parity.
static size_t seq_gather_lds(const NetDev &net);
template <int NPT>
static int seq_sl_resident(int device, size_t lds, int threads) {
  static int cached[16][9] = {}; // per device and block size / 64
  if (device < 0 || device >= 16 || threads < 64 || threads > 512) return 0;
  int &c = cached[device][threads / 64];
  if (!c) {
    hipDeviceProp_t prop;
    int per_cu = 0;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_layer_seq_gather_sl<NPT>, threads, lds) != hipSuccess) return 0;
    c = per_cu * prop.multiProcessorCount;
  }
  return c;
}
// Slices per batch element for the sequential part of layers wider than 256 neurons (1: one workgroup per batch
// element).  All workgroups of a launch must be resident at once (they wait for each other), every wide layer may
// have a job in the same launch, a slice is whole spike words and a whole number of rounds of its block, and the
// exchange buffer of the chip-wide kernels must hold the entries of every (job, batch element).  Used from 2048
// neurons (a single compute unit's L1 then bounds the step).  SNN_SEQ_SLICES=1 turns it off, =2, 4, 8 asks for
// that many at any width.
static int seq_slices(const NetDev &net, const SeqJobs &ga, const WsArgs *ws, int *npt, int *threads) {
  if (!ws || !ws->xg || ga.count < 1) return 1;
  const int forced = net.sel_slices;
  if (forced == 1) return 1;
  const int N = net.N[ga.j[0].l], Wd = net.Wd[ga.j[0].l + 1];
  int n_wide = 0;
  for (int l = 0; l < net.L; ++l) n_wide += net.N[l] > 256;
  for (int i = 0; i < ga.count; ++i)
    if (net.N[ga.j[i].l] != N) return 1;
  // narrower layers: measured slower with slices at 512 and 1024 neurons (a wavefront walks every active row whatever
  // the number of columns its workgroup owns, and that walk, not the compute unit's L1, is what takes the time)
  if (!forced && N < 2048) return 1;
  if ((size_t)n_wide * net.B * 4 * Wd * sizeof(uint64_t) > (size_t)ws->xg_stride * SNN_MAXL * sizeof(float)) return 1;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return 1;
  const size_t lds = seq_gather_lds(net);
  for (int S = 8; S >= 2; S /= 2) {
    if (forced && S != forced) continue;
    if (N % (64 * S) != 0) continue;
    const int Ns = N / S;
    int p = 1;
    while (Ns / p > 512) p *= 2;
    if (p > 16 || Ns % (64 * p) != 0) continue;
    const int th = Ns / p;
    int resident = 0;
    switch (p) {
      case 1: resident = seq_sl_resident<1>(device, lds, th); break;
      case 2: resident = seq_sl_resident<2>(device, lds, th); break;
      case 4: resident = seq_sl_resident<4>(device, lds, th); break;
      case 8: resident = seq_sl_resident<8>(device, lds, th); break;
      case 16: resident = seq_sl_resident<16>(device, lds, th); break;
      default: continue;
    }
    if (S * net.B * n_wide > resident) continue;
    *npt = p;
    *threads = th;
    return S;
  }
  return 1;
}

// The compressed-row version of the sliced sequential part: every job's layer has compressed rows, the same width
// (a multiple of 4 SNN_CSR_SUBW), all workgroups of the launch are resident at once and the exchange buffer holds
// the entries of every (job, batch element).  Returns the slices per batch element, 0 if it cannot run.
static size_t seq_csr_lds(int N, int Wd) {
  return (size_t)Wd * 8 + 16 + (size_t)4 * SNN_CSR_SUBW * 4 + (size_t)((N + 7) & ~7) * 2 + (size_t)4 * 64 * 4;
}
static int seq_csr_resident(int device, size_t lds) {
  static int cached[16] = {};
  if (device < 0 || device >= 16) return 0;
  if (!cached[device]) {
    hipDeviceProp_t prop;
    int per_cu = 0;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_layer_seq_csr_sl, 256, lds) != hipSuccess) return 0;
    cached[device] = per_cu * prop.multiProcessorCount;
  }
  return cached[device];
}
// The fused stage launch (k_fwd_stage_csr): workgroups per compute unit, queried once per device, outside any capture.
#define SNN_FWD_STAGE_CSR_LDS ((size_t)2 * 16 * SNN_DENSE_MB_ * SNN_DENSE_AP * sizeof(float))
static int fwd_stage_csr_per_cu(int device, int *n_cu) {
  static int cached[16] = {}, cus[16] = {};
  if (device < 0 || device >= 16) return 0;
  if (!cached[device]) {
    hipDeviceProp_t prop;
    int per_cu = 0;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
    const size_t a = seq_csr_lds(8192, 128), lds = a > SNN_FWD_STAGE_CSR_LDS ? a : SNN_FWD_STAGE_CSR_LDS;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_fwd_stage_csr, 256, lds) != hipSuccess) return 0;
    cached[device] = per_cu > 0 ? per_cu : -1;
    cus[device] = prop.multiProcessorCount;
  }
  *n_cu = cus[device];
  return cached[device] > 0 ? cached[device] : 0;
}
static int seq_csr_slices(const NetDev &net, const SeqJobs &ga, const WsArgs *ws, bool need_rows = true) {
  if (!ws || !ws->xg || ga.count < 1 || net.sel_slices == 1) return 0;
  // The walk over compressed rows pays per presynaptic spike and per synapse that exists: it runs where the
  // context's firing-rate policy has picked the gather over compressed rows for the recompute or, at higher
  // activity, for this walk alone (cur_pol 1, 3, 4), or wherever the hook asks.
  if (need_rows && net.sel_csr != 2) {
    if (net.sel_csr == 1) return 0;
    for (int i = 0; i < ga.count; ++i) {
      const int pol = net.cur_pol[1][ga.j[i].l];
      if (pol != 1 && pol != 3 && pol != 4) return 0;
    }
  }
  const int N = net.N[ga.j[0].l], Wd = net.Wd[ga.j[0].l + 1];
  if (N % (4 * SNN_CSR_SUBW) != 0) return 0;
  int n_wide = 0;
  for (int l = 0; l < net.L; ++l) n_wide += net.N[l] > 256;
  for (int i = 0; i < ga.count; ++i)
    if (net.N[ga.j[i].l] != N || (need_rows && !net.csr_sub[ga.j[i].l])) return 0;
  if ((size_t)n_wide * net.B * 4 * Wd * sizeof(uint64_t) > (size_t)ws->xg_stride * SNN_MAXL * sizeof(float)) return 0;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return 0;
  // LDS of the widest layer the kernel can meet on this device (the occupancy is queried once, outside any capture)
  const int S = N / (4 * SNN_CSR_SUBW);
  if (S * net.B * n_wide > seq_csr_resident(device, seq_csr_lds(8192, 128))) return 0;
  return S;
}

hipError_t launch_forward(const NetDev &net, const int *bounds, int n_tiles, float *state, const StoreSpec &st,
                          double *readout, int readout_init, float *work, hipStream_t s, const SpanHook *hook,
                          const FwdCallbacks *cb, const WsArgs *ws) {
  if (n_tiles < 0) return hipErrorInvalidValue;
  for (int k = 0; k < n_tiles; ++k)
    if (bounds[k + 1] <= bounds[k] || bounds[k + 1] - bounds[k] > SNN_FWD_TILE) return hipErrorInvalidValue;
  auto hb = [&](int kind) { if (hook) hook->begin(hook->ctx, kind); };
  auto he = [&]() { if (hook) hook->end(hook->ctx); };
  const int B = net.B, O = net.n_out, L = net.L;
  float *iin[SNN_MAXL][2];
  for (int l = 0; l < L; ++l)
    for (int par = 0; par < 2; ++par)
      iin[l][par] = work + (size_t)SNN_FWD_TILE * B * ((size_t)par * net.SN + net.off[l]); // [tile][B][N_l]
  float *iout = work + (size_t)2 * SNN_FWD_TILE * B * net.SN;                              // [tile][B][O]
  const LaunchCfg c = forward_cfg(net);
  int nmax = 0;
  for (int l = 0; l < L; ++l) nmax = net.N[l] > nmax ? net.N[l] : nmax;
  // Layers of up to 256 neurons: the register-stationary chain (one FMA per presynaptic neuron, whatever the
  // activity) or, where the context's policy has measured a low firing rate (or the hook asks), the event-driven
  // gather over the rows of the neurons that fired.  Both give the same bits.
  auto narrow_gather = [&](int l) {
    return net.N[l] <= 256 && (net.sel_seq == 1 || (net.sel_seq == 0 && net.seq_pol[l] == 1));
  };
  bool any_narrow_gather = false;
  for (int l = 0; l < L; ++l) any_narrow_gather = any_narrow_gather || narrow_gather(l);
  const bool fuse = nmax > 128 && nmax <= 256 && currents_use_mfma(net) && fwd_stage_fits(net) && !any_narrow_gather;
  int ro_steps = 0, ro_tiles = 0;
  bool ro_first = true;
  RoJob ro_pending{};
  for (int stage = 0; stage < n_tiles + 2 * L; ++stage) {
    // ---- parallel part: feed-forward currents for the next stage's sequential parts, readout currents ----
    CurJobs cj{};
    for (int l = 0; l < L; ++l) {
      const int k = stage - 2 * l;
      if (k < 0 || k >= n_tiles) continue;
      cj.j[cj.count++] = CurJob{1, l, bounds[k], bounds[k + 1] - bounds[k], bounds[k], iin[l][k & 1], 0};
    }
    // readout currents of the tile whose last-layer spikes are complete.  Fused stages: the leaky scan over a
    // tile rides in the launch after the one that computed its currents (two tile buffers, by parity).
    // Otherwise the currents queue up in iout and the (cheap, sequential) scan runs once per SNN_RO_TILES tiles.
    const int ko = stage - 2 * L;
    const bool ro_now = ko >= 0 && ko < n_tiles;
    if (ro_now) {
      float *dst = fuse ? iout + (size_t)(ko & 1) * SNN_FWD_TILE * B * O : iout + (size_t)ro_steps * B * O;
      cj.j[cj.count++] = CurJob{2, L, bounds[ko], bounds[ko + 1] - bounds[ko], bounds[ko], dst, 0};
    }
    // ---- sequential part: every layer's current tile ----------------------------------------------
    SeqJobs rs{}, ga{};
    int nw = 64;
    for (int l = 0; l < L; ++l) {
      const int k = stage - 2 * l - 1;
      if (k < 0 || k >= n_tiles) continue;
      const SeqJob job{l, bounds[k], bounds[k + 1], bounds[k], iin[l][k & 1]};
      if (net.N[l] <= 256 && !narrow_gather(l)) { rs.j[rs.count++] = job; nw = net.N[l] > nw ? net.N[l] : nw; }
      else ga.j[ga.count++] = job;
    }
    hipError_t e = hipSuccess;
    auto scan_now = [&](const RoJob &r) { // a launch of its own
      hb(5);
      hipLaunchKernelGGL(k_readout_scan, dim3((B * O + 255) / 256), dim3(256), 0, s, r.iout, readout, B, O, r.nsteps,
                         net.beta, r.init);
      he();
    };
    if (fuse) {
      if (rs.count && cj.count && !ga.count) {
        hb(8);
        e = launch_fwd_stage(net, rs, state, st, cj, ro_pending, readout, s);
        he();
        if (e != hipSuccess) return e;
        ro_pending = RoJob{};
      } else {
        hb(5);
        e = launch_currents(net, cj, s);
        he();
        if (e != hipSuccess) return e;
        if (rs.count) {
          hb(4);
          hipLaunchKernelGGL((k_layer_seq_rs<256>), dim3(B, rs.count), dim3(256), 0, s, net, rs, state, st);
          he();
        }
        if (ro_pending.n) { scan_now(ro_pending); ro_pending = RoJob{}; }
      }
      if (ro_now) { // its currents are in flight: scan it with (or after) the next launch
        ro_pending = RoJob{1, iout + (size_t)(ko & 1) * SNN_FWD_TILE * B * O, bounds[ko + 1] - bounds[ko],
                           (ro_first && readout_init) ? 1 : 0};
        ro_first = false;
      }
    } else {
      int npt_sl = 0, th_sl = 0;
      const int S_csr = ga.count ? seq_csr_slices(net, ga, ws) : 0;
      const int S = (ga.count && !S_csr) ? seq_slices(net, ga, ws, &npt_sl, &th_sl) : 1;
      // Wide layers over compressed rows: the dense feed-forward currents for the next stage ride in the launch
      // of this stage's sequential parts (k_fwd_stage_csr) when all sequential workgroups fit beside one current
      // workgroup per compute unit; other current jobs (readout, matrices that fit the L2) go out on their own.
      CurJobs cj_fused{};
      if (S_csr && !net.no_fwd_fuse && currents_use_mfma(net)) {
        int device = 0, n_cu = 0;
        if (hipGetDevice(&device) != hipSuccess) return hipErrorInvalidDevice;
        const int per_cu = fwd_stage_csr_per_cu(device, &n_cu);
        if (per_cu >= 2 && B * S_csr * ga.count <= (per_cu - 1) * n_cu) {
          CurJobs rest{};
          for (int i = 0; i < cj.count; ++i) {
            const bool dense = cj.j[i].nsteps > 0 && cj.j[i].mode == 1 && currents_job_kernel(net, cj.j[i]) == 1;
            CurJobs &dst = dense ? cj_fused : rest;
            dst.j[dst.count++] = cj.j[i];
          }
          if (cj_fused.count) cj = rest;
        }
      }
      hb(5);
      e = launch_currents(net, cj, s);
      he();
      if (e != hipSuccess) return e;
      hb(cj_fused.count ? 8 : 4);
      if (rs.count) {
        if (nw <= 64) hipLaunchKernelGGL((k_layer_seq_rs<64>), dim3(B, rs.count), dim3(64), 0, s, net, rs, state, st);
        else if (nw <= 128) hipLaunchKernelGGL((k_layer_seq_rs<128>), dim3(B, rs.count), dim3(128), 0, s, net, rs, state, st);
        else hipLaunchKernelGGL((k_layer_seq_rs<256>), dim3(B, rs.count), dim3(256), 0, s, net, rs, state, st);
      }
      if (S_csr) {
        // tags of the exchange entries start from zero in every launch
        e = launch_fill_zero(ws->xg, (size_t)ga.count * B * 4 * net.Wd[ga.j[0].l + 1] * sizeof(uint64_t), s);
        if (e != hipSuccess) return e;
        const int Nc = net.N[ga.j[0].l];
        const size_t lds_seq = seq_csr_lds(Nc, net.Wd[ga.j[0].l + 1]);
        if (cj_fused.count) {
          unsigned gx = 0;
          for (int i = 0; i < cj_fused.count; ++i) {
            const CurJob &j = cj_fused.j[i];
            const unsigned g = (unsigned)(((j.nsteps * B + 16 * SNN_DENSE_MB - 1) / (16 * SNN_DENSE_MB)) * ((net.N[j.lsel] + 255) >> 8));
            gx = g > gx ? g : gx;
          }
          const size_t lds = lds_seq > SNN_FWD_STAGE_CSR_LDS ? lds_seq : SNN_FWD_STAGE_CSR_LDS;
          hipLaunchKernelGGL(k_fwd_stage_csr, dim3(B * S_csr * ga.count + gx * cj_fused.count), dim3(256), lds, s, net, ga, state,
                             st, S_csr, reinterpret_cast<uint64_t *>(ws->xg), ws->err, ws->spin_limit, cj_fused, B * S_csr, (int)gx);
        } else {
          hipLaunchKernelGGL(k_layer_seq_csr_sl, dim3(B * S_csr, ga.count), dim3(256), lds_seq, s,
                             net, ga, state, st, S_csr, reinterpret_cast<uint64_t *>(ws->xg), ws->err, ws->spin_limit);
        }
      } else if (ga.count && S > 1) {
        // tags of the exchange entries start from zero in every launch
        e = launch_fill_zero(ws->xg, (size_t)ga.count * B * 4 * net.Wd[ga.j[0].l + 1] * sizeof(uint64_t), s);
        if (e != hipSuccess) return e;
        const size_t lds = seq_gather_lds(net);
        const dim3 grid(B * S, ga.count), block(th_sl);
        uint64_t *xw = reinterpret_cast<uint64_t *>(ws->xg);
#define SEQ_CASE(NPT_)                                                                                         \
  case NPT_:                                                                                                    \
    hipLaunchKernelGGL((k_layer_seq_gather_sl<NPT_>), grid, block, lds, s, net, ga, state, st, S, xw,          \
                       ws->err, ws->spin_limit);                                                                \
    break;
        switch (npt_sl) {
          SEQ_CASE(1) SEQ_CASE(2) SEQ_CASE(4) SEQ_CASE(8) SEQ_CASE(16)
          default: return hipErrorInvalidValue;
        }
#undef SEQ_CASE
      } else if (ga.count) {
        const size_t lds = seq_gather_lds(net);
        const dim3 grid(B, ga.count), block(c.nt_neuron);
#define SEQ_CASE(NPT_)                                                                               \
  case NPT_:                                                                                          \
    hipLaunchKernelGGL((k_layer_seq_gather<NPT_>), grid, block, lds, s, net, ga, state, st);          \
    break;
        switch (c.npt) {
          SEQ_CASE(1) SEQ_CASE(2) SEQ_CASE(4) SEQ_CASE(8) SEQ_CASE(16)
          default: return hipErrorInvalidValue;
        }
#undef SEQ_CASE
      }
      he();
    }
    if (!fuse && ro_now) {
      ro_steps += bounds[ko + 1] - bounds[ko];
      if (++ro_tiles == SNN_RO_TILES || ko == n_tiles - 1) {
        hb(5);
        hipLaunchKernelGGL(k_readout_scan, dim3((B * O + 255) / 256), dim3(256), 0, s, iout, readout, B, O, ro_steps,
                           net.beta, (ro_first && readout_init) ? 1 : 0);
        he();
        ro_first = false;
        ro_steps = 0;
        ro_tiles = 0;
      }
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (cb)
      for (int l = 0; l < L; ++l) {
        const int k = stage - 2 * l - 1;
        if (k < 0 || k >= n_tiles) continue;
        e = cb->layer_tile_done(cb->ctx, l, bounds[k + 1]);
        if (e != hipSuccess) return e;
      }
  }
  if (ro_pending.n) { // the last tile's readout
    hb(5);
    hipLaunchKernelGGL(k_readout_scan, dim3((B * O + 255) / 256), dim3(256), 0, s, ro_pending.iout, readout, B, O,
                       ro_pending.nsteps, net.beta, ro_pending.init);
    he();
  }
  return hipGetLastError();
}

hipError_t launch_recompute(const NetDev &net, int t0, int t1, const float *state_in, float *buf, int t_base,
                            size_t slot_stride, int store_all, float *state_out, hipStream_t s) {
  if (t1 <= t0) return hipErrorInvalidValue;
  CurJobs cj{};
  for (int l = 0; l < net.L; ++l) cj.j[cj.count++] = CurJob{0, l, t0, t1 - t0, t_base, buf, slot_stride};
  hipError_t e = launch_currents(net, cj, s);
  if (e != hipSuccess) return e;
  const size_t n = (size_t)net.B * net.SN;
  hipLaunchKernelGGL(k_scan, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, net, t0, t1, state_in, buf, t_base,
                     slot_stride, store_all, state_out, (const float *)nullptr, 0);
  return hipGetLastError();
}

hipError_t launch_recompute_currents(const NetDev &net, int t0, int t1, float *buf, int t_base, size_t slot_stride,
                                     hipStream_t s) {
  if (t1 <= t0) return hipErrorInvalidValue;
  CurJobs cj{};
  for (int l = 0; l < net.L; ++l) cj.j[cj.count++] = CurJob{0, l, t0, t1 - t0, t_base, buf, slot_stride};
  return launch_currents(net, cj, s);
}

hipError_t launch_recompute_scan(const NetDev &net, int t0, int t1, const float *state_in, float *buf, int t_base,
                                 size_t slot_stride, int store_all, float *state_out, hipStream_t s, const float *cur_src,
                                 int src_base) {
  if (t1 <= t0) return hipErrorInvalidValue;
  const size_t n = (size_t)net.B * net.SN;
  hipLaunchKernelGGL(k_scan, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, net, t0, t1, state_in, buf, t_base,
                     slot_stride, store_all, state_out, cur_src, src_base);
  return hipGetLastError();
}

hipError_t launch_loss(const double *readout, const int32_t *labels, int B, int O, int T, float *ubar, float *g,
                       float *loss, hipStream_t s) {
  hipLaunchKernelGGL(k_loss, dim3(1), dim3(256), (size_t)B * sizeof(double), s, readout, labels, B, O, T, ubar, g, loss);
  return hipGetLastError();
}

static hipError_t launch_up_gemm(const float *A, int lda, const float *W, int K, int N, float *C, int M,
                                 hipStream_t s) {
  // The choice of kernel may depend on the layer's shape and on alignments that are the same for every
  // tile (lda % 4 == 0 makes the alignment of A independent of the slot it starts at), never on M.
  const bool aligned16 = K % 16 == 0 && lda % 4 == 0 && ((uintptr_t)A & 15) == 0 && ((uintptr_t)W & 15) == 0;
  if (aligned16 && (size_t)N * K <= 65536) {
    const int tiles = ((M + 15) / 16) * ((N + 15) / 16);
    hipLaunchKernelGGL(k_up_gemm16, dim3((tiles + 3) / 4), dim3(256), 0, s, A, lda, W, K, N, C, N, M);
  } else if (up_gemm_big(N, K)) {
    if (N >= 4096 && M >= 2048)
      hipLaunchKernelGGL((k_up_gemm<4, 4, 2, 2>), dim3((M + 255) / 256, (N + 255) / 256), dim3(1024), 0, s, A, lda, W, K, N, C, N, M);
    else
      hipLaunchKernelGGL((k_up_gemm<2, 2, 2, 2>), dim3((M + 127) / 128, (N + 127) / 128), dim3(256), 0, s, A, lda, W, K, N, C, N, M);
  } else // 64 x 64 tiles: measured faster than 32 x 32 blocks (one wavefront each) and than 128 x 64 up to 1024 x 1024
    hipLaunchKernelGGL((k_up_gemm<2, 2>), dim3((M + 63) / 64, (N + 63) / 64), dim3(256), 0, s, A, lda, W, K, N, C, N, M);
  return hipGetLastError();
}

hipError_t launch_adjoint_head(const NetDev &net, int t0, int t1, int t_base, float *dubuf, const float *g,
                               float *carry, int carry_init, float *up_top, hipStream_t s, const SpanHook *hook) {
  if (t1 <= t0) return hipErrorInvalidValue;
  const int B = net.B, O = net.n_out, L = net.L;
  const size_t s0 = (size_t)(t0 - t_base);
  hipLaunchKernelGGL(k_du_scan, dim3((B * O + 255) / 256), dim3(256), 0, s, g, carry, dubuf, B, O, net.SN, t0, t1,
                     t_base, net.beta, carry_init);
  if (hook) hook->begin(hook->ctx, 6);
  const hipError_t e = launch_up_gemm(dubuf + s0 * B * O, O, net.W_out, O, net.N[L - 1], up_top, (t1 - t0) * B, s);
  if (hook) hook->end(hook->ctx);
  return e;
}

hipError_t launch_up_product(const NetDev &net, int l, int t0, int t1, int t_base, const float *vbuf, float *up_l,
                             hipStream_t s, const SpanHook *hook) {
  if (t1 <= t0 || l < 0 || l + 1 >= net.L) return hipErrorInvalidValue;
  const size_t s0 = (size_t)(t0 - t_base);
  if (hook) hook->begin(hook->ctx, 6);
  const hipError_t e = launch_up_gemm(vbuf + s0 * ((size_t)net.B * net.SN) + net.off[l + 1], net.SN, net.W_in[l + 1],
                                      net.N[l + 1], net.N[l], up_l, (t1 - t0) * net.B, s);
  if (hook) hook->end(hook->ctx);
  return e;
}

static bool ws_use_mfma(const NetDev &net);

// Chip-wide recurrence of a wide layer: geometry and launch.
template <int RB, int NBB>
static hipError_t launch_adj_wide_t(const NetDev &net, const AdjJob &jb, float *carry, const WsArgs &ws, int device,
                                    hipStream_t s, bool dry, int *resident) {
  const int N = net.N[jb.l];
  const size_t lds = (size_t)4 * (16 * RB) * (16 * NBB) * sizeof(float);
  static int cached[16] = {}; // resident workgroups per device: the occupancy of the kernel does not change
  if (device < 0 || device >= 16) return hipErrorInvalidValue;
  if (!cached[device]) {
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_adj_rec_wide<RB, NBB>, 256, lds);
    if (e != hipSuccess) return e;
    cached[device] = per_cu * prop.multiProcessorCount;
  }
  *resident = cached[device];
  if (dry) return hipSuccess;
  hipLaunchKernelGGL((k_adj_rec_wide<RB, NBB>), dim3(N / (16 * RB)), dim3(256), lds, s, net, jb, carry, ws.xg, ws.bar, ws.err,
                     ws.spin_limit);
  return hipGetLastError();
}
static hipError_t adj_wide_dispatch(const NetDev &net, const AdjJob &jb, float *carry, const WsArgs &ws, hipStream_t s,
                                    bool dry, int *rows, int *resident) {
  const int N = net.N[jb.l], nbb = (net.B + 15) / 16;
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  const int rb = N >= 4096 ? 2 : 1; // 32 rows per workgroup once that still gives 128 workgroups
  *rows = 16 * rb;
  if (rb == 2) {
    if (nbb == 1) return launch_adj_wide_t<2, 1>(net, jb, carry, ws, device, s, dry, resident);
    if (nbb == 2) return launch_adj_wide_t<2, 2>(net, jb, carry, ws, device, s, dry, resident);
    return launch_adj_wide_t<2, 4>(net, jb, carry, ws, device, s, dry, resident);
  }
  if (nbb == 1) return launch_adj_wide_t<1, 1>(net, jb, carry, ws, device, s, dry, resident);
  if (nbb == 2) return launch_adj_wide_t<1, 2>(net, jb, carry, ws, device, s, dry, resident);
  return launch_adj_wide_t<1, 4>(net, jb, carry, ws, device, s, dry, resident);
}
// Chip-wide recurrence over compressed rows (k_adj_rec_csrw): workgroups that can be resident at once, and the row
// blocks per job when `count` jobs share a launch (0: does not fit).
static int adj_csrw_resident() {
  static int cached[16] = {}; // per device: the occupancy of the kernel does not change
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 16) return 0;
  if (!cached[device]) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
    const size_t lds = ((size_t)8192 + 16 * 64) * 4 * sizeof(float); // the widest layer the library takes + the row sums
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(k_adj_rec_csrw), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
      return 0;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_adj_rec_csrw, 1024, lds) != hipSuccess) return 0;
    cached[device] = per_cu * prop.multiProcessorCount;
    if (cached[device] <= 0) cached[device] = -1;
  }
  return cached[device] > 0 ? cached[device] : 0;
}
static int adj_csrw_row_blocks(const NetDev &net, int count, int n_max) {
  const int n_bg = (net.B + 3) / 4;
  const int n_rb = (adj_csrw_resident() / (n_bg * count)) & ~7; // a multiple of 8: whole row blocks per die
  if (n_rb < 8 || (n_max + n_rb - 1) / n_rb > 1024) return 0;   // a wavefront keeps the positions of at most 64 rows
  return n_rb;
}
static bool adj_csrw_ok(const NetDev &net, int l, const WsArgs &ws) {
  const int N = net.N[l], B = net.B;
  if ((net.sel_adjoint != 0 && net.sel_adjoint < 6) || !net.csr_sub[l] || N <= 1024 || N > 8192 || B > 64 || !ws.xg) return false;
  if ((size_t)8 * ((B + 3) / 4) * N > (size_t)ws.xg_stride) return false;
  return adj_csrw_row_blocks(net, 1, N) > 0;
}
// SNN_WS_KERNEL=stream keeps wide layers on the one-workgroup-per-batch-element kernel
static bool adj_wide_ok(const NetDev &net, int l, const WsArgs &ws) {
  const int N = net.N[l], B = net.B;
  if (net.sel_adjoint == 2) return false;
  if (!ws.xg || N % 64 != 0 || B > 64) return false;
  const int bp = ((B + 15) / 16 == 3 ? 4 : (B + 15) / 16) * 16;
  if ((size_t)2 * bp * N > (size_t)ws.xg_stride) return false;
  AdjJob probe{};
  probe.l = l;
  int rows = 0, resident = 0;
  if (adj_wide_dispatch(net, probe, nullptr, ws, nullptr, true, &rows, &resident) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return N / rows <= resident;
}
// Called once when a context is created: the occupancy queries run outside any stream capture.
void adjoint_prepare(const NetDev &net, const WsArgs &ws) {
  for (int l = 0; l < net.L; ++l)
    if (net.N[l] > 1024) {
      (void)adj_wide_ok(net, l, ws);
      (void)adj_csrw_resident();
    }
  for (int l = 0; l < net.L; ++l)
    if (net.N[l] > 256) { // the sliced sequential part of the forward pass
      SeqJobs probe{};
      probe.j[0].l = l;
      probe.count = 1;
      int npt = 0, th = 0;
      (void)seq_slices(net, probe, &ws, &npt, &th);
      (void)seq_csr_slices(net, probe, &ws, false);
      int device = 0, n_cu = 0;
      if (hipGetDevice(&device) == hipSuccess) (void)fwd_stage_csr_per_cu(device, &n_cu);
    }
}
static hipError_t launch_adj_wide(const NetDev &net, const AdjJob &jb, float *carry, const WsArgs &ws, hipStream_t s) {
  int rows = 0, resident = 0;
  return adj_wide_dispatch(net, jb, carry, ws, s, false, &rows, &resident);
}

hipError_t launch_adjoint_jobs(const NetDev &net, const AdjJobs &jobs, float *carry, const WsArgs &ws, hipStream_t s,
                               const SpanHook *hook) {
  const int B = net.B;
  for (int i = 0; i < jobs.count; ++i)
    if (jobs.j[i].t1 <= jobs.j[i].t0 || jobs.j[i].l < 0 || jobs.j[i].l >= net.L) return hipErrorInvalidValue;
  if (hook) hook->begin(hook->ctx, 2);
  // register-stationary layers of one size class go out together (blockIdx.y = job)
  for (int cls = 0; cls < 2; ++cls) {
    AdjJobs rs{};
    int nthr = 0;
    for (int i = 0; i < jobs.count; ++i) {
      const int N = net.N[jobs.j[i].l];
      if (N > 256 || (N <= 128) != (cls == 0)) continue;
      const int nt = 2 * ((N + 63) & ~63); // H threads per R postsynaptic rows, H = 2R
      if (nthr && nt != nthr) { // same class, different block size: a launch of its own
        if (cls == 0) hipLaunchKernelGGL((k_adj_rec_rs<16, 8, 4>), dim3(B, rs.count), dim3(nthr), 0, s, net, rs, carry);
        else hipLaunchKernelGGL((k_adj_rec_rs<32, 8, 4>), dim3(B, rs.count), dim3(nthr), 0, s, net, rs, carry);
        rs.count = 0;
      }
      nthr = nt;
      rs.j[rs.count++] = jobs.j[i];
    }
    if (rs.count) {
      if (cls == 0) hipLaunchKernelGGL((k_adj_rec_rs<16, 8, 4>), dim3(B, rs.count), dim3(nthr), 0, s, net, rs, carry);
      else hipLaunchKernelGGL((k_adj_rec_rs<32, 8, 4>), dim3(B, rs.count), dim3(nthr), 0, s, net, rs, carry);
    }
  }
  bool taken[SNN_MAXL] = {};
  for (int i = 0; i < jobs.count; ++i) {
    const AdjJob &jb = jobs.j[i];
    const int l = jb.l, N = net.N[l];
    if (N <= 256 || taken[i]) continue;
    // Event-driven rows under a surrogate window: layers wider than 1024 (the streamed kernels pay for every row
    // of the matrix every step), or wherever the hook asks (3: listed rows, 4: the same kernel listing every row)
    if (net.sel_adjoint == 3 || net.sel_adjoint == 4 || (net.sel_adjoint == 0 && net.win > 0.0f && N > 1024)) {
      AdjJobs grp{};
      for (int k = i; k < jobs.count; ++k)
        if (!taken[k] && net.N[jobs.j[k].l] == N) {
          grp.j[grp.count++] = jobs.j[k];
          taken[k] = true;
        }
      const size_t lds = (size_t)2 * N * sizeof(float) + (size_t)((N + 7) & ~7) * sizeof(uint16_t);
      if (lds > 48 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_adj_rec_rows),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
      }
      hipLaunchKernelGGL(k_adj_rec_rows, dim3(B, grp.count), dim3(1024), lds, s, net, grp, carry, net.sel_adjoint == 4 ? 1 : 0);
      continue;
    }
    if (N <= 1024 && ws.xg && ws_use_mfma(net) && (B + 15) / 16 <= 64 && ((N + 31) / 32) * ((B + 15) / 16) <= ws.max_groups_m) {
      // matrix-core version: workgroup = 32 rows x 16 batch elements, or x 2 groups of 16 half a step apart (two
      // groups per workgroup double the products a workgroup runs one after the other per step and halve the
      // workgroups per layer; only where net.sel_adjoint == 8 asks and the batch has an even number of groups;
      // 7 keeps 32 rows and one group per workgroup).
      const int G_b = (B + 15) / 16;
      // Workgroups of eight wavefronts and 64 rows (RH = 2) halve the workgroups per layer as well, and with them
      // the reads of the exchange buffer, at one batch group per workgroup: measured faster than two groups where
      // the stage's layers do not fit one launch otherwise (configuration 2: 147 against 171 ms per step), slower
      // where they do (configuration 3: 36 against 28 ms: few workgroups, each with twice the products per step).
      // net.sel_adjoint == 9 forces them.
      int cnt = 0;
      for (int k = i; k < jobs.count; ++k)
        if (!taken[k] && net.N[jobs.j[k].l] == N) ++cnt;
      const int per1 = ((N + 31) / 32) * G_b, cap1 = ws.max_groups_m / per1;
      const bool plain = net.sel_adjoint == 7 || net.sel_adjoint == 8;
      const int RH = (net.sel_adjoint == 9 || (!plain && cap1 >= 1 && cnt > cap1)) ? 2 : 1;
      const int NG = (G_b % 2 == 0 && net.sel_adjoint == 8) ? 2 : 1;
      const int G_w = G_b / NG, n_slices = (N + 32 * RH - 1) / (32 * RH), bpj = n_slices * G_w;
      const int NK = N <= 512 ? 32 : 64;
      const size_t lds = (size_t)NG * ((size_t)16 * NK * 16 + RH * 4 * 32 * 16) * sizeof(float);
      AdjJobs grp{};
      for (int k = i; k < jobs.count; ++k)
        if (!taken[k] && net.N[jobs.j[k].l] == N && (grp.count + 1) * bpj <= ws.max_groups_m) {
          grp.j[grp.count++] = jobs.j[k];
          taken[k] = true;
        }
      // tags of the exchange entries start from zero in every launch
      hipError_t e = launch_fill_zero(ws.xg, (size_t)grp.count * ws.xg_stride * sizeof(float), s);
      if (e != hipSuccess) return e;
      const dim3 grid(bpj * grp.count), block(256 * RH);
#define WSM_CASE(NK_, NG_, RH_)                                                                                         \
  {                                                                                                                     \
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_adj_rec_wsm<NK_, NG_, RH_>),                               \
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                                      \
    if (e != hipSuccess) return e;                                                                                      \
    hipLaunchKernelGGL((k_adj_rec_wsm<NK_, NG_, RH_>), grid, block, lds, s, net, grp, carry, ws.xg, ws.bar, ws.err,     \
                       G_w, ws.spin_limit, bpj, ws.xg_stride);                                                          \
  }
      if (RH == 2) {
        if (NK == 32) WSM_CASE(32, 1, 2) else WSM_CASE(64, 1, 2)
      } else if (NK == 32) {
        if (NG == 1) WSM_CASE(32, 1, 1) else WSM_CASE(32, 2, 1)
      } else {
        if (NG == 1) WSM_CASE(64, 1, 1) else WSM_CASE(64, 2, 1)
      }
#undef WSM_CASE
    } else if (N <= 1024 && ws.xg && (B + 7) / 8 <= 64 && ((N + 31) / 32) * ((B + 7) / 8) <= ws.max_groups) {
      const int G_b = (B + 7) / 8, n_slices = (N + 31) / 32, bpj = n_slices * G_b;
      const int NR = N <= 512 ? 64 : 128;
      const size_t lds = ((size_t)NR * 8 * 8 + 8 * 32 * 8) * sizeof(float);
      // layers of the same width go out together as long as all their workgroups can be resident at once
      AdjJobs grp{};
      for (int k = i; k < jobs.count; ++k)
        if (!taken[k] && net.N[jobs.j[k].l] == N && (grp.count + 1) * bpj <= ws.max_groups) {
          grp.j[grp.count++] = jobs.j[k];
          taken[k] = true;
        }
      hipError_t e = launch_fill_zero(ws.bar, (size_t)64 * SNN_MAXL * sizeof(unsigned), s);
      if (e != hipSuccess) return e;
      if (NR == 64)
        hipLaunchKernelGGL((k_adj_rec_ws<64>), dim3(bpj * grp.count), dim3(256), lds, s, net, grp, carry, ws.xg, ws.bar,
                           ws.err, G_b, ws.spin_limit, bpj, ws.xg_stride);
      else
        hipLaunchKernelGGL((k_adj_rec_ws<128>), dim3(bpj * grp.count), dim3(256), lds, s, net, grp, carry, ws.xg, ws.bar,
                           ws.err, G_b, ws.spin_limit, bpj, ws.xg_stride);
    } else if (adj_csrw_ok(net, l, ws)) {
      // masked wide layers: every such job of the stage in one launch, the chip divided among them
      AdjJobs grp{};
      int n_max = 0;
      for (int k = i; k < jobs.count; ++k) {
        const int lk = jobs.j[k].l;
        if (taken[k] || !adj_csrw_ok(net, lk, ws)) continue;
        const int nm = net.N[lk] > n_max ? net.N[lk] : n_max;
        if (grp.count && !adj_csrw_row_blocks(net, grp.count + 1, nm)) continue;
        grp.j[grp.count++] = jobs.j[k];
        taken[k] = true;
        n_max = nm;
      }
      const int n_bg = (B + 3) / 4, n_rb = adj_csrw_row_blocks(net, grp.count, n_max);
      if (n_rb <= 0) return hipErrorInvalidValue;
      hipError_t e = launch_fill_zero(ws.bar, (size_t)64 * SNN_MAXL * sizeof(unsigned), s);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(k_adj_rec_csrw, dim3(grp.count * n_rb * n_bg), dim3(1024), ((size_t)n_max + 16 * 64) * 4 * sizeof(float),
                         s, net, grp, carry, ws.xg, ws.bar, ws.err, ws.spin_limit, n_rb, n_bg, ws.xg_stride, n_max);
    } else if (adj_wide_ok(net, l, ws)) {
      taken[i] = true;
      hipError_t e = launch_fill_zero(ws.bar, (size_t)64 * sizeof(unsigned), s);
      if (e != hipSuccess) return e;
      e = launch_adj_wide(net, jb, carry, ws, s);
      if (e != hipSuccess) return e;
    } else {
      taken[i] = true;
      const int nt = 1024;
      const size_t lds = ((size_t)2 * N + nt) * sizeof(float);
      if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_adj_rec_stream),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
      }
      hipLaunchKernelGGL(k_adj_rec_stream, dim3(B), dim3(nt), lds, s, net, l, jb.t0, jb.t1, jb.vbuf, jb.t_base, jb.up, N,
                         carry, jb.carry_init);
    }
  }
  if (hook) hook->end(hook->ctx);
  return hipGetLastError();
}

static bool ws_use_mfma(const NetDev &net) { return net.sel_adjoint != 1; } // 1: the VALU version of the chip-wide recurrence

int ws_max_resident_groups_mfma(int device) {
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
  int per_cu = 0;
  // the version with two batch groups per workgroup has the larger LDS footprint and bounds both
  const size_t lds = (size_t)2 * ((size_t)16 * 64 * 16 + 4 * 32 * 16) * sizeof(float);
  if (hipFuncSetAttribute(reinterpret_cast<const void *>(k_adj_rec_wsm<64, 2, 1>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)lds) != hipSuccess)
    return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_adj_rec_wsm<64, 2, 1>, 256, lds) != hipSuccess) return 0;
  return per_cu * prop.multiProcessorCount;
}

int ws_max_resident_groups(int device) {
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
  int per_cu = 0;
  const size_t lds = ((size_t)128 * 8 * 8 + 8 * 32 * 8) * sizeof(float);
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_adj_rec_ws<128>, 256, lds) != hipSuccess) return 0;
  return per_cu * prop.multiProcessorCount;
}

hipError_t launch_dw(const uint64_t *pre_mask, int pre_words, int n_pre, int lag, const float *postbuf,
                     size_t slot_stride, int post_stride, int post_off, int n_post, int B, int t0, int t1,
                     int t_base, double *dW, hipStream_t s, int pre_ring) {
  if (t1 <= t0) return hipSuccess;
  const dim3 grid(n_pre, (n_post + 256 * DW_NPT - 1) / (256 * DW_NPT));
  hipLaunchKernelGGL(k_dw, grid, dim3(256), 0, s, pre_mask, pre_words, lag, postbuf, slot_stride, post_stride,
                     post_off, n_post, B, t0, t1, t_base, dW, pre_ring);
  return hipGetLastError();
}

static hipError_t launch_dw_csr(DwBatch batch, int B, hipStream_t s) {
  if (batch.count <= 0) return hipSuccess;
  if (B > 32) return hipErrorInvalidValue; // a tile is at least one whole time step of at most 32 rows
  int total = 0;
  for (int i = 0; i < batch.count; ++i) {
    if (batch.d[i].t1 <= batch.d[i].t0 || !batch.d[i].csr_sub || batch.d[i].n_pre != batch.d[i].n_post) return hipErrorInvalidValue;
    batch.d[i].tiles_n = (batch.d[i].n_post + SNN_CSR_SUBW - 1) / SNN_CSR_SUBW; // = sub-ranges of a compressed row
    batch.d[i].tile0 = total;
    total += ((batch.d[i].n_pre + 255) / 256) * batch.d[i].tiles_n;
  }
  const size_t lds = (size_t)2 * 32 * SNN_CSR_SUBW * sizeof(float) + (size_t)2 * 4 * 32 * sizeof(uint64_t) + (size_t)DWC_WAVES * 64 * (sizeof(double) + sizeof(uint32_t));
  const hipError_t e = hipFuncSetAttribute(B == 32 ? reinterpret_cast<const void *>(k_dw_csr<true>)
                                                   : reinterpret_cast<const void *>(k_dw_csr<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  if (B == 32) hipLaunchKernelGGL(k_dw_csr<true>, dim3(total), dim3(64 * DWC_WAVES), lds, s, batch, B);
  else hipLaunchKernelGGL(k_dw_csr<false>, dim3(total), dim3(64 * DWC_WAVES), lds, s, batch, B);
  return hipGetLastError();
}

hipError_t launch_finish_grad_csr(const double *acc, const uint32_t *csr_sub, const uint16_t *csr_col, int N, float *dW,
                                  hipStream_t s) {
  hipLaunchKernelGGL(k_finish_grad_csr, dim3(N), dim3(256), 0, s, acc, csr_sub, csr_col, N,
                     (N + SNN_CSR_SUBW - 1) / SNN_CSR_SUBW, dW);
  return hipGetLastError();
}

hipError_t launch_dw_tile(DwBatch batch, int B, hipStream_t s) {
  if (batch.count <= 0) return hipSuccess;
  if (B > 64) return hipErrorInvalidValue; // a tile is at least one whole time step of at most 64 rows
  { // matrices that go through their compressed rows: a launch of their own
    DwBatch cs{}, dn{};
    cs.wide = dn.wide = batch.wide;
    for (int i = 0; i < batch.count; ++i) (batch.d[i].csr_sub ? cs.d[cs.count++] : dn.d[dn.count++]) = batch.d[i];
    if (cs.count) {
      const hipError_t e = launch_dw_csr(cs, B, s);
      if (e != hipSuccess) return e;
      batch = dn;
      if (batch.count <= 0) return hipSuccess;
    }
  }
  int total = 0;
  for (int i = 0; i < batch.count; ++i) {
    if (batch.d[i].t1 <= batch.d[i].t0) return hipErrorInvalidValue;
    batch.d[i].tiles_n = (batch.d[i].n_post + 255) / 256;
    batch.d[i].tile0 = total;
    total += ((batch.d[i].n_pre + 127) / 128) * batch.d[i].tiles_n;
  }
  const size_t lds = (size_t)2 * 64 * 256 * sizeof(float) + (size_t)2 * 2 * 64 * sizeof(uint64_t);
  const void *fn = B == 32 ? reinterpret_cast<const void *>(k_dw_tile<32>)
                   : B == 64 ? reinterpret_cast<const void *>(k_dw_tile<64>) : reinterpret_cast<const void *>(k_dw_tile<0>);
  const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  if (B == 32) hipLaunchKernelGGL(k_dw_tile<32>, dim3(total), dim3(64 * DWT_WAVES), lds, s, batch, B);
  else if (B == 64) hipLaunchKernelGGL(k_dw_tile<64>, dim3(total), dim3(64 * DWT_WAVES), lds, s, batch, B);
  else hipLaunchKernelGGL(k_dw_tile<0>, dim3(total), dim3(64 * DWT_WAVES), lds, s, batch, B);
  return hipGetLastError();
}

hipError_t launch_dw_mfma(DwBatch batch, int B, hipStream_t s) {
  if (batch.count <= 0) return hipSuccess;
  for (int i = 0; i < batch.count; ++i)
    if (batch.d[i].t1 <= batch.d[i].t0) return hipErrorInvalidValue;
  const int Bp = (B + 3) & ~3;
  if (Bp > 128) return hipErrorInvalidValue; // the staging registers cover at most 128 batch rows
  // wide tiles when the network's matrices already fill the chip with them; otherwise narrow ones and
  // two wavefronts per SIMD
  const bool wide = batch.wide && Bp <= 64;
  const int cols = wide ? 64 : 32; // a stage holds DW_STAGE_ELEMS / cols rows
  int total = 0;
  for (int i = 0; i < batch.count; ++i) {
    batch.d[i].tiles_n = (batch.d[i].n_post + cols - 1) / cols;
    batch.d[i].tile0 = total;
    total += ((batch.d[i].n_pre + 63) / 64) * batch.d[i].tiles_n;
  }
  const int rows = DW_STAGE_ELEMS / cols;
  const size_t lds = (size_t)2 * rows * (cols + 16) * sizeof(float) + (size_t)2 * rows * 8;
  {
    const hipError_t e = hipFuncSetAttribute(wide ? reinterpret_cast<const void *>(k_dw_mfma<4, 1>)
                                                  : reinterpret_cast<const void *>(k_dw_mfma<1, 2>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  if (wide) hipLaunchKernelGGL((k_dw_mfma<4, 1>), dim3(total), dim3(256), lds, s, batch, B);
  else hipLaunchKernelGGL((k_dw_mfma<1, 2>), dim3(total), dim3(512), lds, s, batch, B);
  return hipGetLastError();
}

// Where the recompute work of later chunks can ride: 2 = in the stage launch (8 wavefronts per workgroup beside
// 43 KB of static LDS), 1 = in the launch between stages (4 wavefronts, 25 KB static), 0 = nowhere (the spike
// words and lists of so wide a presynaptic layer do not fit).
int bwd_pre_placement(const NetDev &net) {
  int pmax = net.n_in;
  for (int l = 0; l < net.L; ++l) pmax = net.N[l] > pmax ? net.N[l] : pmax;
  const int ws = ((pmax + 63) / 64 + 1) | 1, lcap = ((pmax + 31) & ~31) + 32;
  if (currents_lds(8, ws, lcap) + 43 * 1024 <= SNN_LDS_PER_CU) return 2;
  if (currents_lds(4, ws, lcap) + 25 * 1024 <= SNN_LDS_PER_CU) return 1;
  return 0;
}

bool bwd_stage_fusable(const NetDev &net, int dw_wide) {
  // the fused stage kernel is built for 512-thread recurrences (layers of 193..256 neurons) and the narrow
  // contraction tiles
  const int Bp = (net.B + 3) & ~3;
  if ((dw_wide && Bp <= 64) || Bp > 128 || net.L < 2) return false;
  for (int l = 0; l < net.L; ++l)
    if (net.N[l] <= 192 || net.N[l] > 256) return false;
  return true;
}

// Geometry of the recompute jobs for a kernel with nwv wavefronts per workgroup; returns the LDS they need.
static hipError_t plan_pre(const NetDev &net, PreJobs *pre, int nwv, size_t *lds) {
  pre->cur_gx = 0;
  pre->ws = pre->lcap = 0;
  *lds = 0;
  if (pre->cur.count > 0) {
    for (int i = 0; i < pre->cur.count; ++i)
      if (pre->cur.j[i].mode != 0 || pre->cur.j[i].nsteps <= 0) return hipErrorInvalidValue;
    unsigned gx;
    currents_geometry(net, pre->cur, &gx, &pre->ws, &pre->lcap, nwv);
    pre->cur_gx = (int)gx;
    *lds = (size_t)nwv * 16 * pre->ws * sizeof(uint64_t) + (size_t)nwv * pre->lcap * sizeof(uint32_t);
  }
  if (pre->n_scan != 0) {
    if (pre->t1 <= pre->t0) return hipErrorInvalidValue;
    pre->n_scan = (int)(((size_t)net.B * net.SN + 64 * nwv - 1) / (64 * nwv));
  }
  return hipSuccess;
}

hipError_t launch_bwd_stage(const NetDev &net, const AdjJobs &jobs, float *carry, DwBatch batch, DuJob du,
                            const float *g, PreJobs pre, hipStream_t s, const SpanHook *hook) {
  if (!bwd_stage_fusable(net, batch.wide) || jobs.count < 1 || batch.count < 0) return hipErrorInvalidValue;
  for (int i = 0; i < jobs.count; ++i)
    if (jobs.j[i].t1 <= jobs.j[i].t0 || jobs.j[i].l < 0 || jobs.j[i].l >= net.L) return hipErrorInvalidValue;
  for (int i = 0; i < batch.count; ++i)
    if (batch.d[i].t1 <= batch.d[i].t0) return hipErrorInvalidValue;
  const int cols = 32, rows = DW_STAGE_ELEMS / cols;
  int total = 0;
  for (int i = 0; i < batch.count; ++i) {
    batch.d[i].tiles_n = (batch.d[i].n_post + cols - 1) / cols;
    batch.d[i].tile0 = total;
    total += ((batch.d[i].n_pre + 63) / 64) * batch.d[i].tiles_n;
  }
  size_t lds = (size_t)2 * rows * (cols + 16) * sizeof(float) + (size_t)2 * rows * 8;
  if (du.n != 0) {
    if (du.t1 <= du.t0 || !du.dubuf) return hipErrorInvalidValue;
    du.n = (net.B * net.n_out + 511) / 512;
  }
  {
    size_t lp;
    const hipError_t e = plan_pre(net, &pre, 8, &lp);
    if (e != hipSuccess) return e;
    lds = lp > lds ? lp : lds;
  }
  {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_bwd_stage<32, 8, 4>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  const int n_adj = net.B * jobs.count;
  if (hook) hook->begin(hook->ctx, 7);
  const int grid = n_adj + du.n + total + pre.cur_gx * pre.cur.count + pre.n_scan;
  hipLaunchKernelGGL((k_bwd_stage<32, 8, 4>), dim3(grid), dim3(512), lds, s, net, jobs, carry, batch, du, g, pre, n_adj,
                     total);
  if (hook) hook->end(hook->ctx);
  return hipGetLastError();
}

// Fills kind / n_blocks / tiles_m of an inter-layer product by the same rule as launch_up_gemm (shapes and
// tile-independent alignments only).
static void plan_gemm(GemmJob *gj) {
  const bool aligned16 = gj->K % 16 == 0 && gj->lda % 4 == 0 && ((uintptr_t)gj->A & 15) == 0 && ((uintptr_t)gj->W & 15) == 0;
  if (aligned16 && (size_t)gj->N * gj->K <= 65536) {
    gj->kind = 0;
    gj->tiles_m = (gj->M + 15) / 16;
    gj->n_blocks = (gj->tiles_m * ((gj->N + 15) / 16) + 3) / 4;
  } else if (up_gemm_big(gj->N, gj->K)) {
    gj->kind = 2;
    gj->tiles_m = (gj->M + 127) / 128;
    gj->n_blocks = gj->tiles_m * ((gj->N + 127) / 128);
  } else {
    gj->kind = 1;
    gj->tiles_m = (gj->M + 63) / 64;
    gj->n_blocks = gj->tiles_m * ((gj->N + 63) / 64);
  }
}

hipError_t launch_bwd_inter(const NetDev &net, InterJobs ij, hipStream_t s, const SpanHook *hook) {
  if (ij.n_gemm < 0 || ij.n_gemm > SNN_MAXL + 1) return hipErrorInvalidValue;
  int grid = 0, kept = 0;
  for (int q = 0; q < ij.n_gemm; ++q)
    if (ij.g[q].M <= 0 || ij.g[q].N <= 0 || ij.g[q].K <= 0) return hipErrorInvalidValue;
  PreJobs &pre = ij.pre;
  size_t lds = 0;
  {
    const hipError_t e = plan_pre(net, &pre, 4, &lds);
    if (e != hipSuccess) return e;
  }
  if (hook) hook->begin(hook->ctx, 6);
  for (int q = 0; q < ij.n_gemm; ++q) {
    plan_gemm(&ij.g[q]);
    if (ij.g[q].kind == 2) {
      // products of large matrices fill the chip by themselves and want the registers of the 128 x 128 tiles:
      // launches of their own, the fused launch keeps the rest
      const GemmJob &gj = ij.g[q];
      // 256 x 256 tiles (16 wavefronts) where they still give a workgroup to every compute unit, else 128 x 128:
      // 54 against 58 ms per step at configuration 4, T = 512 (256 x 128 with 8 wavefronts: 56; with 4: 62).  The
      // operations per element of C are the same for every tile shape, so this choice may look at M.
      if (gj.N >= 4096 && gj.M >= 2048)
        hipLaunchKernelGGL((k_up_gemm<4, 4, 2, 2>), dim3((gj.M + 255) / 256, (gj.N + 255) / 256), dim3(1024), 0, s, gj.A, gj.lda,
                           gj.W, gj.K, gj.N, gj.C, gj.N, gj.M);
      else
        hipLaunchKernelGGL((k_up_gemm<2, 2, 2, 2>), dim3(gj.tiles_m, (gj.N + 127) / 128), dim3(256), 0, s, gj.A, gj.lda, gj.W,
                           gj.K, gj.N, gj.C, gj.N, gj.M);
      continue;
    }
    grid += ij.g[q].n_blocks;
    ij.g[kept++] = ij.g[q];
  }
  ij.n_gemm = kept;
  grid += pre.cur_gx * pre.cur.count + pre.n_scan;
  if (grid > 0) {
    hipError_t e = hipSuccess;
    if (lds > 32 * 1024)
      e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_bwd_inter), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) hipLaunchKernelGGL(k_bwd_inter, dim3(grid), dim3(256), lds, s, net, ij);
    if (e != hipSuccess) {
      if (hook) hook->end(hook->ctx);
      return e;
    }
  }
  if (hook) hook->end(hook->ctx);
  return hipGetLastError();
}

hipError_t launch_transpose(const float *src, float *dst, int rows, int cols, hipStream_t s) {
  hipLaunchKernelGGL(k_transpose, dim3((cols + 31) / 32, (rows + 31) / 32), dim3(32, 8), 0, s, src, dst, rows, cols);
  return hipGetLastError();
}

hipError_t launch_finish_grad(const double *acc, const uint8_t *mask, float *dW, size_t n, hipStream_t s) {
  hipLaunchKernelGGL(k_finish_grad, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, acc, mask, dW, n);
  return hipGetLastError();
}

hipError_t launch_unpack_spikes(const uint64_t *mask, int words, int N, int T, int B, uint8_t *dst, hipStream_t s) {
  const size_t TB = (size_t)T * B, n = TB * N;
  // skip row 0 (t = 0)
  hipLaunchKernelGGL(k_unpack, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, mask + (size_t)B * words, words, N,
                     TB, dst);
  return hipGetLastError();
}

hipError_t launch_count_spikes(const uint64_t *mask, size_t n_words, unsigned long long *count, hipStream_t s) {
  hipLaunchKernelGGL(k_count, dim3(512), dim3(256), 0, s, mask, n_words, count);
  return hipGetLastError();
}

hipError_t launch_copy(const void *src, void *dst, size_t bytes, hipStream_t s) {
  if (bytes % 16) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_copy, dim3(4096), dim3(256), 0, s, (const float4 *)src, (float4 *)dst, bytes / 16);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  hipLaunchKernelGGL(k_zero, dim3(1024), dim3(256), 0, s, (uint32_t *)p, bytes / 4);
  return hipGetLastError();
}
