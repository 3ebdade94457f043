// Checkpoint plan and schedule: pure integer host logic, no GPU calls.
//
// Checkpoints sit at multiples of the interval starting at x_0 (the zero initial state); the last
// segment may be shorter; the coarse interval need not be a multiple of the fine one.  A segment
// (a, b] recomputed from x_a yields x_{a+1..b} from the stored spikes.  State-slot counts are the
// paper's closed forms (eq. M_Base, M_Standard, M_Remote, M_Double) plus, for the host tier, a second
// slot for prefetched checkpoints and SNN_FWD_LAG + 2 slots that stage device-to-host copies (the layers
// of the forward pass are pipelined two tiles apart, so up to SNN_FWD_LAG + 1 segment ends are being
// assembled while one is on its way to the host).
#include <cmath>

#include "snn_internal.h"

static int cdiv(int a, int b) { return (a + b - 1) / b; }
static int isqrt_ceil(int x) {
  int r = (int)std::ceil(std::sqrt((double)x));
  while ((long long)r * r < x) ++r;
  while (r > 1 && (long long)(r - 1) * (r - 1) >= x) --r;
  return r < 1 ? 1 : r;
}

bool snn_make_plan(int strategy, int T, int C, int F, Plan *p) {
  if (T < 1 || C < 0 || F < 0) return false;
  Plan q{};
  q.keep_from = -1;
  q.strategy = strategy;
  q.T = T;
  q.n_chunk_bufs = 1;
  switch (strategy) {
    case 0: // STANDARD: every state
      q.C = q.F = 0;
      q.chunk_len = T;
      break;
    case 1: // CHUNK: local checkpoints every F steps (default sqrt T) + one chunk buffer
      q.F = F ? F : isqrt_ceil(T);
      if (q.F > T) return false;
      q.C = 0;
      q.chunk_len = q.F;
      q.n_local_ckpt = cdiv(T, q.F);
      break;
    case 2: // REMOTE: host checkpoints every C steps, chunk buffer of C states
      q.C = C ? C : isqrt_ceil(T);
      if (q.C > T) return false;
      q.F = 0;
      q.chunk_len = q.C;
      q.n_load_slots = 2;
      q.n_stage_slots = SNN_FWD_LAG + 2;
      q.n_remote = cdiv(T, q.C);
      break;
    case 3: // DOUBLE: host checkpoints every C, recomputed local checkpoints every F
      q.C = C ? C : isqrt_ceil(T);
      if (q.C > T) return false;
      q.F = F ? F : isqrt_ceil(q.C);
      if (q.F > q.C) return false;
      q.chunk_len = q.F;
      q.n_local_ckpt = cdiv(q.C, q.F) - 1; // the first fine checkpoint of a segment is the loaded coarse one
      q.n_load_slots = 2;
      q.n_stage_slots = SNN_FWD_LAG + 2;
      q.n_remote = cdiv(T, q.C);
      break;
    case 4: { // HIER: checkpoints every F steps, moved to/from the host in batches of C = nb_local
      q.F = F ? F : isqrt_ceil(T);
      if (q.F > T) return false;
      const int n_ckpt = cdiv(T, q.F);
      q.C = C ? C : isqrt_ceil(n_ckpt);
      if (q.C < 1) return false;
      q.chunk_len = q.F;
      // ring of batches: the one in use, the one in flight to/from the host, and enough more that the
      // lowest layer of the pipelined forward pass never laps the top layer (up to SNN_FWD_LAG
      // checkpoints behind)
      q.n_local_ckpt = (2 + cdiv(SNN_FWD_LAG, q.C)) * q.C;
      q.n_remote = (cdiv(n_ckpt, q.C) - 1) * q.C;
      break;
    }
    default:
      return false;
  }
  *p = q;
  return true;
}

int64_t snn_make_schedule(const Plan &p, SchedOp *out, int64_t cap) {
  int64_t n = 0;
  auto emit = [&](int op, int a, int b) {
    if (out && n < cap) out[n] = SchedOp{op, a, b};
    ++n;
  };
  const int T = p.T;
  auto imin = [](int a, int b) { return a < b ? a : b; };
  switch (p.strategy) {
    case 0:
      emit(OP_BACKWARD, T, 1);
      break;
    case 1:
      for (int c = 0; c < T; c += p.F) emit(OP_SAVE_LOCAL, c, 0);
      for (int k = cdiv(T, p.F) - 1; k >= 0; --k) {
        const int a = k * p.F, e = imin(a + p.F, T);
        emit(OP_REFWD2, a, e);
        emit(OP_BACKWARD, e, a + 1);
      }
      break;
    case 2:
      for (int c = 0; c < T; c += p.C) emit(OP_SAVE_REMOTE, c, 0);
      for (int k = cdiv(T, p.C) - 1; k >= 0; --k) {
        const int a = k * p.C, e = imin(a + p.C, T);
        emit(OP_LOAD_REMOTE, a, 0);
        emit(OP_REFWD2, a, e);
        emit(OP_BACKWARD, e, a + 1);
      }
      break;
    case 3:
      for (int c = 0; c < T; c += p.C) emit(OP_SAVE_REMOTE, c, 0);
      for (int K = cdiv(T, p.C) - 1; K >= 0; --K) {
        const int s0 = K * p.C, e = imin(s0 + p.C, T);
        emit(OP_LOAD_REMOTE, s0, 0);
        const int nf = cdiv(e - s0, p.F);
        const int last = s0 + (nf - 1) * p.F;
        if (last > s0) {
          emit(OP_REFWD1, s0, last);
          for (int c = s0 + p.F; c <= last; c += p.F) emit(OP_KEEP_FINE, c, 0);
        }
        for (int m = nf - 1; m >= 0; --m) {
          const int a = s0 + m * p.F, fe = imin(a + p.F, e);
          emit(OP_REFWD2, a, fe);
          emit(OP_BACKWARD, fe, a + 1);
        }
      }
      break;
    case 4: {
      const int n_ckpt = cdiv(T, p.F), n_batches = cdiv(n_ckpt, p.C);
      for (int k = 0; k < n_ckpt; ++k) {
        emit(OP_SAVE_LOCAL, k * p.F, 0);
        if (k % p.C == p.C - 1 && k / p.C < n_batches - 1) emit(OP_SAVE_BATCH, (k / p.C) * p.C * p.F, p.C);
      }
      for (int g = n_batches - 1; g >= 0; --g) {
        if (g < n_batches - 1) emit(OP_LOAD_BATCH, g * p.C * p.F, p.C);
        for (int k = imin((g + 1) * p.C, n_ckpt) - 1; k >= g * p.C; --k) {
          const int a = k * p.F, e = imin(a + p.F, T);
          emit(OP_REFWD2, a, e);
          emit(OP_BACKWARD, e, a + 1);
        }
      }
      break;
    }
  }
  return n;
}
