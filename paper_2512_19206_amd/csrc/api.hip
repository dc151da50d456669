// Host side of libmixkvq: configuration checks, the block-record layout, the
// cache state machine (residual window and lazy flush of Appendix D.1) and the
// C ABI.  All device work is enqueued by the launchers in the kernel files.
#include <new>
#include <stdio.h>
#include <string.h>
#include "mixkvq_internal.h"

namespace mixkvq {

static thread_local char g_hip_msg[256] = "no HIP error recorded";

static int hip_fail(hipError_t e) {
  snprintf(g_hip_msg, sizeof(g_hip_msg), "HIP error %d: %s", (int)e, hipGetErrorString(e));
  (void)hipGetLastError();
  return MIXKVQ_EHIP;
}
#define MIXKVQ_TRY_HIP(expr)                          \
  do {                                                \
    hipError_t e__ = (expr);                          \
    if (e__ != hipSuccess) return hip_fail(e__);      \
  } while (0)

static inline int al16(int n) { return (n + 15) / 16 * 16; }

// Tokens per stored record.  A block of R tokens is one record, except: R = 256 is stored as two records of 128 tokens,
// and R = 96 with key groups that divide 32 as three records of 32 (the sizes the matrix-core kernel takes).
int rec_tokens(const mixkvq_config& c) {
  if (c.R > kMaxR) return kMaxR;
  if (c.R == 96 && c.Gk > 0 && 32 % c.Gk == 0) return 32;
  return c.R;
}

int compute_layout(const mixkvq_config& c, Layout* out) {
  if (c.B < 1 || c.Hq < 1 || c.Hkv < 1 || c.Hq % c.Hkv != 0) return MIXKVQ_EINVAL;
  if (c.Hq / c.Hkv > 8) return MIXKVQ_EINVAL;
  if (c.D != kD) return MIXKVQ_EINVAL;
  // residual length: a multiple of 16 up to 128, or 256 (see rec_tokens)
  if (c.R < 16 || c.R % 16 != 0 || (c.R > kMaxR && c.R != kMaxWindow)) return MIXKVQ_EINVAL;
  const int Rr = rec_tokens(c);
  if (c.Gk < 16 || c.Gk % 16 != 0 || Rr % c.Gk != 0) return MIXKVQ_EINVAL;
  if (c.Gv < 16 || c.Gv % 16 != 0 || c.D % c.Gv != 0) return MIXKVQ_EINVAL;
  if (c.k4 < 0 || c.k16 < 0 || c.k4 % 8 != 0 || c.k16 % 4 != 0 || c.k4 + c.k16 >= c.D) return MIXKVQ_EINVAL;
  if (c.T_max < c.R || c.T_max % c.R != 0) return MIXKVQ_EINVAL;
  if (c.flush_mode < 0 || c.flush_mode > 1 || c.score_mode < 0 || c.score_mode > 1) return MIXKVQ_EINVAL;
  if ((int64_t)c.B * c.Hkv > (1 << 20)) return MIXKVQ_EINVAL;
  if ((int64_t)c.B * c.Hkv * (c.T_max / Rr) >= (1ll << 31)) return MIXKVQ_EINVAL;   // record indices are 32-bit
  if (c.policy < 0 || c.policy > 1) return MIXKVQ_EINVAL;
  if (c.policy == 1 && !(c.tau16 >= 0.0 && c.tau4 >= 0.0)) return MIXKVQ_EINVAL;   // also rejects NaN
  if (c.sink < 0 || c.sink > 128 || c.sink % 32 != 0) return MIXKVQ_EINVAL;
  if (c.in_dtype < 0 || c.in_dtype > 1) return MIXKVQ_EINVAL;
  Layout l;
  memset(&l, 0, sizeof(l));
  const int ks = c.k4 + c.k16;
  l.NL = c.policy == 1 ? c.D : c.D - ks;
  l.Wlo = (l.NL + 15) / 16;
  l.NLp = 16 * l.Wlo;
  l.NG = Rr / c.Gk;
  l.NVG = c.D / c.Gv;
  l.W4 = c.k4 / 8;
  int off = 0;
  auto plane = [&](int32_t* dst, int bytes) { *dst = off; off += al16(bytes); };
  plane(&l.off_idx, ks);
  plane(&l.off_kmax, (l.NG + 1) * 2);
  plane(&l.off_klo_s, l.NG * l.NLp * 2);
  plane(&l.off_klo_z, l.NG * l.NLp * 2);
  plane(&l.off_k4_s, l.NG * c.k4 * 2);
  plane(&l.off_k4_z, l.NG * c.k4 * 2);
  plane(&l.off_klo, Rr * l.Wlo * 4);
  plane(&l.off_k4, Rr * l.W4 * 4);
  plane(&l.off_k16, Rr * c.k16 * 2);
  plane(&l.off_v, (Rr / 16) * c.D * 4);
  plane(&l.off_v_s, Rr * l.NVG * 2);
  plane(&l.off_v_z, Rr * l.NVG * 2);
  l.rec_bytes = off;
  l.v_interleave = (c.Gk == 32 && Rr % 64 == 0) ? 1 : 0;
  if (l.rec_bytes > kMaxRec) return MIXKVQ_EINVAL;
  *out = l;
  return MIXKVQ_OK;
}

int max_splits_for(int P) {
  int s = (kSplitTargetWGs + P - 1) / P;
  if (s < 1) s = 1;
  if (s > kMaxSplits) s = kMaxSplits;
  return s;
}

static inline uint64_t al256(uint64_t n) { return (n + 255) / 256 * 256; }

}  // namespace mixkvq

using namespace mixkvq;

struct SeqState {
  int64_t n_quant;   // quantized tokens
  int32_t n_res;     // tokens in the residual window
  int32_t n_sink;    // tokens in the sink
  bool operator==(const SeqState& o) const { return n_quant == o.n_quant && n_res == o.n_res && n_sink == o.n_sink; }
};

struct mixkvq_cache {
  CacheView v;       // v.cfg.R is the number of tokens per RECORD (what the kernels work on): rec_tokens()
  int32_t Rw;        // the residual length R of the configuration: window size and flush unit, Rw / v.cfg.R records per block
  SeqState* seq;     // [B]: every sequence has its own counts (they are equal while the batch runs in lock-step)
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;   // optional timing of the split kernel
  int last_path = MIXKVQ_PATH_NONE;                   // kernel of the last attention launch
};

namespace mixkvq {

// View of sequences [b0, b0 + nb) of the cache: the same kernels run on it as on the whole batch.
static CacheView sub_view(const mixkvq_cache* c, int b0, int nb) {
  CacheView v = c->v;
  const size_t p0 = (size_t)b0 * v.cfg.Hkv;
  v.cfg.B = nb;
  v.P = nb * v.cfg.Hkv;
  if (v.table) v.table += (size_t)b0 * v.NB;      // the pool itself is shared by all sequences
  else v.blocks += p0 * v.NB * v.lay.rec_bytes;
  v.res_k += p0 * v.RW * kD;
  v.res_v += p0 * v.RW * kD;
  v.qacc += p0 * kD;
  v.qcnt += p0;
  return v;
}

// What an append of n_new tokens does to a sequence in state st: tokens for the sink, blocks flushed, what remains.
struct AppendPlan { int take; int64_t F; int n_rest; int n_win; };
static AppendPlan plan_append(const mixkvq_config& cfg, int R, const SeqState& st, int n_new) {
  const int S = cfg.sink;
  AppendPlan pl;
  // the first S tokens of the sequence go to the sink; the others take the window / flush path
  pl.take = st.n_sink < S ? (n_new < S - st.n_sink ? n_new : S - st.n_sink) : 0;
  pl.n_win = n_new - pl.take;
  const int64_t total = (int64_t)st.n_res + pl.n_win;
  // Deferred: a full window is flushed just before the next token enters, so 1..R tokens remain.
  // Eager: a window is flushed as soon as it is full, so 0..R-1 tokens remain.
  pl.F = cfg.flush_mode == 0 ? (total + R - 1) / R - 1 : total / R;
  if (pl.F < 0) pl.F = 0;
  pl.n_rest = (int)(total - pl.F * R);
  return pl;
}

// Appends n_new tokens to sequences [b0, b0 + nb), which share one state.  k_new, v_new point at batch entry b0.
static int append_range(mixkvq_cache* c, int b0, int nb, const __half* k_new, const __half* v_new, int n_new,
                        Strides3 kvs, const uint8_t* sel, hipStream_t s) {
  const mixkvq_config& cfg = c->v.cfg;
  const int R = c->Rw, Rr = cfg.R, per = R / Rr, S = cfg.sink;      // a block of R tokens = `per` records of Rr
  const SeqState st = c->seq[b0];
  const AppendPlan pl = plan_append(cfg, R, st, n_new);
  const CacheView v = sub_view(c, b0, nb);
  SeqState nx = st;
  if (pl.take > 0) {
    MIXKVQ_TRY_HIP(launch_residual_copy(v, k_new, v_new, kvs, 0, st.n_sink, pl.take, s));
    nx.n_sink += pl.take;
  }
  if (pl.n_win > 0) {
    // from here on "new tokens" are the n_win tokens after the sink's share (strides are multiples of 8 elements,
    // so the shifted pointers keep their 16-byte alignment)
    const __half* kw = k_new + (int64_t)pl.take * kvs.t;
    const __half* vw = v_new + (int64_t)pl.take * kvs.t;
    const int r0 = st.n_res;
    const int first_rec = (int)(st.n_quant / Rr);
    if (pl.F > 0 && (sel || per == 1 || cfg.k4 + cfg.k16 == 0)) {
      // one selection for the call, blocks of one record each (the pack kernel scores those itself), or nothing to select
      MIXKVQ_TRY_HIP(launch_flush(v, kw, vw, kvs, r0, first_rec, (int)pl.F * per, sel, s));
    } else if (pl.F > 0) {
      // blocks of several records without a given selection: every block is scored over all its R tokens first
      // (they may lie partly in the window, partly in the new tokens), then its records are packed with that choice
      uint8_t* sel_blk = select_scratch(v);
      const Strides3 ws{(int64_t)cfg.Hkv * v.RW * kD, (int64_t)v.RW * kD, (int64_t)kD};
      for (int64_t u = 0; u < pl.F; ++u) {
        const int64_t p0 = u * R, p1 = p0 + R;                  // stream positions of (window ++ new tokens)
        const int nA = p0 < r0 ? (int)((p1 < r0 ? p1 : r0) - p0) : 0;      // tokens taken from the window
        const __half* kA = v.res_k + (size_t)(S + p0) * kD;
        const __half* kB = kw + (p0 + nA - r0) * kvs.t;
        MIXKVQ_TRY_HIP(launch_select2(v, kA, nA, ws, kB, R - nA, kvs, sel_blk, s));
        // (stream origin shifted so that record 0 of this launch is record u * per of the call; r0 - u R <= 0 for u >= 1)
        MIXKVQ_TRY_HIP(launch_flush(v, kw + (u ? (u * R - r0) * kvs.t : 0), vw + (u ? (u * R - r0) * kvs.t : 0), kvs,
                                    u ? 0 : r0, first_rec + (int)u * per, per, sel_blk, s));
      }
    }
    // Tokens that stay in the window.  Stream position x of (old residual ++ new tokens) maps to
    // new-token index x - r0; after F flushes positions [F*R, total) remain.
    const int64_t rest_first = pl.F * R;
    if (pl.F == 0) {
      MIXKVQ_TRY_HIP(launch_residual_copy(v, kw, vw, kvs, 0, S + r0, pl.n_win, s));
    } else if (pl.n_rest > 0) {
      MIXKVQ_TRY_HIP(launch_residual_copy(v, kw, vw, kvs, (int)(rest_first - r0), S, pl.n_rest, s));
    }
    if (pl.F > 0 && cfg.qacc_reset_on_flush) MIXKVQ_TRY_HIP(launch_zero_qacc(v, s));
    nx.n_quant += pl.F * R;
    nx.n_res = pl.n_rest;
  }
  for (int b = b0; b < b0 + nb; ++b) c->seq[b] = nx;
  return MIXKVQ_OK;
}

static bool lock_step(const mixkvq_cache* c) {
  for (int b = 1; b < c->v.cfg.B; ++b)
    if (!(c->seq[b] == c->seq[0])) return false;
  return true;
}

// Counts for a decode launch: the scalar maxima, and per sequence when they differ (sc->enabled).
// Returns false when the batch is ragged and too large for the by-value table.
static bool decode_counts(const mixkvq_cache* c, int extra_fp16, int* n_blocks, int* n_fp16, SeqCounts* sc) {
  const mixkvq_config& cfg = c->v.cfg;
  int mb = 0, mf = 0;
  for (int b = 0; b < cfg.B; ++b) {
    const SeqState& st = c->seq[b];
    const int nb = (int)(st.n_quant / cfg.R), nf = st.n_sink + st.n_res + extra_fp16;
    mb = nb > mb ? nb : mb;
    mf = nf > mf ? nf : mf;
  }
  *n_blocks = mb;
  *n_fp16 = mf;
  sc->enabled = lock_step(c) ? 0 : 1;
  if (sc->enabled) {
    if (cfg.B > kMaxRaggedB) return false;
    for (int b = 0; b < cfg.B; ++b) {
      const SeqState& st = c->seq[b];
      const int nf = st.n_sink + st.n_res;
      sc->n_blocks[b] = (int)(st.n_quant / cfg.R);
      sc->n_fp16[b] = (uint16_t)(nf + extra_fp16);
    }
  }
  return true;
}

}  // namespace mixkvq

extern "C" {

int mixkvq_block_layout(const mixkvq_config* cfg, mixkvq_block_layout_t* out) {
  if (!cfg || !out) return MIXKVQ_EINVAL;
  Layout l;
  int rc = compute_layout(*cfg, &l);
  if (rc != MIXKVQ_OK) return rc;
  *out = l;
  return MIXKVQ_OK;
}

int mixkvq_cache_sizes(const mixkvq_config* cfg, mixkvq_sizes* out) {
  if (!cfg || !out) return MIXKVQ_EINVAL;
  Layout l;
  int rc = compute_layout(*cfg, &l);
  if (rc != MIXKVQ_OK) return rc;
  const uint64_t P = (uint64_t)cfg->B * cfg->Hkv;
  out->blocks = al256(P * (uint64_t)(cfg->T_max / rec_tokens(*cfg)) * (uint64_t)l.rec_bytes);
  out->res_k = al256(P * (uint64_t)(cfg->R + cfg->sink) * cfg->D * 2);
  out->res_v = out->res_k;
  out->qacc = al256(P * (uint64_t)(cfg->D + 1) * 8);
  uint64_t a = decode_workspace_bytes(*cfg), b = select_workspace_bytes(*cfg);
  out->workspace = al256(a > b ? a : b);
  return MIXKVQ_OK;
}

int mixkvq_cache_create(const mixkvq_config* cfg, const mixkvq_buffers* bufs, mixkvq_cache** out) {
  if (!cfg || !bufs || !out) return MIXKVQ_EINVAL;
  Layout l;
  int rc = compute_layout(*cfg, &l);
  if (rc != MIXKVQ_OK) return rc;
  const void* ptrs[5] = {bufs->blocks, bufs->res_k, bufs->res_v, bufs->qacc, bufs->workspace};
  for (const void* p : ptrs)
    if (!p || ((uintptr_t)p & 255u)) return MIXKVQ_EINVAL;
  mixkvq_cache* c = new (std::nothrow) mixkvq_cache;
  if (!c) return MIXKVQ_ENOMEM;
  c->seq = new (std::nothrow) SeqState[cfg->B];
  if (!c->seq) {
    delete c;
    return MIXKVQ_ENOMEM;
  }
  c->v.cfg = *cfg;
  c->v.cfg.R = rec_tokens(*cfg);      // what the kernels call R: the tokens of one record
  c->Rw = cfg->R;
  c->v.lay = l;
  c->v.P = cfg->B * cfg->Hkv;
  c->v.g = cfg->Hq / cfg->Hkv;
  c->v.NB = cfg->T_max / c->v.cfg.R;
  c->v.S = cfg->sink;
  c->v.RW = cfg->sink + cfg->R;
  c->v.blocks = (uint8_t*)bufs->blocks;
  c->v.table = nullptr;
  c->v.res_k = (__half*)bufs->res_k;
  c->v.res_v = (__half*)bufs->res_v;
  c->v.qacc = (unsigned long long*)bufs->qacc;
  c->v.qcnt = c->v.qacc + (size_t)c->v.P * cfg->D;
  c->v.ws = (uint8_t*)bufs->workspace;
  for (int b = 0; b < cfg->B; ++b) c->seq[b] = SeqState{0, 0, 0};
  *out = c;
  return MIXKVQ_OK;
}

void mixkvq_cache_destroy(mixkvq_cache* c) {
  if (!c) return;
  delete[] c->seq;
  delete c;
}

int mixkvq_cache_reset(mixkvq_cache* c, void* stream) {
  if (!c) return MIXKVQ_EINVAL;
  MIXKVQ_TRY_HIP(launch_zero_qacc(c->v, (hipStream_t)stream));
  for (int b = 0; b < c->v.cfg.B; ++b) c->seq[b] = SeqState{0, 0, 0};
  return MIXKVQ_OK;
}

int mixkvq_cache_reset_seq(mixkvq_cache* c, int32_t b, void* stream) {
  if (!c || b < 0 || b >= c->v.cfg.B) return MIXKVQ_EINVAL;
  if (c->v.cfg.B > kMaxRaggedB) return MIXKVQ_EINVAL;     // such a batch could not be attended over once it is ragged
  MIXKVQ_TRY_HIP(launch_zero_qacc(sub_view(c, b, 1), (hipStream_t)stream));
  c->seq[b] = SeqState{0, 0, 0};
  return MIXKVQ_OK;
}

int mixkvq_cache_state(const mixkvq_cache* c, int64_t* n_quantized, int32_t* n_residual, int32_t* n_sink) {
  if (!c) return MIXKVQ_EINVAL;
  if (!lock_step(c)) return MIXKVQ_ERAGGED;
  if (n_quantized) *n_quantized = c->seq[0].n_quant;
  if (n_residual) *n_residual = c->seq[0].n_res;
  if (n_sink) *n_sink = c->seq[0].n_sink;
  return MIXKVQ_OK;
}

int mixkvq_cache_state_seq(const mixkvq_cache* c, int32_t b, int64_t* n_quantized, int32_t* n_residual, int32_t* n_sink) {
  if (!c || b < 0 || b >= c->v.cfg.B) return MIXKVQ_EINVAL;
  if (n_quantized) *n_quantized = c->seq[b].n_quant;
  if (n_residual) *n_residual = c->seq[b].n_res;
  if (n_sink) *n_sink = c->seq[b].n_sink;
  return MIXKVQ_OK;
}

// Is (nq, nr, ns) a state the append rules can produce?
static bool reachable_state(const mixkvq_cache* c, int64_t nq, int32_t nr, int32_t ns) {
  const mixkvq_config& cfg = c->v.cfg;
  const int R = c->Rw;
  if (nq < 0 || nr < 0 || ns < 0 || nq % R != 0 || nq > cfg.T_max || ns > cfg.sink) return false;
  if (ns < cfg.sink && (nq != 0 || nr != 0)) return false;      // the window only fills once the sink is full
  if (cfg.flush_mode == 0 ? nr > R : nr >= R) return false;     // deferred: up to R tokens wait; eager: fewer than R
  if (cfg.flush_mode == 0 && nq > 0 && nr == 0) return false;   // a deferred flush always leaves the token that caused it
  return true;
}

int mixkvq_cache_set_state(mixkvq_cache* c, int64_t n_quantized, int32_t n_residual, int32_t n_sink) {
  if (!c || !reachable_state(c, n_quantized, n_residual, n_sink)) return MIXKVQ_EINVAL;
  for (int b = 0; b < c->v.cfg.B; ++b) c->seq[b] = SeqState{n_quantized, n_residual, n_sink};
  return MIXKVQ_OK;
}

int mixkvq_cache_set_state_seq(mixkvq_cache* c, int32_t b, int64_t n_quantized, int32_t n_residual, int32_t n_sink) {
  if (!c || b < 0 || b >= c->v.cfg.B || !reachable_state(c, n_quantized, n_residual, n_sink)) return MIXKVQ_EINVAL;
  if (c->v.cfg.B > kMaxRaggedB) return MIXKVQ_EINVAL;
  c->seq[b] = SeqState{n_quantized, n_residual, n_sink};
  return MIXKVQ_OK;
}

int mixkvq_select_channels(mixkvq_cache* c, const void* q, int32_t Lq, const int64_t q_strides[3],
                           const void* k, int32_t L, const int64_t k_strides[3], uint8_t* sel, void* stream) {
  if (!c || !k || !k_strides || !sel || L < 1 || Lq < 0) return MIXKVQ_EINVAL;
  if (Lq > 0 && (!q || !q_strides)) return MIXKVQ_EINVAL;
  if (c->v.cfg.k4 + c->v.cfg.k16 == 0) return MIXKVQ_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (Lq > 0) {
    Strides3 qs{q_strides[0], q_strides[1], q_strides[2]};
    MIXKVQ_TRY_HIP(launch_qabs_accumulate(c->v, (const __half*)q, Lq, qs, s));
  }
  Strides3 ks{k_strides[0], k_strides[1], k_strides[2]};
  MIXKVQ_TRY_HIP(launch_select(c->v, (const __half*)k, L, ks, sel, s));
  return MIXKVQ_OK;
}

int mixkvq_select_channels_seq(mixkvq_cache* c, int32_t b, const void* q, int32_t Lq, const int64_t q_strides[2],
                               const void* k, int32_t L, const int64_t k_strides[2], uint8_t* sel, void* stream) {
  if (!c || b < 0 || b >= c->v.cfg.B || !k || !k_strides || !sel || L < 1 || Lq < 0) return MIXKVQ_EINVAL;
  if (Lq > 0 && (!q || !q_strides)) return MIXKVQ_EINVAL;
  if (c->v.cfg.k4 + c->v.cfg.k16 == 0) return MIXKVQ_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const CacheView v = sub_view(c, b, 1);
  if (Lq > 0) {
    Strides3 qs{0, q_strides[0], q_strides[1]};
    MIXKVQ_TRY_HIP(launch_qabs_accumulate(v, (const __half*)q, Lq, qs, s));
  }
  Strides3 ks{0, k_strides[0], k_strides[1]};
  MIXKVQ_TRY_HIP(launch_select(v, (const __half*)k, L, ks, sel, s));
  return MIXKVQ_OK;
}

static int check_kv_args(const void* k_new, const void* v_new, const int64_t* strides, int n_strides) {
  if (!k_new || !v_new || !strides) return MIXKVQ_EINVAL;
  // rows are moved with 16-byte accesses
  if (((uintptr_t)k_new & 15u) || ((uintptr_t)v_new & 15u)) return MIXKVQ_EINVAL;
  for (int i = 0; i < n_strides; ++i)
    if (strides[i] % 8 != 0) return MIXKVQ_EINVAL;
  return MIXKVQ_OK;
}

int mixkvq_quantize_append(mixkvq_cache* c, const void* k_new, const void* v_new, int32_t n_new,
                           const int64_t kv_strides[3], const uint8_t* sel, void* stream) {
  if (!c || n_new < 0) return MIXKVQ_EINVAL;
  if (n_new == 0) return MIXKVQ_OK;
  int rc = check_kv_args(k_new, v_new, kv_strides, 3);
  if (rc != MIXKVQ_OK) return rc;
  const mixkvq_config& cfg = c->v.cfg;
  for (int b = 0; b < cfg.B; ++b) {     // nothing is touched unless every sequence has room
    const AppendPlan pl = plan_append(cfg, c->Rw, c->seq[b], n_new);
    if (c->seq[b].n_quant + pl.F * c->Rw > cfg.T_max) return MIXKVQ_ECAPACITY;
    if (pl.F > (1 << 24)) return MIXKVQ_EINVAL;
  }
  Strides3 kvs{kv_strides[0], kv_strides[1], kv_strides[2]};
  const int ks = cfg.k4 + cfg.k16;
  // Runs of neighbouring sequences in the same state are appended to together (one run while the batch is in
  // lock-step).  The run boundaries are fixed before the first append (a run's append changes its sequences' state),
  // and if a launch fails part-way the token counts of every sequence go back to what they were: the host state
  // never describes an append that was not enqueued as a whole.
  SeqState* before = new (std::nothrow) SeqState[cfg.B];
  if (!before) return MIXKVQ_ENOMEM;
  for (int b = 0; b < cfg.B; ++b) before[b] = c->seq[b];
  rc = MIXKVQ_OK;
  for (int b0 = 0; b0 < cfg.B && rc == MIXKVQ_OK;) {
    int b1 = b0 + 1;
    while (b1 < cfg.B && before[b1] == before[b0]) ++b1;
    rc = append_range(c, b0, b1 - b0, (const __half*)k_new + (int64_t)b0 * kvs.b, (const __half*)v_new + (int64_t)b0 * kvs.b,
                      n_new, kvs, sel ? sel + (size_t)b0 * cfg.Hkv * ks : nullptr, (hipStream_t)stream);
    b0 = b1;
  }
  if (rc != MIXKVQ_OK)
    for (int b = 0; b < cfg.B; ++b) c->seq[b] = before[b];
  delete[] before;
  return rc;
}

int mixkvq_prefill(mixkvq_cache* c, const void* q, int32_t Lq, const int64_t q_strides[3], const void* k, const void* v,
                   int32_t L, const int64_t kv_strides[3], uint8_t* sel, void* stream) {
  if (!c || !k || !v || !kv_strides || !sel || L < 1 || Lq < 0) return MIXKVQ_EINVAL;
  if (Lq > 0 && (!q || !q_strides)) return MIXKVQ_EINVAL;
  if (c->v.cfg.k4 + c->v.cfg.k16 == 0) return MIXKVQ_EINVAL;
  // everything the append could refuse is checked before the scoring pass touches the accumulator
  int rc = check_kv_args(k, v, kv_strides, 3);
  if (rc != MIXKVQ_OK) return rc;
  const mixkvq_config& cfg = c->v.cfg;
  for (int b = 0; b < cfg.B; ++b) {
    const AppendPlan pl = plan_append(cfg, c->Rw, c->seq[b], L);
    if (c->seq[b].n_quant + pl.F * c->Rw > cfg.T_max) return MIXKVQ_ECAPACITY;
    if (pl.F > (1 << 24)) return MIXKVQ_EINVAL;
  }
  hipStream_t s = (hipStream_t)stream;
  if (Lq > 0) {
    Strides3 qs{q_strides[0], q_strides[1], q_strides[2]};
    MIXKVQ_TRY_HIP(launch_qabs_accumulate(c->v, (const __half*)q, Lq, qs, s));
  }
  Strides3 ks{kv_strides[0], kv_strides[1], kv_strides[2]};
  MIXKVQ_TRY_HIP(launch_select(c->v, (const __half*)k, L, ks, sel, s));
  return mixkvq_quantize_append(c, k, v, L, kv_strides, sel, stream);
}

int mixkvq_quantize_append_seq(mixkvq_cache* c, int32_t b, const void* k_new, const void* v_new, int32_t n_new,
                               const int64_t kv_strides[2], const uint8_t* sel, void* stream) {
  if (!c || b < 0 || b >= c->v.cfg.B || n_new < 0) return MIXKVQ_EINVAL;
  if (c->v.cfg.B > kMaxRaggedB) return MIXKVQ_EINVAL;     // such a batch could not be attended over once it is ragged
  if (n_new == 0) return MIXKVQ_OK;
  int rc = check_kv_args(k_new, v_new, kv_strides, 2);
  if (rc != MIXKVQ_OK) return rc;
  const mixkvq_config& cfg = c->v.cfg;
  const AppendPlan pl = plan_append(cfg, c->Rw, c->seq[b], n_new);
  if (c->seq[b].n_quant + pl.F * c->Rw > cfg.T_max) return MIXKVQ_ECAPACITY;
  if (pl.F > (1 << 24)) return MIXKVQ_EINVAL;
  Strides3 kvs{0, kv_strides[0], kv_strides[1]};
  return append_range(c, b, 1, (const __half*)k_new, (const __half*)v_new, n_new, kvs, sel, (hipStream_t)stream);
}

int mixkvq_decode_attention(mixkvq_cache* c, const void* q, void* out, float* lse, float scale,
                            int32_t accumulate_q, void* stream) {
  if (!c || !q || !out) return MIXKVQ_EINVAL;
  const mixkvq_config& cfg = c->v.cfg;
  int n_blocks, n_fp16;
  SeqCounts sc;
  if (!decode_counts(c, 0, &n_blocks, &n_fp16, &sc)) return MIXKVQ_EINVAL;
  if (n_blocks == 0 && n_fp16 == 0) return MIXKVQ_EEMPTY;
  hipStream_t s = (hipStream_t)stream;
  if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)cfg.D);
  MIXKVQ_TRY_HIP(launch_decode(c->v, (const __half*)q, (__half*)out, lse, scale, n_blocks, n_fp16, accumulate_q,
                               NewToken{nullptr, nullptr, {0, 0, 0}, 0}, sc.enabled ? &sc : nullptr, s, c->ev_start,
                               c->ev_stop, &c->last_path));
  return MIXKVQ_OK;
}

int mixkvq_decode_attention_noalloc(mixkvq_cache* c, const void* q, void* out, float* lse, float scale,
                                    int32_t accumulate_q, void* stream) {
  if (!c || !q || !out) return MIXKVQ_EINVAL;
  const mixkvq_config& cfg = c->v.cfg;
  int n_blocks, n_fp16;
  SeqCounts sc;
  if (!decode_counts(c, 0, &n_blocks, &n_fp16, &sc)) return MIXKVQ_EINVAL;
  if (n_blocks == 0 && n_fp16 == 0) return MIXKVQ_EEMPTY;
  if (decode_launch_partials_bytes(c->v, n_blocks, n_fp16) > kNoAllocScratchBytes) return MIXKVQ_ESCRATCH;
  void* part = nullptr;
  MIXKVQ_TRY_HIP(noalloc_scratch(&part));
  hipStream_t s = (hipStream_t)stream;
  if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)cfg.D);
  MIXKVQ_TRY_HIP(launch_decode(c->v, (const __half*)q, (__half*)out, lse, scale, n_blocks, n_fp16, accumulate_q,
                               NewToken{nullptr, nullptr, {0, 0, 0}, 0}, sc.enabled ? &sc : nullptr, s, c->ev_start,
                               c->ev_stop, &c->last_path, (float*)part));
  return MIXKVQ_OK;
}

int mixkvq_decode_step(mixkvq_cache* c, const void* k_new, const void* v_new, const int64_t kv_strides[3],
                       const void* q, void* out, float* lse, float scale, int32_t accumulate_q, void* stream) {
  if (!c || !q || !out) return MIXKVQ_EINVAL;
  int rc = check_kv_args(k_new, v_new, kv_strides, 3);
  if (rc != MIXKVQ_OK) return rc;
  const mixkvq_config& cfg = c->v.cfg;
  const int R = c->Rw;
  // some sequence flushes a block or still feeds its sink, or the sequences differ in length: take the general path
  bool general = !lock_step(c);
  for (int b = 0; b < cfg.B; ++b) {
    const SeqState& st = c->seq[b];
    const int total = st.n_res + 1;
    general |= (cfg.flush_mode == 0 ? total > R : total >= R) || st.n_sink < cfg.sink;
  }
  if (general) {
    // everything the attention call could refuse is checked before the append changes the cache: a batch whose
    // sequences differ in length can only be attended over up to kMaxRaggedB sequences (the counts go by value)
    if (!lock_step(c) && cfg.B > kMaxRaggedB) return MIXKVQ_EINVAL;
    rc = mixkvq_quantize_append(c, k_new, v_new, 1, kv_strides, nullptr, stream);
    if (rc != MIXKVQ_OK) return rc;
    return mixkvq_decode_attention(c, q, out, lse, scale, accumulate_q, stream);
  }
  int n_blocks, n_fp16;
  SeqCounts sc;
  if (!decode_counts(c, 1, &n_blocks, &n_fp16, &sc)) return MIXKVQ_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)cfg.D);
  // the attention launch moves the new rows into the window itself (row = the last fp16 row then in use)
  NewToken nt{(const __half*)k_new, (const __half*)v_new, Strides3{kv_strides[0], kv_strides[1], kv_strides[2]},
              n_fp16 - 1};
  MIXKVQ_TRY_HIP(launch_decode(c->v, (const __half*)q, (__half*)out, lse, scale, n_blocks, n_fp16, accumulate_q, nt,
                               sc.enabled ? &sc : nullptr, s, c->ev_start, c->ev_stop, &c->last_path));
  for (int b = 0; b < cfg.B; ++b) c->seq[b].n_res += 1;
  return MIXKVQ_OK;
}

int mixkvq_cache_set_block_table(mixkvq_cache* c, const int32_t* table) {
  if (!c) return MIXKVQ_EINVAL;
  for (int b = 0; b < c->v.cfg.B; ++b)      // the layout may only change while no block is stored
    if (c->seq[b].n_quant != 0) return MIXKVQ_EINVAL;
  c->v.table = table;
  return MIXKVQ_OK;
}

int mixkvq_set_timing_events(mixkvq_cache* c, void* start_event, void* stop_event) {
  if (!c || ((start_event == nullptr) != (stop_event == nullptr))) return MIXKVQ_EINVAL;
  c->ev_start = (hipEvent_t)start_event;
  c->ev_stop = (hipEvent_t)stop_event;
  return MIXKVQ_OK;
}

int mixkvq_decode_path(const mixkvq_cache* c) { return c ? c->last_path : MIXKVQ_EINVAL; }

const char* mixkvq_strerror(int code) {
  switch (code) {
    case MIXKVQ_OK: return "ok";
    case MIXKVQ_EINVAL: return "invalid argument or unsupported configuration";
    case MIXKVQ_ECAPACITY: return "append would exceed the cache capacity T_max";
    case MIXKVQ_EHIP: return mixkvq::g_hip_msg;
    case MIXKVQ_ENOMEM: return "host allocation failed";
    case MIXKVQ_EEMPTY: return "the cache holds no token";
    case MIXKVQ_ESCRATCH: return "the split-K partials of this launch exceed the library's built-in scratch buffer (8 MiB)";
    case MIXKVQ_ERAGGED: return "the sequences of the batch hold different numbers of tokens: ask per sequence";
    default: return "unknown mixkvq error code";
  }
}

}  // extern "C"
