// Host side of the AdaCGD engine: configuration checks, workspace layout, the
// kernel sequence of one iteration of Algorithm 2, and the C ABI of adacgd.h.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/adacgd.h"
#include "devutil.h"
#include "engine.h"

using namespace adacgd;

namespace {

thread_local char g_err[256] = "";

void set_err(char* buf, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void set_err(char* buf, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, 256, fmt, ap);
  va_end(ap);
}

// bump allocator over the caller's workspace; with base == nullptr it only measures
struct Carver {
  char* base;
  size_t off = 0;
  template <typename T>
  T* take(size_t count) {
    off = (off + 255) & ~size_t(255);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

// omega of the b-bit quantiser on a vector (or block) of `len` coordinates
double quant_omega(int b, double len) {
  const double s = (double)((1 << (b - 1)) - 1);
  return std::fmin(len / (4.0 * s * s), std::sqrt(len) / s);
}

double level_alpha(const adacgd_level& lv, int64_t d) {
  if (lv.kind == ADACGD_TOPK) return (double)lv.param / (double)d;
  if (lv.kind == ADACGD_RANK) return (double)lv.param / (double)lv.block;     // K / min(rows, columns), rows >= columns
  return 1.0 / (1.0 + quant_omega((int)lv.param, lv.kind == ADACGD_QUANT_BLOCK ? (double)lv.block : (double)d));
}

int build_levels(const adacgd_level* in, int m, float zeta, const adacgd_trigger* trig, int64_t d, uint32_t flags,
                 LevelTable* lt, char* err) {
  std::memset(lt, 0, sizeof(*lt));
  if (m < 0 || m > ADACGD_MAX_LEVELS) { set_err(err, "level count %d out of range", m); return ADACGD_ERR_ARG; }
  if (m > 0 && !in) { set_err(err, "level array is null"); return ADACGD_ERR_ARG; }
  if (!trig && (!std::isfinite(zeta) || zeta < 0.f)) { set_err(err, "zeta must be finite and >= 0"); return ADACGD_ERR_ARG; }
  lt->m = m;
  for (int j = 0; j < m; ++j) {
    const float z = trig ? trig[j].zeta : zeta, e = trig ? trig[j].eta : 0.f;
    if (!std::isfinite(z) || z < 0.f || !std::isfinite(e) || e < 0.f) {
      set_err(err, "trigger %d: zeta and eta must be finite and >= 0", j);
      return ADACGD_ERR_ARG;
    }
    lt->tz[j] = (double)z;
    lt->te[j] = (double)e;
  }
  for (int j = 0; j < m; ++j) {
    if (in[j].kind == ADACGD_TOPK) {
      if (in[j].param < 1 || in[j].param > d) {
        set_err(err, "level %d: Top-K needs 1 <= K <= d, got %lld", j + 1, (long long)in[j].param);
        return ADACGD_ERR_ARG;
      }
    } else if (in[j].kind == ADACGD_QUANT || in[j].kind == ADACGD_QUANT_BLOCK) {
      if (in[j].param < 2 || in[j].param > 16) {
        set_err(err, "level %d: quantiser needs 2 <= b <= 16, got %lld", j + 1, (long long)in[j].param);
        return ADACGD_ERR_ARG;
      }
      const int B = in[j].block;
      if (in[j].kind == ADACGD_QUANT_BLOCK && (B < kSeg || B > kWaveTile || (B & (B - 1)) != 0)) {
        set_err(err, "level %d: block length must be a power of two in [64, 2048], got %d", j + 1, B);
        return ADACGD_ERR_ARG;
      }
    } else if (in[j].kind == ADACGD_RANK) {
      const int c = in[j].block;
      if (c != 16 && c != 32 && c != 64) {
        set_err(err, "level %d: Rank-K needs 16, 32 or 64 columns, got %d", j + 1, c);
        return ADACGD_ERR_ARG;
      }
      if (d % c != 0 || d / c < c) {
        set_err(err, "level %d: Rank-K with %d columns needs d to be a multiple of %d and at least %d", j + 1, c, c, c * c);
        return ADACGD_ERR_ARG;
      }
      if (in[j].param < 1 || in[j].param > c) {
        set_err(err, "level %d: Rank-K needs 1 <= K <= columns, got %lld", j + 1, (long long)in[j].param);
        return ADACGD_ERR_ARG;
      }
      if (lt->rcols && lt->rcols != c) {
        set_err(err, "level %d: all Rank-K levels of a level set must use the same number of columns", j + 1);
        return ADACGD_ERR_ARG;
      }
      lt->rcols = c;
    } else {
      set_err(err, "level %d: unknown kind %d", j + 1, in[j].kind);
      return ADACGD_ERR_ARG;
    }
    if (j > 0 && !(flags & ADACGD_FLAG_ANY_LEVEL_ORDER) && level_alpha(in[j - 1], d) > level_alpha(in[j], d)) {
      set_err(err, "levels %d and %d are not ordered by contraction parameter", j, j + 1);
      return ADACGD_ERR_LEVELS;
    }
  }
  // distinct Top-K sizes ascending -> slots (no heap memory: this also runs for adacgd_init_static)
  uint32_t ks[kMaxLevels];
  int nk = 0;
  for (int j = 0; j < m; ++j)
    if (in[j].kind == ADACGD_TOPK) ks[nk++] = (uint32_t)in[j].param;
  std::sort(ks, ks + nk);
  nk = (int)(std::unique(ks, ks + nk) - ks);
  lt->p = nk;
  for (int s = 0; s < lt->p; ++s) lt->K[s] = ks[s];
  for (int j = 0; j < m; ++j) {
    lt->kind[j] = in[j].kind == ADACGD_TOPK ? kTopK : in[j].kind == ADACGD_RANK ? kRank : kQuant;
    if (in[j].kind == ADACGD_RANK) {
      lt->ref[j] = lt->nr;
      lt->rK[lt->nr++] = (int)in[j].param;
    } else if (in[j].kind == ADACGD_TOPK) {
      lt->ref[j] = (int)(std::lower_bound(ks, ks + nk, (uint32_t)in[j].param) - ks);
    } else {
      const int b = (int)in[j].param;
      const int B = in[j].kind == ADACGD_QUANT_BLOCK ? in[j].block : 0;
      int q = -1;
      for (int i = 0; i < lt->nq; ++i)
        if (lt->qbits[i] == b && lt->qblock[i] == B) q = i;
      if (q < 0) {
        q = lt->nq++;
        const double s = (double)((1 << (b - 1)) - 1);
        lt->qbits[q] = b;
        lt->qblock[q] = B;
        lt->nqb += B ? 1 : 0;
        lt->qs[q] = (float)s;
        lt->qdenom[q] = s * (1.0 + quant_omega(b, B ? (double)B : (double)d));
      }
      lt->ref[j] = q;
    }
  }
  return ADACGD_OK;
}

void carve_nodeset(Carver& c, NodeSet& ns) {
  const size_t nn = ns.nn, p = ns.lv.p, nq = ns.lv.nq, m = ns.lv.m, tiles = ns.groups;
  ns.hist0 = c.take<uint32_t>(nn * kBins0);
  ns.gcur = c.take<uint32_t>(nn * 64);   // one cursor per 256 bytes
  ns.sel_hist = c.take<uint32_t>(nn * p * kBins1);
  ns.sel_done = c.take<uint32_t>(nn * p * (kArriveFan + 1) * kCounterStride);
  ns.done = c.take<uint32_t>(nn * (kArriveFan + 1) * kCounterStride);
  ns.agg_done = ns.AS > 1 ? c.take<uint32_t>((size_t)ns.groups * (kArriveFan + 1) * kCounterStride) : nullptr;
  ns.level_hist = c.take<unsigned long long>(m + 2);
  ns.repairs = ns.level_hist ? ns.level_hist + m + 1 : nullptr;   // (null when only measuring)
  // everything up to here must start at zero
  ns.prefix = c.take<uint32_t>(nn * p);
  ns.rank = c.take<uint32_t>(nn * p);
  ns.eqcnt = c.take<uint32_t>(nn * p);
  ns.bmin = c.take<uint32_t>(nn);
  ns.amax = c.take<uint32_t>(nn);
  ns.best = c.take<uint32_t>(nn);
  ns.redo = c.take<uint32_t>(nn);
  ns.skip = c.take<uint32_t>(nn);
  ns.partU = c.take<uint32_t>(nn * ns.G);
  ns.partS = c.take<double>(nn * ns.G);
  ns.partD = c.take<double>(nn * ns.G);
  ns.partEb = c.take<double>(nn * ns.G);
  ns.partQ = c.take<double>(nn * ns.G * nq);
  ns.partStrict = c.take<double>(nn * ns.G2 * p);
  ns.S = c.take<double>(nn);
  ns.D = c.take<double>(nn);
  ns.Eb = c.take<double>(nn);
  ns.qerr = c.take<double>(nn * nq);
  ns.err = c.take<double>(nn * m);
  ns.grp_count = c.take<uint32_t>(nn * tiles);
  ns.cnt_gt = c.take<uint32_t>(nn * p * tiles);
  ns.cnt_eq = c.take<uint32_t>(nn * p * tiles);
  ns.blk_gt = c.take<uint32_t>(nn * p * ns.G2);
  ns.blk_eq = c.take<uint32_t>(nn * p * ns.G2);
  ns.blk_out = c.take<uint32_t>(nn * ns.G2);
  ns.blk_eqb = c.take<uint32_t>(nn * ns.G2);
  ns.grp_off = c.take<uint32_t>(nn * (tiles + 1));
  ns.cand_val = p ? c.take<uint32_t>(nn * (size_t)ns.d) : nullptr;
  ns.cand_off = p ? c.take<uint16_t>(nn * (size_t)ns.d) : nullptr;
  ns.glist = p ? c.take<uint32_t>(nn * (size_t)ns.d) : nullptr;
  ns.level = c.take<int32_t>(nn);
  ns.sel_slot = c.take<int32_t>(nn);
  ns.sel_q = c.take<int32_t>(nn);
  ns.sel_T = c.take<uint32_t>(nn);
  ns.sel_r = c.take<uint32_t>(nn);
  ns.msg_count = c.take<uint32_t>(nn);
  ns.msg_idx = c.take<int32_t>(nn * (size_t)ns.Kcap);
  ns.msg_val = c.take<float>(nn * (size_t)ns.Kcap);
  ns.qcodes = nq ? c.take<int16_t>(nn * (size_t)ns.d) : nullptr;
  ns.qscale = c.take<float>(nn);
  ns.nseg = (int)((ns.d + kSeg - 1) / kSeg);
  ns.segmax = ns.lv.nqb ? c.take<uint32_t>(nn * (size_t)ns.nseg) : nullptr;
  ns.qbscale = ns.lv.nqb ? c.take<float>(nn * (size_t)ns.nseg) : nullptr;
  ns.accbuf = (nq || ns.lv.nr) ? c.take<double>((size_t)ns.d) : nullptr;
  if (ns.lv.nr) {
    const size_t cc = (size_t)ns.lv.rcols * ns.lv.rcols, nr = ns.lv.nr;
    ns.gram_part = c.take<double>(nn * ns.GR * cc);
    ns.rk_lambda = c.take<double>(nn * ns.lv.rcols);
    ns.rk_V = c.take<double>(nn * cc);
    ns.rk_part = c.take<double>(nn * ns.GR * nr);
    ns.rk_err = c.take<double>(nn * nr);
    ns.rdense = c.take<float>(nn * (size_t)ns.d);
    ns.sel_rk = c.take<int32_t>(nn);
  }
  ns.agg_part = ns.AS > 1 ? c.take<double>((size_t)ns.AS * ns.groups * kWaveTile) : nullptr;
}

void shape_nodeset(NodeSet& ns, int nn, int64_t d, bool force_two_pass) {
  ns.nn = nn;
  ns.d = d;
  ns.tiles = (int)((d + kTile - 1) / kTile);
  ns.groups = (int)((d + kWaveTile - 1) / kWaveTile);
  // candidate kernels: about 2048 blocks in all, each owning a contiguous range of groups
  int g2 = (ns.groups + 3) / 4;
  int want2 = (2048 + nn - 1) / nn;
  if (want2 > 512) want2 = 512;
  if (g2 > want2) g2 = want2;
  const int gb = (ns.groups + g2 - 1) / g2;
  ns.G2 = (ns.groups + gb - 1) / gb;
  ns.Kcap = ns.lv.p ? ns.lv.K[ns.lv.p - 1] : 0;
  // One-pass sequence: Top-K levels only, 16-byte vector path, vectors long enough for a
  // 1/32 sample to be informative, and a candidate set that is a minor part of the vector.
  ns.onepass = (!force_two_pass && ns.lv.nq == 0 && ns.lv.p > 0 && d % 4 == 0 && ns.tiles >= 128 &&
                4 * (int64_t)ns.Kcap <= d) ? 1 : 0;
  ns.small = (!force_two_pass && d <= kSmallMax) ? 1 : 0;
  if (ns.lv.nr > 0) {            // Rank-K levels: the general two-pass sequence plus the Rank-K kernels
    ns.onepass = 0;
    ns.small = 0;
    const int64_t rows = d / ns.lv.rcols;
    int64_t gr = (rows + 63) / 64;                 // at least 64 rows per block, about 512 blocks in all, at most 64 per node
    const int64_t cap = std::min<int64_t>(64, std::max<int64_t>(1, 512 / nn));
    ns.GR = (int)std::max<int64_t>(1, std::min(gr, cap));
  }
  // streaming kernels: about 5120 blocks in all for the fused scan (several short blocks per CU
  // interleave better with kernels of another stream than few long ones), about 2048 for the
  // two-pass scan (whose blocks each flush a full histogram); at most 640 per node
  int want = ((ns.onepass ? 5120 : 2048) + nn - 1) / nn;
  if (want > 640) want = 640;
  ns.G = ns.tiles < want ? ns.tiles : want;
  if (ns.G < 1) ns.G = 1;
  if (!ns.onepass) {
    // The two-pass kernels are short: 2048 blocks are resident at once, and a launch that needs a
    // second round of blocks, or whose blocks own unequal numbers of tiles, waits for its stragglers.
    // Hence at most one round, every block with the same number of tiles (the last one may have fewer).
    const int per_block = (ns.tiles + ns.G - 1) / ns.G;
    ns.G = (ns.tiles + per_block - 1) / per_block;
  }
  // select kernels: up to 8 blocks per (Top-K size, node) share a long list (most lists are
  // short and all but a few blocks exit at once, so the launch should stay small)
  // aggregation: one block per group of 2048 coordinates adds every worker's share; short vectors
  // with many workers have too few groups to fill the device, so up to 1024 / groups blocks share
  // a group's workers (at least 8 workers each) and the last one to finish adds their partial sums
  ns.AS = 1;
  if (nn >= 64 && ns.groups < 256) {
    const int by_workers = (nn + 7) / 8, by_groups = 1024 / ns.groups;
    ns.AS = by_workers < by_groups ? by_workers : by_groups;
    if (ns.AS < 1) ns.AS = 1;
  }
  int gz = (int)((d + 262143) / 262144);
  ns.GZ = gz < 1 ? 1 : (gz > 8 ? 8 : gz);
  // one 1024-thread select block is resident per compute unit: keep the launch within one round
  const int one_round = 256 / (nn * (ns.lv.p > 0 ? ns.lv.p : 1));
  if (ns.GZ > one_round) ns.GZ = one_round < 1 ? 1 : one_round;
}

}  // namespace

struct adacgd_ctx {
  int64_t n, d;
  int grad_mode;
  uint32_t flags;
  double gamma;
  uint64_t seed;
  hipStream_t st;        // the caller's stream
  hipStream_t cs;        // stream the next launch goes to
  hipStream_t wst;       // overlap mode: the library's stream for the worker chain, else null
  hipEvent_t ev_worker, ev_agg;
  bool agg_recorded;
  char* ws_base;
  NodeSet W, M;
  bool has_master;
  float* x;
  float* x_next;    // x - gamma g, when the kernel that produced g has already written it (short vectors)
  bool x_next_valid;
  float* g_own;     // master estimator g when the master compresses
  float* gt[2];     // g~^t and g~^{t-1}; cur indexes g~^t
  int cur;
  float* gi;        // [n][d] worker estimators
  float* yb[2];     // [n][d] gradient buffers
  int ycur;         // yb[ycur] holds grad f_i(x^t) unless y_ext is set
  const float* y_ext;
  LogisticData ld;
  int64_t step;
  uint64_t w_zero_bytes, m_zero_bytes;
  char err[256];
  // kernel timing
  bool timing;
  struct Span { int slot; hipEvent_t a, b; };
  std::vector<Span> spans;
  std::vector<hipEvent_t> pool;
  double ms_sum[ADACGD_NUM_KERNELS];
  double ms_cnt[ADACGD_NUM_KERNELS];
  int static_dev = -1;   // >= 0: made by adacgd_init_static on this device (context and workspace are the library's)

  const float* g() const { return has_master ? g_own : gt[cur]; }
  const float* ycurp() const { return y_ext ? y_ext : yb[ycur]; }
};

namespace {

inline bool logistic_mode(int mode) { return mode == ADACGD_GRAD_LOGISTIC || mode == ADACGD_GRAD_LOGISTIC_CSR; }

int validate(const adacgd_config* cfg, LevelTable* wl, LevelTable* ml, char* err) {
  if (!cfg) { set_err(err, "config is null"); return ADACGD_ERR_ARG; }
  if (cfg->n < 1 || cfg->n > 65535) { set_err(err, "n must be in [1, 65535]"); return ADACGD_ERR_ARG; }
  if (cfg->d < 1 || cfg->d >= (int64_t(1) << 31)) { set_err(err, "d must be in [1, 2^31)"); return ADACGD_ERR_ARG; }
  if (cfg->grad_mode < 0 || cfg->grad_mode > 3) { set_err(err, "unknown grad_mode"); return ADACGD_ERR_ARG; }
  if (cfg->init_mode < 0 || cfg->init_mode > 2) { set_err(err, "unknown init_mode"); return ADACGD_ERR_ARG; }
  if (cfg->grad_mode == ADACGD_DIFF_EXTERNAL && cfg->init_mode != ADACGD_INIT_ZERO) {
    set_err(err, "DIFF_EXTERNAL requires INIT_ZERO");
    return ADACGD_ERR_ARG;
  }
  if (!std::isfinite(cfg->gamma)) { set_err(err, "gamma must be finite"); return ADACGD_ERR_ARG; }
  if (cfg->m_worker < 1) { set_err(err, "at least one worker level is required"); return ADACGD_ERR_ARG; }
  int rc = build_levels(cfg->worker_levels, cfg->m_worker, cfg->zeta_worker, cfg->worker_triggers, cfg->d, cfg->flags, wl, err);
  if (rc) return rc;
  if (cfg->init_mode == ADACGD_INIT_COMPRESSED && wl->kind[wl->m - 1] != kTopK) {
    set_err(err, "INIT_COMPRESSED needs a Top-K sparsifier as the last worker level");
    return ADACGD_ERR_ARG;
  }
  rc = build_levels(cfg->master_levels, cfg->m_master, cfg->zeta_master, cfg->master_triggers, cfg->d, cfg->flags, ml, err);
  if (rc) return rc;
  if (logistic_mode(cfg->grad_mode)) {
    if (!cfg->shard_offsets) { set_err(err, "shard_offsets is null"); return ADACGD_ERR_ARG; }
    if (!std::isfinite(cfg->lambda)) { set_err(err, "lambda must be finite"); return ADACGD_ERR_ARG; }
    if (cfg->shard_offsets[0] != 0) { set_err(err, "shard_offsets[0] must be 0"); return ADACGD_ERR_ARG; }
    for (int64_t i = 0; i < cfg->n; ++i)
      if (cfg->shard_offsets[i + 1] <= cfg->shard_offsets[i]) {
        set_err(err, "worker %lld has an empty shard", (long long)i);
        return ADACGD_ERR_ARG;
      }
  }
  if (cfg->grad_mode == ADACGD_GRAD_LOGISTIC_CSR) {
    // The kernels index x and the gradient rows with the stored columns: every one is checked here.
    const int64_t rows = cfg->shard_offsets[cfg->n];
    const int64_t* rp = cfg->csr_row_ptr;
    const int32_t* ci = cfg->csr_col;
    if (rows >= (int64_t(1) << 31)) { set_err(err, "more than 2^31 - 1 rows"); return ADACGD_ERR_ARG; }
    if (!rp) { set_err(err, "csr_row_ptr is null"); return ADACGD_ERR_ARG; }
    if (rp[0] != 0) { set_err(err, "csr_row_ptr[0] must be 0"); return ADACGD_ERR_ARG; }
    for (int64_t l = 0; l < rows; ++l)
      if (rp[l + 1] < rp[l]) { set_err(err, "csr_row_ptr decreases at row %lld", (long long)l); return ADACGD_ERR_ARG; }
    if (rp[rows] > 0 && !ci) { set_err(err, "csr_col is null"); return ADACGD_ERR_ARG; }
    for (int64_t l = 0; l < rows; ++l)
      for (int64_t k = rp[l]; k < rp[l + 1]; ++k)
        if (ci[k] < 0 || ci[k] >= cfg->d || (k > rp[l] && ci[k] <= ci[k - 1])) {
          set_err(err, "row %lld: columns must be in [0, d) and strictly ascending", (long long)l);
          return ADACGD_ERR_ARG;
        }
    for (int64_t i = 0; i < cfg->n; ++i)
      if (rp[cfg->shard_offsets[i + 1]] - rp[cfg->shard_offsets[i]] >= (int64_t(1) << 32)) {
        set_err(err, "worker %lld stores 2^32 or more entries", (long long)i);
        return ADACGD_ERR_ARG;
      }
  }
  return ADACGD_OK;
}

struct Layout {
  float *x, *x_next, *g_own, *gt0, *gt1, *gi, *yb0, *yb1;
  int64_t* offsets;
  int32_t* row_node;
  double* margins;
  double* part;
  uint32_t* col_done;
  int64_t *rp, *wbase;
  int32_t *ci, *trow;
  float *cv, *tval;
  uint32_t* cptr;
  size_t w_zero, m_zero;
};

size_t carve_all(char* base, const adacgd_config* cfg, NodeSet& W, NodeSet& M, LogisticData& ld, Layout& L) {
  Carver c{base};
  const size_t n = cfg->n, d = cfg->d;
  const size_t w0 = c.off;
  carve_nodeset(c, W);
  // the arrays that must be zero come first in carve_nodeset: up to and including level_hist
  L.w_zero = base ? (size_t)((char*)W.prefix - (char*)W.hist0) : 0;
  (void)w0;
  if (M.lv.m > 0) {
    carve_nodeset(c, M);
    L.m_zero = base ? (size_t)((char*)M.prefix - (char*)M.hist0) : 0;
  }
  L.x = c.take<float>(d);
  L.x_next = (W.small || M.lv.m == 0) ? c.take<float>(d) : nullptr;
  L.g_own = M.lv.m > 0 ? c.take<float>(d) : nullptr;
  L.gt0 = c.take<float>(d);
  L.gt1 = c.take<float>(d);
  L.gi = c.take<float>(n * d);
  if (cfg->grad_mode != ADACGD_DIFF_EXTERNAL) {
    L.yb0 = c.take<float>(n * d);
    const bool second = logistic_mode(cfg->grad_mode) || !(cfg->flags & ADACGD_FLAG_RETAIN_EXT);
    L.yb1 = second ? c.take<float>(n * d) : nullptr;
  } else {
    L.yb0 = L.yb1 = nullptr;
  }
  if (logistic_mode(cfg->grad_mode)) {
    const size_t rows = cfg->shard_offsets[n];
    L.offsets = c.take<int64_t>(n + 1);
    L.row_node = c.take<int32_t>(rows);
    L.margins = c.take<double>(rows);
    L.part = ld.row_chunks > 1 ? c.take<double>(n * ld.row_chunks * d) : nullptr;
    L.col_done = ld.row_chunks > 1 ? c.take<uint32_t>(n * ((d + 63) / 64)) : nullptr;
  } else {
    L.offsets = nullptr; L.row_node = nullptr; L.margins = nullptr; L.part = nullptr; L.col_done = nullptr;
  }
  if (ld.csr) {
    const size_t rows = cfg->shard_offsets[n], nnz = (size_t)ld.nnz;
    L.rp = c.take<int64_t>(rows + 1);
    L.wbase = c.take<int64_t>(n + 1);
    L.cptr = c.take<uint32_t>(n * (d + 1));
    L.ci = c.take<int32_t>(nnz);
    L.trow = c.take<int32_t>(nnz);
    L.cv = ld.binary ? nullptr : c.take<float>(nnz);
    L.tval = ld.binary ? nullptr : c.take<float>(nnz);
  }
  return (c.off + 255) & ~size_t(255);
}

void shape_logistic(const adacgd_config* cfg, LogisticData& ld) {
  std::memset(&ld, 0, sizeof(ld));
  if (!logistic_mode(cfg->grad_mode)) return;
  ld.rows = cfg->shard_offsets[cfg->n];
  if (cfg->grad_mode == ADACGD_GRAD_LOGISTIC_CSR) {
    ld.csr = 1;
    ld.binary = cfg->csr_val == nullptr;
    ld.nnz = cfg->csr_row_ptr[ld.rows];
    ld.row_chunks = 1;
    ld.lambda = (double)cfg->lambda;
    return;
  }
  int64_t mx = 0;
  for (int64_t i = 0; i < cfg->n; ++i) mx = std::max<int64_t>(mx, cfg->shard_offsets[i + 1] - cfg->shard_offsets[i]);
  ld.max_rows = mx;
  int64_t chunks = (mx + 255) / 256;    // about 256 rows per block (64 per wavefront) ...
  if (chunks > 64) chunks = 64;         // ... but a bounded number of partial sums
  ld.row_chunks = (int)chunks;
  ld.lambda = (double)cfg->lambda;
}

#define HIPCHK(ctx, call)                                                            \
  do {                                                                               \
    hipError_t e_ = (call);                                                          \
    if (e_ != hipSuccess) {                                                          \
      set_err((ctx)->err, "%s failed: %s", #call, hipGetErrorString(e_));            \
      return ADACGD_ERR_DEVICE;                                                      \
    }                                                                                \
  } while (0)

template <typename F>
int timed(adacgd_ctx* c, int slot, F&& f) {
  hipEvent_t a = nullptr, b = nullptr;
  if (c->timing) {
    for (hipEvent_t* e : {&a, &b}) {
      if (!c->pool.empty()) { *e = c->pool.back(); c->pool.pop_back(); }
      else HIPCHK(c, hipEventCreate(e));
    }
    HIPCHK(c, hipEventRecord(a, c->cs));
  }
  hipError_t e = f();
  if (e != hipSuccess) {
    set_err(c->err, "kernel launch (slot %d) failed: %s", slot, hipGetErrorString(e));
    return ADACGD_ERR_DEVICE;
  }
  if (c->timing) {
    HIPCHK(c, hipEventRecord(b, c->cs));
    c->spans.push_back({slot, a, b});
  }
  return ADACGD_OK;
}

int drain_spans(adacgd_ctx* c) {
  for (auto& s : c->spans) {
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, s.a, s.b));
    c->ms_sum[s.slot] += ms;
    c->ms_cnt[s.slot] += 1.0;
    c->pool.push_back(s.a);
    c->pool.push_back(s.b);
  }
  c->spans.clear();
  return ADACGD_OK;
}

// One application of the AdaCGD compressor to every node of a set, on the stream c->cs.
// `before_tally`, if set, is an event the stream waits for before the kernels that overwrite the
// message tables (tally, compact, qapply): in overlap mode the previous step's aggregation, which
// reads them on the other stream, must have finished.
int compress(adacgd_ctx* c, NodeSet& ns, const PassArgs& a, int slot0, hipEvent_t before_tally) {
  int rc;
  if (ns.small) {      // short vectors: the whole step of a node in one block (timed in the scan's slot)
    if (before_tally) HIPCHK(c, hipStreamWaitEvent(c->cs, before_tally, 0));
    return timed(c, slot0 + 1, [&] { return launch_small(ns, a, c->cs); });
  }
  if (ns.onepass) {
    if ((rc = timed(c, slot0 + 0, [&] { return launch_sample(ns, a, c->cs); }))) return rc;
    if ((rc = timed(c, slot0 + 1, [&] { return launch_scanx(ns, a, false, c->cs); }))) return rc;
    // repair pass: does nothing unless the sampled cut left fewer candidates than the largest K
    if ((rc = timed(c, slot0 + 2, [&] { return launch_scanx(ns, a, true, c->cs); }))) return rc;
  } else {
    if ((rc = timed(c, slot0 + 1, [&] { return launch_scan(ns, a, c->cs); }))) return rc;
    if ((rc = timed(c, slot0 + 2, [&] { return launch_filter(ns, a, c->cs); }))) return rc;
  }
  if (ns.lv.nr > 0) {
    const int rank_slot = slot0 == ADACGD_K_W_SAMPLE ? ADACGD_K_W_RANK : ADACGD_K_M_RANK;
    const int eig_slot = slot0 == ADACGD_K_W_SAMPLE ? ADACGD_K_W_EIG : ADACGD_K_M_EIG;
    if ((rc = timed(c, rank_slot, [&] { return launch_rank_gram(ns, a, c->cs); }))) return rc;
    if ((rc = timed(c, eig_slot, [&] { return launch_rank_eig(ns, a, c->cs); }))) return rc;
    if ((rc = timed(c, rank_slot, [&] { return launch_rank_errors(ns, a, c->cs); }))) return rc;
  }
  if (ns.lv.p > 0 && (rc = timed(c, slot0 + 3, [&] { return launch_gather(ns, c->cs); }))) return rc;
  if (ns.lv.p > 0 && (rc = timed(c, slot0 + 4, [&] { return launch_select(ns, c->cs); }))) return rc;
  if (before_tally) HIPCHK(c, hipStreamWaitEvent(c->cs, before_tally, 0));
  if ((rc = timed(c, slot0 + 5, [&] { return launch_tally(ns, c->cs); }))) return rc;
  if (ns.lv.p > 0 && (rc = timed(c, slot0 + 6, [&] { return launch_compact(ns, a, c->cs); }))) return rc;
  if (ns.lv.nq > 0 && (rc = timed(c, slot0 + 7, [&] { return launch_qapply(ns, a, c->cs); }))) return rc;
  if (ns.lv.nr > 0 && (rc = timed(c, slot0 == ADACGD_K_W_SAMPLE ? ADACGD_K_W_RANK : ADACGD_K_M_RANK,
                                  [&] { return launch_rank_apply(ns, a, c->cs); }))) return rc;
  return ADACGD_OK;
}

int gradients(adacgd_ctx* c, float* out) {
  int rc;
  if ((rc = timed(c, ADACGD_K_GRAD_MARGIN, [&] { return launch_grad_margins(c->ld, c->x, c->d, c->cs); }))) return rc;
  return timed(c, ADACGD_K_GRAD_COLS, [&] { return launch_grad_cols(c->ld, c->x, out, (int)c->n, c->d, c->cs); });
}

int one_step(adacgd_ctx* c, const float* ext, const double* extD) {
  int rc;
  // Overlap mode: the worker chain runs on the library's own stream, the server chain (iterate
  // update, aggregation, master compression) on the caller's; the worker chain of step t+1 does not
  // depend on the server chain of step t (gradients are supplied), so the two run concurrently.
  const bool ov = c->wst != nullptr;
  c->cs = c->st;
  // x^{t+1} = x^t - gamma g^t (already there if the kernel that finished g^t wrote it as well)
  if (c->x_next_valid) {
    std::swap(c->x, c->x_next);
    c->x_next_valid = false;
  } else if ((rc = timed(c, ADACGD_K_XUPDATE, [&] { return launch_xupdate(c->x, c->g(), c->gamma, c->d, c->cs); }))) {
    return rc;
  }
  // Short vectors, few workers, Top-K messages only: the one-block kernel of the workers also does the
  // aggregation (its last block), and the kernel that finishes g the next iterate update.
  const bool serve = c->W.small && c->W.lv.nq == 0 && c->W.lv.nr == 0 && c->n <= kSmallServeMax && !ov;
  PassArgs a{};
  a.h = c->gi;
  a.seed = c->seed;
  a.step = (uint32_t)c->step;
  a.node_flag = 0;
  if (logistic_mode(c->grad_mode)) {
    float* fresh = c->yb[c->ycur ^ 1];
    if ((rc = gradients(c, fresh))) return rc;
    a.x = fresh;
    a.y = c->yb[c->ycur];
  } else if (c->grad_mode == ADACGD_GRAD_EXTERNAL) {
    a.x = ext;
    a.y = c->ycurp();
    a.ycopy = (c->flags & ADACGD_FLAG_RETAIN_EXT) ? nullptr : c->yb[c->ycur ^ 1];
  } else {
    a.x = ext;
    a.diff = 1;
    a.extD = extD;
  }
  float* gt_old = c->gt[c->cur];
  float* gt_new = c->gt[c->cur ^ 1];
  if (serve) {
    a.agg_old = gt_old;
    a.agg_new = gt_new;
    if (!c->has_master) {
      a.xu_x = c->x;
      a.xu_out = c->x_next;
      a.xu_gamma = c->gamma;
      c->x_next_valid = true;
    }
  }
  // g~_i^{t+1} = C^AC_{g~_i^t, grad f_i(x^t)}(grad f_i(x^{t+1}))
  if (ov) c->cs = c->wst;
  if ((rc = compress(c, c->W, a, ADACGD_K_W_SAMPLE, ov && c->agg_recorded ? c->ev_agg : nullptr))) return rc;
  if (ov) {
    HIPCHK(c, hipEventRecord(c->ev_worker, c->wst));
    c->cs = c->st;
    HIPCHK(c, hipStreamWaitEvent(c->st, c->ev_worker, 0));
  }
  if (logistic_mode(c->grad_mode)) {
    c->ycur ^= 1;
  } else if (c->grad_mode == ADACGD_GRAD_EXTERNAL) {
    if (c->flags & ADACGD_FLAG_RETAIN_EXT) c->y_ext = ext;
    else c->ycur ^= 1;
  }
  // g~^{t+1} = g~^t + (1/n) sum_i messages
  if (!serve) {
    IterateUpdate xu{};
    if (!c->has_master) {           // g is g~: the aggregation also writes the next iterate
      xu.x = c->x;
      xu.out = c->x_next;
      xu.gamma = c->gamma;
      c->x_next_valid = true;
    }
    if ((rc = timed(c, ADACGD_K_AGGREGATE, [&] { return launch_aggregate(c->W, gt_old, gt_new, xu, c->cs); }))) return rc;
  }
  if (ov) {
    HIPCHK(c, hipEventRecord(c->ev_agg, c->st));
    c->agg_recorded = true;
  }
  c->cur ^= 1;
  // g^{t+1} = C^AC_{g^t, g~^t}(g~^{t+1})
  if (c->has_master) {
    PassArgs m{};
    m.x = gt_new;
    m.h = c->g_own;
    m.y = gt_old;
    m.seed = c->seed;
    m.step = (uint32_t)c->step;
    m.node_flag = 0x80000000u;
    if (c->M.small) {
      m.xu_x = c->x;
      m.xu_out = c->x_next;
      m.xu_gamma = c->gamma;
      c->x_next_valid = true;
    }
    if ((rc = compress(c, c->M, m, ADACGD_K_M_SAMPLE, nullptr))) return rc;
  }
  c->step += 1;
  return ADACGD_OK;
}

uint64_t ceil_log2(uint64_t v) {
  uint64_t b = 0;
  while ((uint64_t(1) << b) < v) ++b;
  return b;
}

void comm_of(const NodeSet& ns, const unsigned long long* hist, uint64_t copies, uint64_t* values, uint64_t* bits) {
  const uint64_t idb = std::max<uint64_t>(1, ceil_log2((uint64_t)ns.lv.m + 1));
  const uint64_t ib = std::max<uint64_t>(1, ceil_log2((uint64_t)ns.d));
  *values = 0;
  *bits = 0;
  for (int j = 0; j <= ns.lv.m; ++j) {
    uint64_t v = 0, b = idb;
    if (j > 0) {
      if (ns.lv.kind[j - 1] == kTopK) {
        v = ns.lv.K[ns.lv.ref[j - 1]];
        b += v * (32 + ib);
      } else if (ns.lv.kind[j - 1] == kRank) {          // K scaled left factors of d/c floats and K right factors of c
        v = (uint64_t)ns.lv.rK[ns.lv.ref[j - 1]] * ((uint64_t)ns.d / ns.lv.rcols + ns.lv.rcols);
        b += 32 * v;
      } else {
        const int q = ns.lv.ref[j - 1];
        v = (uint64_t)ns.d;
        const uint64_t nscales = ns.lv.qblock[q] ? ((uint64_t)ns.d + ns.lv.qblock[q] - 1) / ns.lv.qblock[q] : 1;
        b += (uint64_t)ns.d * ns.lv.qbits[q] + 32 * nscales;
      }
    }
    *values += hist[j] * v * copies;
    *bits += hist[j] * b * copies;
  }
}

// ---------------------------------------------------------------------------
// adacgd_init_static: workspace and context in memory the library owns from load time.
// `scratch` is the device array; in host code its name is only a handle for
// hipGetSymbolAddress, never a device address.  Each device has its own copy at its own
// address, resolved once per device (with that device current) and kept in its slot; all
// host code below uses slot.ptr.  (The compiler gives the device-side symbol of a static variable
// global binding because host code names it; the runtime finds it by that name.  A `used`
// attribute would keep the symbol local, and the lookup would then fail.)
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[ADACGD_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
struct StaticSlot {
  void* ptr = nullptr;      // device address of `scratch` on this device
  bool in_use = false;      // a context made by adacgd_init_static is alive on this device
  alignas(adacgd_ctx) unsigned char ctx_mem[sizeof(adacgd_ctx)];
};
StaticSlot g_slots[kMaxDevices];
std::mutex g_slots_mu;

// Ends a context: the heap object of adacgd_init, or the one in the static slot of adacgd_init_static
// (`free_slot`: also hand the device's static workspace back; a failing adacgd_init_static does that itself).
void release_ctx(adacgd_ctx* c, bool free_slot) {
  if (c->static_dev >= 0) {
    StaticSlot& sl = g_slots[c->static_dev];
    c->~adacgd_ctx();
    if (free_slot) {
      std::lock_guard<std::mutex> lk(g_slots_mu);
      sl.in_use = false;
    }
  } else {
    delete c;
  }
}

}  // namespace

static int init_impl(const adacgd_config* cfg, adacgd_ctx** out, int static_dev);

extern "C" {

int adacgd_workspace_bytes(const adacgd_config* cfg, int64_t* bytes) {
  LevelTable wl, ml;
  int rc = validate(cfg, &wl, &ml, g_err);
  if (rc) return rc;
  if (!bytes) { set_err(g_err, "bytes is null"); return ADACGD_ERR_ARG; }
  NodeSet W{}, M{};
  W.lv = wl; M.lv = ml;
  shape_nodeset(W, (int)cfg->n, cfg->d, (cfg->flags & ADACGD_FLAG_TWO_PASS) != 0);
  shape_nodeset(M, 1, cfg->d, (cfg->flags & ADACGD_FLAG_TWO_PASS) != 0);
  LogisticData ld;
  shape_logistic(cfg, ld);
  Layout L{};
  *bytes = (int64_t)carve_all(nullptr, cfg, W, M, ld, L);
  return ADACGD_OK;
}

int adacgd_init(const adacgd_config* cfg, adacgd_ctx** out) { return init_impl(cfg, out, -1); }

int adacgd_init_static(const adacgd_config* cfg, adacgd_ctx** out) {
  if (!cfg) { set_err(g_err, "config is null"); return ADACGD_ERR_ARG; }
  if (!out) { set_err(g_err, "out is null"); return ADACGD_ERR_ARG; }
  *out = nullptr;
  if (cfg->grad_mode != ADACGD_GRAD_EXTERNAL && cfg->grad_mode != ADACGD_DIFF_EXTERNAL) {
    set_err(g_err, "adacgd_init_static takes GRAD_EXTERNAL or DIFF_EXTERNAL only (the logistic modes build host tables)");
    return ADACGD_ERR_STATE;
  }
  if (cfg->flags & (ADACGD_FLAG_OVERLAP | ADACGD_FLAG_KERNEL_TIMING)) {
    set_err(g_err, "adacgd_init_static does not take FLAG_OVERLAP or FLAG_KERNEL_TIMING (they create a stream and events)");
    return ADACGD_ERR_STATE;
  }
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { set_err(g_err, "hipGetDevice failed: %s", hipGetErrorString(e)); return ADACGD_ERR_DEVICE; }
  if (dev < 0 || dev >= kMaxDevices) { set_err(g_err, "device index %d out of range", dev); return ADACGD_ERR_DEVICE; }
  {
    std::lock_guard<std::mutex> lk(g_slots_mu);
    StaticSlot& sl = g_slots[dev];
    if (sl.in_use) {
      set_err(g_err, "device %d: the static workspace is in use by another context (destroy it first)", dev);
      return ADACGD_ERR_STATE;
    }
    if (!sl.ptr) {        // once per device, with that device current
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) {
        set_err(g_err, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
        return ADACGD_ERR_DEVICE;
      }
      sl.ptr = p;
    }
    sl.in_use = true;
  }
  const int rc = init_impl(cfg, out, dev);
  if (rc != ADACGD_OK) {
    std::lock_guard<std::mutex> lk(g_slots_mu);
    g_slots[dev].in_use = false;
  }
  return rc;
}

}  // extern "C"

// Input line of Algorithm 1.  static_dev < 0: the caller's workspace and a heap context; otherwise the
// static workspace and context slot of that device (no memory is allocated on either side).
static int init_impl(const adacgd_config* cfg, adacgd_ctx** out, int static_dev) {
  LevelTable wl, ml;
  int rc = validate(cfg, &wl, &ml, g_err);
  if (rc) return rc;
  if (!out) { set_err(g_err, "out is null"); return ADACGD_ERR_ARG; }
  *out = nullptr;
  if (!cfg->x0) { set_err(g_err, "x0 is null"); return ADACGD_ERR_ARG; }
  if (cfg->grad_mode == ADACGD_GRAD_LOGISTIC && (!cfg->A || !cfg->labels)) {
    set_err(g_err, "A / labels is null");
    return ADACGD_ERR_ARG;
  }
  if (cfg->grad_mode == ADACGD_GRAD_LOGISTIC_CSR && !cfg->labels) {
    set_err(g_err, "labels is null");
    return ADACGD_ERR_ARG;
  }
  if (cfg->grad_mode == ADACGD_GRAD_EXTERNAL && !cfg->grad0) {
    set_err(g_err, "grad0 is required in GRAD_EXTERNAL mode");
    return ADACGD_ERR_ARG;
  }
  void* const workspace = static_dev >= 0 ? g_slots[static_dev].ptr : cfg->workspace;
  const int64_t workspace_bytes = static_dev >= 0 ? (int64_t)ADACGD_STATIC_WORKSPACE_BYTES : cfg->workspace_bytes;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) {
    set_err(g_err, "workspace is null or not 256-byte aligned");
    return ADACGD_ERR_ALLOC;
  }
  adacgd_ctx* c = static_dev >= 0 ? new (g_slots[static_dev].ctx_mem) adacgd_ctx() : new (std::nothrow) adacgd_ctx();
  if (!c) { set_err(g_err, "out of host memory"); return ADACGD_ERR_ALLOC; }
  c->static_dev = static_dev;
  c->n = cfg->n; c->d = cfg->d; c->grad_mode = cfg->grad_mode; c->flags = cfg->flags;
  c->gamma = (double)cfg->gamma; c->seed = cfg->seed; c->st = (hipStream_t)cfg->stream;
  c->ws_base = (char*)workspace;
  c->has_master = cfg->m_master > 0;
  c->timing = (cfg->flags & ADACGD_FLAG_KERNEL_TIMING) != 0;
  c->step = 0; c->cur = 0; c->ycur = 0; c->y_ext = nullptr; c->err[0] = 0;
  c->cs = c->st; c->wst = nullptr; c->ev_worker = nullptr; c->ev_agg = nullptr; c->agg_recorded = false;
  std::memset(c->ms_sum, 0, sizeof(c->ms_sum));
  std::memset(c->ms_cnt, 0, sizeof(c->ms_cnt));
  c->W = NodeSet{}; c->M = NodeSet{};
  c->W.lv = wl; c->M.lv = ml;
  shape_nodeset(c->W, (int)cfg->n, cfg->d, (cfg->flags & ADACGD_FLAG_TWO_PASS) != 0);
  shape_nodeset(c->M, 1, cfg->d, (cfg->flags & ADACGD_FLAG_TWO_PASS) != 0);
  shape_logistic(cfg, c->ld);
  Layout L{};
  const size_t need = carve_all(c->ws_base, cfg, c->W, c->M, c->ld, L);
  if ((int64_t)need > workspace_bytes) {
    if (static_dev >= 0)
      set_err(g_err, "configuration needs %zu bytes of workspace, the static workspace holds %lld: use adacgd_init",
              need, (long long)workspace_bytes);
    else
      set_err(g_err, "workspace too small: need %zu bytes, got %lld", need, (long long)workspace_bytes);
    release_ctx(c, false);
    return ADACGD_ERR_ALLOC;
  }
  c->x = L.x; c->x_next = L.x_next; c->x_next_valid = false; c->g_own = L.g_own; c->gt[0] = L.gt0; c->gt[1] = L.gt1; c->gi = L.gi;
  c->yb[0] = L.yb0; c->yb[1] = L.yb1;
  c->ld.A = cfg->A; c->ld.labels = cfg->labels; c->ld.offsets = L.offsets; c->ld.row_node = L.row_node;
  c->ld.margins = L.margins; c->ld.part = L.part; c->ld.col_done = L.col_done;
  if (c->ld.csr) {
    c->ld.rp = L.rp; c->ld.wbase = L.wbase; c->ld.cptr = L.cptr; c->ld.ci = L.ci; c->ld.trow = L.trow;
    c->ld.cv = L.cv; c->ld.tval = L.tval;
  }

  auto fail = [&](int code) { std::memcpy(g_err, c->err, sizeof(g_err)); release_ctx(c, false); return code; };
#define INITCHK(call)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      set_err(c->err, "%s failed: %s", #call, hipGetErrorString(e_));                       \
      return fail(ADACGD_ERR_DEVICE);                                                       \
    }                                                                                       \
  } while (0)

  const size_t nd = (size_t)c->n * (size_t)c->d;
  INITCHK(launch_fill_u32((uint32_t*)c->W.hist0, 0u, L.w_zero / 4, c->st));
  if (c->has_master) INITCHK(launch_fill_u32((uint32_t*)c->M.hist0, 0u, L.m_zero / 4, c->st));
  INITCHK(launch_copy_f32(c->x, cfg->x0, (size_t)c->d, c->st));
  if (c->ld.csr) {
    // Device copy of the rows, and of every shard sorted by column (a counting sort that keeps
    // the row order inside a column), one worker at a time.
    const int64_t rows = c->ld.rows, d = c->d;
    const int64_t* rp = cfg->csr_row_ptr;
    const size_t nnz = (size_t)c->ld.nnz;
    INITCHK(hipMemcpy(L.rp, rp, (size_t)(rows + 1) * sizeof(int64_t), hipMemcpyHostToDevice));
    if (nnz) {
      INITCHK(hipMemcpy(L.ci, cfg->csr_col, nnz * sizeof(int32_t), hipMemcpyHostToDevice));
      if (L.cv) INITCHK(hipMemcpy(L.cv, cfg->csr_val, nnz * sizeof(float), hipMemcpyHostToDevice));
    }
    std::vector<int64_t> wbase((size_t)c->n + 1);
    std::vector<uint32_t> cp((size_t)d + 1), cur((size_t)d);
    std::vector<int32_t> trow;
    std::vector<float> tval;
    for (int64_t i = 0; i < c->n; ++i) {
      const int64_t r0 = cfg->shard_offsets[i], r1 = cfg->shard_offsets[i + 1];
      const int64_t e0 = rp[r0], e1 = rp[r1];
      wbase[(size_t)i] = e0;
      std::fill(cp.begin(), cp.end(), 0u);
      for (int64_t k = e0; k < e1; ++k) ++cp[(size_t)cfg->csr_col[k] + 1];
      for (int64_t j = 0; j < d; ++j) cp[(size_t)j + 1] += cp[(size_t)j];
      std::copy(cp.begin(), cp.end() - 1, cur.begin());
      trow.resize((size_t)(e1 - e0));
      if (L.tval) tval.resize((size_t)(e1 - e0));
      for (int64_t l = r0; l < r1; ++l)
        for (int64_t k = rp[l]; k < rp[l + 1]; ++k) {
          const uint32_t at = cur[(size_t)cfg->csr_col[k]]++;
          trow[at] = (int32_t)l;
          if (L.tval) tval[at] = cfg->csr_val[k];
        }
      INITCHK(hipMemcpy(L.cptr + (size_t)i * (size_t)(d + 1), cp.data(), cp.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
      if (e1 > e0) {
        INITCHK(hipMemcpy(L.trow + e0, trow.data(), trow.size() * sizeof(int32_t), hipMemcpyHostToDevice));
        if (L.tval) INITCHK(hipMemcpy(L.tval + e0, tval.data(), tval.size() * sizeof(float), hipMemcpyHostToDevice));
      }
    }
    wbase[(size_t)c->n] = rp[rows];
    INITCHK(hipMemcpy(L.wbase, wbase.data(), wbase.size() * sizeof(int64_t), hipMemcpyHostToDevice));
  }
  if (L.col_done) INITCHK(launch_fill_u32(L.col_done, 0u, (size_t)c->n * (size_t)((c->d + 63) / 64), c->st));
  if (logistic_mode(cfg->grad_mode)) {
    std::vector<int32_t> rn((size_t)c->ld.rows);
    for (int64_t i = 0; i < c->n; ++i)
      for (int64_t l = cfg->shard_offsets[i]; l < cfg->shard_offsets[i + 1]; ++l) rn[(size_t)l] = (int32_t)i;
    INITCHK(hipMemcpyAsync(L.offsets, cfg->shard_offsets, (size_t)(c->n + 1) * sizeof(int64_t), hipMemcpyHostToDevice,
                           c->st));
    INITCHK(hipMemcpyAsync(L.row_node, rn.data(), rn.size() * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
    INITCHK(hipStreamSynchronize(c->st));   // rn goes out of scope
    INITCHK(launch_grad_margins(c->ld, c->x, c->d, c->st));
    INITCHK(launch_grad_cols(c->ld, c->x, c->yb[0], (int)c->n, c->d, c->st));
  } else if (cfg->grad_mode == ADACGD_GRAD_EXTERNAL) {
    INITCHK(launch_copy_f32(c->yb[0], cfg->grad0, nd, c->st));
  }
  if (cfg->init_mode == ADACGD_INIT_FULLGRAD) INITCHK(launch_copy_f32(c->gi, c->yb[0], nd, c->st));
  else INITCHK(launch_fill_u32((uint32_t*)c->gi, 0u, nd, c->st));
  if (cfg->init_mode == ADACGD_INIT_COMPRESSED) {
    // g~_i^0 = C_m(grad f_i(x^0)) (the CLAG / EF21 start, Section 2.3): one application of the compressor
    // with the last level as the only one, h = 0 (so v is the gradient, bit for bit), applied unconditionally
    // (a zero gradient still selects K zeros) and the selected values stored as they are, so that a selected
    // -0 stays -0
    NodeSet one = c->W;
    const LevelTable& lv = c->W.lv;
    one.lv.m = 1;
    one.lv.kind[0] = kTopK;
    one.lv.ref[0] = lv.ref[lv.m - 1];
    one.lv.tz[0] = 0.0;
    one.lv.te[0] = 0.0;
    PassArgs a{};
    a.x = c->yb[0];
    a.y = c->yb[0];
    a.h = c->gi;
    a.seed = c->seed;
    a.assign = 1;
    const bool timing = c->timing;
    c->timing = false;
    const int rc1 = compress(c, one, a, ADACGD_K_W_SAMPLE, nullptr);
    c->timing = timing;
    if (rc1) return fail(rc1);
    // the counters of that application do not belong to the run
    INITCHK(launch_fill_u32((uint32_t*)c->W.level_hist, 0u, (size_t)(lv.m + 2) * 2, c->st));
  }
  INITCHK(launch_mean(c->gi, c->gt[0], c->gt[1], c->g_own, (int)c->n, c->d, c->st));
  // message tables start empty
  INITCHK(launch_fill_u32((uint32_t*)c->W.sel_slot, 0xFFFFFFFFu, (size_t)c->n, c->st));
  INITCHK(launch_fill_u32((uint32_t*)c->W.sel_q, 0xFFFFFFFFu, (size_t)c->n, c->st));
  if (c->W.lv.nr) INITCHK(launch_fill_u32((uint32_t*)c->W.sel_rk, 0xFFFFFFFFu, (size_t)c->n, c->st));
  if (c->has_master && c->M.lv.nr) INITCHK(launch_fill_u32((uint32_t*)c->M.sel_rk, 0xFFFFFFFFu, 1, c->st));
  INITCHK(launch_fill_u32(c->W.msg_count, 0u, (size_t)c->n, c->st));
  INITCHK(launch_fill_u32((uint32_t*)c->W.level, 0u, (size_t)c->n, c->st));
  if (c->has_master) {
    INITCHK(launch_fill_u32((uint32_t*)c->M.sel_slot, 0xFFFFFFFFu, 1, c->st));
    INITCHK(launch_fill_u32((uint32_t*)c->M.sel_q, 0xFFFFFFFFu, 1, c->st));
    INITCHK(launch_fill_u32(c->M.msg_count, 0u, 1, c->st));
    INITCHK(launch_fill_u32((uint32_t*)c->M.level, 0u, 1, c->st));
  }
  if ((cfg->flags & ADACGD_FLAG_OVERLAP) && !logistic_mode(cfg->grad_mode)) {
    INITCHK(hipStreamSynchronize(c->st));     // the worker stream starts from a finished initial state
    INITCHK(hipStreamCreateWithFlags(&c->wst, hipStreamNonBlocking));
    INITCHK(hipEventCreateWithFlags(&c->ev_worker, hipEventDisableTiming));
    INITCHK(hipEventCreateWithFlags(&c->ev_agg, hipEventDisableTiming));
  }
#undef INITCHK
  *out = c;
  return ADACGD_OK;
}

extern "C" {

int adacgd_step(adacgd_ctx* c, const float* ext, const double* ext_D, int32_t nsteps) {
  if (!c) return ADACGD_ERR_ARG;
  if (nsteps < 0) { set_err(c->err, "nsteps < 0"); return ADACGD_ERR_ARG; }
  if (logistic_mode(c->grad_mode)) {
    if (ext || ext_D) { set_err(c->err, "LOGISTIC mode takes no external arrays"); return ADACGD_ERR_STATE; }
  } else {
    if (!ext) { set_err(c->err, "ext is null"); return ADACGD_ERR_ARG; }
    if (reinterpret_cast<uintptr_t>(ext) & 15u) { set_err(c->err, "ext is not 16-byte aligned"); return ADACGD_ERR_ARG; }
    if (c->grad_mode == ADACGD_DIFF_EXTERNAL && !ext_D) { set_err(c->err, "ext_D is null"); return ADACGD_ERR_ARG; }
    if (c->grad_mode == ADACGD_GRAD_EXTERNAL && ext_D) {
      set_err(c->err, "ext_D is only used in DIFF_EXTERNAL mode");
      return ADACGD_ERR_STATE;
    }
  }
  const size_t nd = (size_t)c->n * (size_t)c->d;
  for (int32_t s = 0; s < nsteps; ++s) {
    int rc = one_step(c, ext ? ext + (size_t)s * nd : nullptr, ext_D ? ext_D + (size_t)s * c->n : nullptr);
    if (rc) return rc;
  }
  return ADACGD_OK;
}

int adacgd_state(adacgd_ctx* c, int32_t field, void* dst, int64_t dst_bytes, int32_t dst_on_device) {
  if (!c) return ADACGD_ERR_ARG;
  if (!dst && dst_bytes != 0) { set_err(c->err, "dst is null"); return ADACGD_ERR_ARG; }
  if (c->wst) HIPCHK(c, hipStreamSynchronize(c->wst));
  HIPCHK(c, hipStreamSynchronize(c->st));
  const int64_t n = c->n, d = c->d;
  const hipMemcpyKind kind = dst_on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
  auto copy = [&](const void* src, int64_t bytes) -> int {
    if (bytes != dst_bytes) {
      set_err(c->err, "field %d holds %lld bytes, destination has %lld", field, (long long)bytes, (long long)dst_bytes);
      return ADACGD_ERR_FIELD;
    }
    if (bytes == 0) return ADACGD_OK;
    if (!src) { set_err(c->err, "field %d is not kept in this mode", field); return ADACGD_ERR_STATE; }
    HIPCHK(c, hipMemcpyAsync(dst, src, (size_t)bytes, kind, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    return ADACGD_OK;
  };
  auto host_out = [&](const void* src, int64_t bytes) -> int {
    if (bytes != dst_bytes) {
      set_err(c->err, "field %d holds %lld bytes, destination has %lld", field, (long long)bytes, (long long)dst_bytes);
      return ADACGD_ERR_FIELD;
    }
    if (dst_on_device) {
      HIPCHK(c, hipMemcpyAsync(dst, src, (size_t)bytes, hipMemcpyHostToDevice, c->st));
      HIPCHK(c, hipStreamSynchronize(c->st));
    } else {
      std::memcpy(dst, src, (size_t)bytes);
    }
    return ADACGD_OK;
  };
  auto packed = [&](const NodeSet& ns, const void* base, size_t elt, bool count_only) -> int {
    std::vector<uint32_t> cnt((size_t)ns.nn);
    HIPCHK(c, hipMemcpyAsync(cnt.data(), ns.msg_count, cnt.size() * 4, hipMemcpyDeviceToHost, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    if (count_only) {
      std::vector<int64_t> c64(cnt.begin(), cnt.end());
      return host_out(c64.data(), (int64_t)c64.size() * 8);
    }
    int64_t total = 0;
    for (uint32_t v : cnt) total += v;
    if (total * (int64_t)elt != dst_bytes) {
      set_err(c->err, "field %d holds %lld bytes, destination has %lld", field, (long long)(total * elt),
              (long long)dst_bytes);
      return ADACGD_ERR_FIELD;
    }
    size_t off = 0;
    for (int i = 0; i < ns.nn; ++i) {
      if (!cnt[i]) continue;
      HIPCHK(c, hipMemcpyAsync((char*)dst + off, (const char*)base + (size_t)i * ns.Kcap * elt, cnt[i] * elt, kind,
                               c->st));
      off += cnt[i] * elt;
    }
    HIPCHK(c, hipStreamSynchronize(c->st));
    return ADACGD_OK;
  };
  const NodeSet& W = c->W;
  const NodeSet& M = c->M;
  const bool hm = c->has_master;
  switch (field) {
    case ADACGD_F_X: return copy(c->x, d * 4);
    case ADACGD_F_G: return copy(c->g(), d * 4);
    case ADACGD_F_GTILDE: return copy(c->gt[c->cur], d * 4);
    case ADACGD_F_GTILDE_PREV: return copy(c->gt[c->cur ^ 1], d * 4);
    case ADACGD_F_GI: return copy(c->gi, n * d * 4);
    case ADACGD_F_PREV_GRAD:
    case ADACGD_F_GRAD:
      return copy(c->grad_mode == ADACGD_DIFF_EXTERNAL ? nullptr : c->ycurp(), n * d * 4);
    case ADACGD_F_LEVEL: return copy(W.level, n * 4);
    case ADACGD_F_SQNORM: return copy(W.S, n * 8);
    case ADACGD_F_D: return copy(W.D, n * 8);
    case ADACGD_F_ERR: return copy(W.err, n * W.lv.m * 8);
    case ADACGD_F_MSG_COUNT: return packed(W, nullptr, 0, true);
    case ADACGD_F_MSG_IDX: return packed(W, W.msg_idx, 4, false);
    case ADACGD_F_MSG_VAL: return packed(W, W.msg_val, 4, false);
    case ADACGD_F_M_LEVEL: return hm ? copy(M.level, 4) : copy(nullptr, 4);
    case ADACGD_F_M_SQNORM: return hm ? copy(M.S, 8) : copy(nullptr, 8);
    case ADACGD_F_M_D: return hm ? copy(M.D, 8) : copy(nullptr, 8);
    case ADACGD_F_M_ERR: return hm ? copy(M.err, (int64_t)M.lv.m * 8) : copy(nullptr, 0);
    case ADACGD_F_M_MSG_COUNT:
      if (!hm) { set_err(c->err, "no master compressor"); return ADACGD_ERR_STATE; }
      return packed(M, nullptr, 0, true);
    case ADACGD_F_M_MSG_IDX:
      if (!hm) { set_err(c->err, "no master compressor"); return ADACGD_ERR_STATE; }
      return packed(M, M.msg_idx, 4, false);
    case ADACGD_F_M_MSG_VAL:
      if (!hm) { set_err(c->err, "no master compressor"); return ADACGD_ERR_STATE; }
      return packed(M, M.msg_val, 4, false);
    case ADACGD_F_STEP: return host_out(&c->step, 8);
    case ADACGD_F_REPAIRS: {
      uint64_t o[2] = {0, 0};
      HIPCHK(c, hipMemcpyAsync(&o[0], W.repairs, 8, hipMemcpyDeviceToHost, c->st));
      if (hm) HIPCHK(c, hipMemcpyAsync(&o[1], M.repairs, 8, hipMemcpyDeviceToHost, c->st));
      HIPCHK(c, hipStreamSynchronize(c->st));
      return host_out(o, 16);
    }
    case ADACGD_F_CANDIDATES: {
      uint64_t o[2] = {0, 0};
      const NodeSet* sets[2] = {&W, hm ? &M : nullptr};
      for (int k = 0; k < 2; ++k) {
        const NodeSet* ns = sets[k];
        if (!ns || !ns->onepass || c->step == 0) continue;
        std::vector<uint32_t> part((size_t)ns->nn * ns->G);
        HIPCHK(c, hipMemcpyAsync(part.data(), ns->partU, part.size() * 4, hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipStreamSynchronize(c->st));
        for (int i = 0; i < ns->nn; ++i)
          for (int b = 0; b < ns->G; ++b) o[k] += part[(size_t)i * ns->G + b];
      }
      return host_out(o, 16);
    }
    case ADACGD_F_ESTIMATOR_ERR: {
      if (c->step == 0) { set_err(c->err, "no step has run yet"); return ADACGD_ERR_STATE; }
      const int m = W.lv.m;
      std::vector<int32_t> lev((size_t)n);
      std::vector<double> S((size_t)n), err((size_t)n * m);
      HIPCHK(c, hipMemcpyAsync(lev.data(), W.level, (size_t)n * 4, hipMemcpyDeviceToHost, c->st));
      HIPCHK(c, hipMemcpyAsync(S.data(), W.S, (size_t)n * 8, hipMemcpyDeviceToHost, c->st));
      HIPCHK(c, hipMemcpyAsync(err.data(), W.err, (size_t)n * m * 8, hipMemcpyDeviceToHost, c->st));
      HIPCHK(c, hipStreamSynchronize(c->st));
      double G = 0.0;     // what is left of x - h after the update: all of it on a skip, else the level's error
      for (int64_t i = 0; i < n; ++i) G += lev[(size_t)i] == 0 ? S[(size_t)i] : err[(size_t)i * m + lev[(size_t)i] - 1];
      G /= (double)n;
      return host_out(&G, 8);
    }
    case ADACGD_F_LEVEL_HIST: return copy(W.level_hist, (int64_t)(W.lv.m + 1) * 8);
    case ADACGD_F_M_LEVEL_HIST: return hm ? copy(M.level_hist, (int64_t)(M.lv.m + 1) * 8) : copy(nullptr, 8);
    case ADACGD_F_COMM: {
      uint64_t o[4] = {0, 0, 0, 0};
      std::vector<unsigned long long> hw(W.lv.m + 1), hmv(M.lv.m + 1);
      HIPCHK(c, hipMemcpyAsync(hw.data(), W.level_hist, hw.size() * 8, hipMemcpyDeviceToHost, c->st));
      if (hm) HIPCHK(c, hipMemcpyAsync(hmv.data(), M.level_hist, hmv.size() * 8, hipMemcpyDeviceToHost, c->st));
      HIPCHK(c, hipStreamSynchronize(c->st));
      comm_of(W, hw.data(), 1, &o[0], &o[1]);
      if (hm) {
        comm_of(M, hmv.data(), (uint64_t)n, &o[2], &o[3]);
      } else {                      // identity master: the dense g~ goes to every worker each step
        o[2] = (uint64_t)c->step * (uint64_t)d * (uint64_t)n;
        o[3] = o[2] * 32;
      }
      return host_out(o, 32);
    }
    case ADACGD_F_QCODES: return copy(W.qcodes, n * d * 2);
    case ADACGD_F_QSCALE: return copy(W.qscale, n * 4);
    case ADACGD_F_QBSCALE: return copy(W.qbscale, n * (int64_t)W.nseg * 4);
    case ADACGD_F_RANK_SPECTRUM: return copy(W.lv.nr ? W.rk_lambda : nullptr, n * (int64_t)W.lv.rcols * 8);
    case ADACGD_F_KERNEL_MS: {
      int rc = drain_spans(c);
      if (rc) return rc;
      double o[2 * ADACGD_NUM_KERNELS];
      for (int k = 0; k < ADACGD_NUM_KERNELS; ++k) { o[k] = c->ms_sum[k]; o[ADACGD_NUM_KERNELS + k] = c->ms_cnt[k]; }
      rc = host_out(o, sizeof(o));
      if (rc == ADACGD_OK) {
        std::memset(c->ms_sum, 0, sizeof(c->ms_sum));
        std::memset(c->ms_cnt, 0, sizeof(c->ms_cnt));
      }
      return rc;
    }
    default:
      set_err(c->err, "unknown field %d", field);
      return ADACGD_ERR_FIELD;
  }
}

int adacgd_set_state(adacgd_ctx* c, int32_t field, const void* src, int64_t src_bytes, int32_t src_on_device) {
  if (!c) return ADACGD_ERR_ARG;
  if (!src) { set_err(c->err, "src is null"); return ADACGD_ERR_ARG; }
  if (c->wst) HIPCHK(c, hipStreamSynchronize(c->wst));
  HIPCHK(c, hipStreamSynchronize(c->st));
  const int64_t n = c->n, d = c->d;
  const hipMemcpyKind kind = src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
  auto put = [&](void* dst, int64_t bytes) -> int {
    if (bytes != src_bytes) {
      set_err(c->err, "field %d holds %lld bytes, source has %lld", field, (long long)bytes, (long long)src_bytes);
      return ADACGD_ERR_FIELD;
    }
    if (!dst) { set_err(c->err, "field %d is not kept in this mode", field); return ADACGD_ERR_STATE; }
    HIPCHK(c, hipMemcpyAsync(dst, src, (size_t)bytes, kind, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    return ADACGD_OK;
  };
  switch (field) {
    case ADACGD_F_X:
      c->x_next_valid = false;      // the iterate written ahead belonged to the old x
      return put(c->x, d * 4);
    case ADACGD_F_G:
      c->x_next_valid = false;
      return put(c->has_master ? c->g_own : nullptr, d * 4);
    case ADACGD_F_GTILDE:
      if (!c->has_master) c->x_next_valid = false;   // g is g~ then
      return put(c->gt[c->cur], d * 4);
    case ADACGD_F_GTILDE_PREV: return put(c->gt[c->cur ^ 1], d * 4);
    case ADACGD_F_GI: return put(c->gi, n * d * 4);
    case ADACGD_F_PREV_GRAD:
    case ADACGD_F_GRAD:
      if (c->grad_mode == ADACGD_DIFF_EXTERNAL) return put(nullptr, n * d * 4);
      if (c->y_ext) {               // the caller's retained array is replaced by the engine's own buffer
        c->y_ext = nullptr;
        c->ycur = 0;
      }
      return put(c->yb[c->ycur], n * d * 4);
    case ADACGD_F_STEP: {
      if (src_bytes != 8) { set_err(c->err, "field %d holds 8 bytes, source has %lld", field, (long long)src_bytes); return ADACGD_ERR_FIELD; }
      int64_t v = 0;
      if (src_on_device) HIPCHK(c, hipMemcpy(&v, src, 8, hipMemcpyDeviceToHost));
      else std::memcpy(&v, src, 8);
      if (v < 0) { set_err(c->err, "step count is negative"); return ADACGD_ERR_ARG; }
      c->step = v;
      return ADACGD_OK;
    }
    case ADACGD_F_LEVEL_HIST: return put(c->W.level_hist, (int64_t)(c->W.lv.m + 1) * 8);
    case ADACGD_F_M_LEVEL_HIST: return put(c->has_master ? c->M.level_hist : nullptr, (int64_t)(c->M.lv.m + 1) * 8);
    default:
      set_err(c->err, "field %d cannot be set", field);
      return ADACGD_ERR_FIELD;
  }
}

int adacgd_destroy(adacgd_ctx* c) {
  if (!c) return ADACGD_OK;
  if (c->wst) {
    (void)hipStreamSynchronize(c->wst);
    (void)hipStreamDestroy(c->wst);
    (void)hipEventDestroy(c->ev_worker);
    (void)hipEventDestroy(c->ev_agg);
  }
  hipError_t e = hipStreamSynchronize(c->st);
  for (auto& s : c->spans) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
  for (auto ev : c->pool) (void)hipEventDestroy(ev);
  release_ctx(c, true);
  return e == hipSuccess ? ADACGD_OK : ADACGD_ERR_DEVICE;
}

const char* adacgd_last_error(const adacgd_ctx* c) { return c ? c->err : g_err; }

}  // extern "C"
