// Server side and objective of the AdaCGD iteration:
//   iterate update x <- x - gamma g                       (Algorithm 1)
//   aggregation    g~ <- g~ + (1/n) sum_i message_i       (Algorithm 1, incremental form)
//   local gradients of the logistic objective with the nonconvex regulariser (Section 6)
#include "devutil.h"
#include "engine.h"

namespace adacgd {

// ---------------------------------------------------------------------------
// small dense kernels
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_xupdate(float* __restrict__ x, const float* __restrict__ g, double gamma,
                                                     int64_t d) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < d) x[i] = (float)((double)x[i] - gamma * (double)g[i]);   // one rounding
}

// g~^0 = (1/n) sum_i g~_i^0, summed in ascending i in fp64; written to up to three vectors
__global__ __launch_bounds__(kBlock) void k_mean(const float* __restrict__ gi, float* o0, float* o1, float* o2, int n,
                                                  int64_t d) {
  const int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (c >= d) return;
  double acc = 0.0;
  for (int i = 0; i < n; ++i) acc += (double)gi[(size_t)i * d + c];
  const float r = (float)(acc / (double)n);
  o0[c] = r;
  if (o1) o1[c] = r;
  if (o2) o2[c] = r;
}

__global__ __launch_bounds__(kBlock) void k_fill_u32(uint32_t* p, uint32_t v, size_t count) {
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (size_t)gridDim.x * kBlock) p[i] = v;
}

__global__ __launch_bounds__(kBlock) void k_copy_f32(float* __restrict__ dst, const float* __restrict__ src,
                                                      size_t count) {
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < count; i += (size_t)gridDim.x * kBlock)
    dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// aggregation: one block per group (2048 coordinates) of the server vector.  The group's
// share of every worker's sorted message is a contiguous range (known from the message
// offsets per group).  The ranges of up to 256 workers at a time are laid end to end and the
// threads stride over that flattened list, adding into an fp64 accumulator in LDS; then
// g~_new = fl(g~_old + acc / n).  Sums of fp32 values in fp64 are exact unless their exponents
// spread over more than ~29 bits, so the result does not depend on the order of the additions.
// ---------------------------------------------------------------------------
// DENSE_LATER (level sets with quantisers): the fp64 sums of the sparse messages go to ws.accbuf and
// k_aggregate_dense adds the dense messages and finishes.
// `xu`: with the identity master g is g~, so the kernel that finishes g~_new can also write the next
// iterate x_next = fl(x - gamma g~_new) (xu.out null = not asked for).
template <bool DENSE_LATER>
__global__ __launch_bounds__(kBlock) void k_aggregate(NodeSet ws, const float* __restrict__ gt_old,
                                                       float* __restrict__ gt_new, IterateUpdate xu) {
  __shared__ double acc[kWaveTile];
  __shared__ uint32_t s_lo[kBlock], s_pre[kBlock + 1];
  __shared__ uint32_t lds4[4];
  __shared__ int s_flag;
  const int g = blockIdx.x, tid = threadIdx.x;
  const int64_t d = ws.d;
  const int64_t base = (int64_t)g * kWaveTile;
  // this block's share of the workers (all of them unless several blocks share the group)
  const int AS = gridDim.y, per = (ws.nn + AS - 1) / AS;
  const int n_lo = (int)blockIdx.y * per, n_hi = min(ws.nn, n_lo + per);
  for (int c = tid; c < kWaveTile; c += kBlock) acc[c] = 0.0;
  __syncthreads();
  for (int n0 = n_lo; n0 < n_hi; n0 += kBlock) {
    const int i = n0 + tid;
    uint32_t lo = 0, cnt = 0;
    if (i < n_hi) {
      if (ws.sel_slot[i] >= 0) {
        lo = ws.grp_off[(size_t)i * (ws.groups + 1) + g];
        cnt = ws.grp_off[(size_t)i * (ws.groups + 1) + g + 1] - lo;
      }
    }
    uint32_t total;
    const uint32_t pre = block_excl_scan(cnt, lds4, &total);
    s_lo[tid] = lo;
    s_pre[tid] = pre;
    if (tid == 0) s_pre[kBlock] = total;
    __syncthreads();
    for (uint32_t e = tid; e < total; e += kBlock) {
      // the worker whose range holds flattened entry e: last j with s_pre[j] <= e
      int lo_j = 0, hi_j = kBlock;
      while (hi_j - lo_j > 1) {
        const int mid = (lo_j + hi_j) >> 1;
        if (s_pre[mid] <= e) lo_j = mid; else hi_j = mid;
      }
      const size_t off = (size_t)(n0 + lo_j) * ws.Kcap + s_lo[lo_j] + (e - s_pre[lo_j]);
      unsafeAtomicAdd(&acc[ws.msg_idx[off] - base], (double)ws.msg_val[off]);
    }
    __syncthreads();
  }
  if (AS > 1) {
    // partial sums of the blocks that share this group; the last one to arrive adds them in block order
    for (int c = tid; c < kWaveTile; c += kBlock)
      st_coherent(&ws.agg_part[((size_t)blockIdx.y * ws.groups + g) * kWaveTile + c], acc[c]);
    if (!arrive_last(&ws.agg_done[(size_t)g * (kArriveFan + 1) * kCounterStride], (uint32_t)AS, blockIdx.y, &s_flag)) return;
    for (int c = tid; c < kWaveTile; c += kBlock) {
      double t = 0.0;
      for (int b = 0; b < AS; ++b) t += ld_coherent(&ws.agg_part[((size_t)b * ws.groups + g) * kWaveTile + c]);
      acc[c] = t;       // thread tid wrote and reads the same entries: no barrier needed
    }
  }
  if (DENSE_LATER) {
    for (int c = tid; c < kWaveTile; c += kBlock)
      if (base + c < d) ws.accbuf[base + c] = acc[c];
    return;
  }
  const double n = (double)ws.nn;
  for (int c = tid; c < kWaveTile; c += kBlock) {
    if (base + c < d) {
      const float gn = (float)((double)gt_old[base + c] + acc[c] / n);
      gt_new[base + c] = gn;
      if (xu.out) xu.out[base + c] = (float)((double)xu.x[base + c] - xu.gamma * (double)gn);
    }
  }
}

// Top-K messages of at most kOrderedMax workers: the same sums taken in ASCENDING WORKER INDEX, so that the
// result is the sequential fp64 sum whatever the data (the kernel above adds in arbitrary order, which gives
// the same bits only while the exponents met at one coordinate spread over less than 53 - 24 - log2 n bits).
// One block per group of 2048 coordinates, and inside it every wavefront owns a quarter of them: it walks
// the group's range of every worker's message, worker after worker, and adds the entries that fall into its
// quarter.  A wavefront's LDS operations execute in the order they are issued, and the coordinates of one
// message are distinct, so every coordinate receives its additions in worker order without any barrier; the
// four wavefronts read the same few kilobytes of messages (the later ones from the cache).
constexpr int kOrderedMax = 64;
constexpr int kAggChunk = 8;          // workers whose first 64 entries are in flight at once

__global__ __launch_bounds__(kBlock) void k_aggregate_ordered(NodeSet ws, const float* __restrict__ gt_old,
                                                               float* __restrict__ gt_new, IterateUpdate xu) {
  __shared__ double acc[kWaveTile];
  constexpr int QUARTER = kWaveTile / 4;
  const int g = blockIdx.x, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int64_t d = ws.d;
  const int64_t base = (int64_t)g * kWaveTile;
  double* mine = acc + w * QUARTER;                       // only this wavefront touches these entries
  const int64_t first = base + w * QUARTER;
  for (int c = lane; c < QUARTER; c += 64) mine[c] = 0.0;
  for (int i0 = 0; i0 < ws.nn; i0 += kAggChunk) {
    uint32_t lo[kAggChunk], cnt[kAggChunk];
    int32_t pidx[kAggChunk];
    float pval[kAggChunk];
#pragma unroll
    for (int u = 0; u < kAggChunk; ++u) {
      const int i = i0 + u;
      lo[u] = 0; cnt[u] = 0;
      if (i < ws.nn && __builtin_amdgcn_readfirstlane(ws.sel_slot[i]) >= 0) {
        const uint32_t l = __builtin_amdgcn_readfirstlane(ws.grp_off[(size_t)i * (ws.groups + 1) + g]);
        lo[u] = l;
        cnt[u] = __builtin_amdgcn_readfirstlane(ws.grp_off[(size_t)i * (ws.groups + 1) + g + 1]) - l;
      }
    }
#pragma unroll
    for (int u = 0; u < kAggChunk; ++u) {                 // first entry per lane of every range
      pidx[u] = 0; pval[u] = 0.f;
      if ((uint32_t)lane < cnt[u]) {
        const size_t off = (size_t)(i0 + u) * ws.Kcap + lo[u] + lane;
        pidx[u] = ws.msg_idx[off];
        pval[u] = ws.msg_val[off];
      }
    }
#pragma unroll
    for (int u = 0; u < kAggChunk; ++u) {
      if (cnt[u] == 0) continue;                          // (the same in every lane)
      uint64_t r = (uint64_t)((int64_t)pidx[u] - first);         // (huge for coordinates below this quarter)
      if ((uint32_t)lane < cnt[u] && r < (uint64_t)QUARTER) mine[r] += (double)pval[u];
      for (uint32_t e = lane + 64; e < cnt[u]; e += 64) {
        const size_t off = (size_t)(i0 + u) * ws.Kcap + lo[u] + e;
        r = (uint64_t)((int64_t)ws.msg_idx[off] - first);
        if (r < (uint64_t)QUARTER) mine[r] += (double)ws.msg_val[off];
      }
    }
  }
  const double n = (double)ws.nn;
  for (int c = lane; c < QUARTER; c += 64) {
    const int64_t l = first + c;
    if (l < d) {
      const float gn = (float)((double)gt_old[l] + mine[c] / n);
      gt_new[l] = gn;
      if (xu.out) xu.out[l] = (float)((double)xu.x[l] - xu.gamma * (double)gn);
    }
  }
}

// Dense (quantised) messages: a block owns 128 coordinates, each lane two of them (one 4-byte
// load per worker); its eight wavefronts take one eighth of the workers each, in ascending order,
// eight workers' loads in flight at a time, and their partial sums are combined in wavefront
// order: g~_new = fl(g~_old + (sparse sums + dense sums) / n).
constexpr int kDenseCols = 128;
constexpr int kDenseWaves = 8;
__global__ __launch_bounds__(64 * kDenseWaves) void k_aggregate_dense(NodeSet ws, const float* __restrict__ gt_old,
                                                                      float* __restrict__ gt_new, IterateUpdate xu) {
  __shared__ double part[kDenseWaves][kDenseCols];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int64_t d = ws.d;
  const int64_t c0 = (int64_t)blockIdx.x * kDenseCols + 2 * lane;
  const bool ok0 = c0 < d, ok1 = c0 + 1 < d;
  const bool pair = ok1 && (d % 2 == 0);       // rows are then 4-byte aligned at c0
  const int q = (ws.nn + kDenseWaves - 1) / kDenseWaves;
  const int i0 = w * q, i1 = min(ws.nn, i0 + q);
  double a0 = 0.0, a1 = 0.0;
  auto decode = [](int code, float sc) {
    const float mag = (float)(code < 0 ? -code : code) * sc;
    return (double)(code < 0 ? -mag : mag);
  };
  // Rank-K messages are dense fp32 vectors: workers that chose one, in ascending order after this
  // wavefront's quantised ones
  if (ws.lv.nr > 0) {
    for (int i = i0; i < i1; ++i) {
      if (ws.sel_rk[i] < 0) continue;
      const float* __restrict__ rd = ws.rdense + (size_t)i * d;
      if (ok0) a0 += (double)rd[c0];
      if (ok1) a1 += (double)rd[c0 + 1];
    }
  }
  constexpr int U = 8;
  for (int i = i0; i < i1; i += U) {
    int k0[U], k1[U];
    float sc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ii = i + u;
      const int qi = (ii < i1 && ws.lv.nq > 0) ? ws.sel_q[ii] : -1;
      const bool dense = qi >= 0;
      const int B = dense ? ws.lv.qblock[qi] : 0;          // block-wise level: the scale of this coordinate pair's block
      sc[u] = !dense ? 0.f : (B ? ws.qbscale[(size_t)ii * ws.nseg + (ok0 ? c0 / B : 0)] : ws.qscale[ii]);
      const int16_t* __restrict__ codes = ws.qcodes + (size_t)(dense ? ii : 0) * d;
      if (pair) {
        const uint32_t two = dense ? *reinterpret_cast<const uint32_t*>(codes + c0) : 0u;
        k0[u] = (int)(int16_t)(two & 0xFFFFu);
        k1[u] = (int)(int16_t)(two >> 16);
      } else {
        k0[u] = (dense && ok0) ? (int)codes[c0] : 0;
        k1[u] = (dense && ok1) ? (int)codes[c0 + 1] : 0;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      a0 += decode(k0[u], sc[u]);
      a1 += decode(k1[u], sc[u]);
    }
  }
  part[w][2 * lane] = a0;
  part[w][2 * lane + 1] = a1;
  __syncthreads();
  if (tid < kDenseCols) {
    const int64_t c = (int64_t)blockIdx.x * kDenseCols + tid;
    if (c < d) {
      double tot = ws.accbuf[c];
#pragma unroll
      for (int j = 0; j < kDenseWaves; ++j) tot += part[j][tid];
      const float gn = (float)((double)gt_old[c] + tot / (double)ws.nn);
      gt_new[c] = gn;
      if (xu.out) xu.out[c] = (float)((double)xu.x[c] - xu.gamma * (double)gn);
    }
  }
}

// ---------------------------------------------------------------------------
// logistic gradient, Section 6:
//   grad f_i(x) = -(1/N_i) sum_l y_l a_l / (1 + exp(y_l a_l^T x)) + 2 lambda x_j / (1 + x_j^2)^2
// margins: LPR lanes per sample (64, or 16 for rows shorter than 1024 so that a wavefront works on four
//          rows at once) compute a_l^T x in fp64 and s_l = -y_l/(1+exp(y_l z_l))/N_i.
// cols   : a block owns 64 column groups (4 columns each on the 16-byte path) and a chunk of the shard's
//          rows; its four wavefronts take every fourth row, sum s_l a_l in fp64, and the four partial
//          sums are added in wavefront order.  Shards of more than 256 rows are shared by several
//          blocks; the one that finishes last adds their sums in chunk order.
// ---------------------------------------------------------------------------
template <int LPR, bool VEC>
__global__ __launch_bounds__(kBlock) void k_grad_margins(LogisticData ld, const float* __restrict__ x, int64_t d) {
  const int64_t l = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / LPR;
  const int sub = threadIdx.x % LPR;
  const bool live = l < ld.rows;
  const float* __restrict__ a = ld.A + (size_t)(live ? l : 0) * d;
  const int64_t dd = live ? d : 0;
  double acc0 = 0.0, acc1 = 0.0;
  if (VEC) {
#pragma unroll 4
    for (int64_t j = (int64_t)sub * 4; j < dd; j += LPR * 4) {
      const float4 av = *reinterpret_cast<const float4*>(a + j);
      const float4 xv = *reinterpret_cast<const float4*>(x + j);
      acc0 = fma((double)av.x, (double)xv.x, acc0);
      acc1 = fma((double)av.y, (double)xv.y, acc1);
      acc0 = fma((double)av.z, (double)xv.z, acc0);
      acc1 = fma((double)av.w, (double)xv.w, acc1);
    }
  } else {
#pragma unroll 4
    for (int64_t j = sub; j < dd; j += LPR) acc0 = fma((double)a[j], (double)x[j], acc0);
  }
  double z = acc0 + acc1;
#pragma unroll
  for (int o = LPR >> 1; o > 0; o >>= 1) z += __shfl_xor(z, o);
  if (live && sub == 0) {
    const int node = ld.row_node[l];
    const double N = (double)(ld.offsets[node + 1] - ld.offsets[node]);
    const double yl = (double)ld.labels[l];
    ld.margins[l] = -yl / (1.0 + exp(yl * z)) / N;
  }
}

__device__ __forceinline__ double reg_grad(double lambda, double xj) {
  const double q = 1.0 + xj * xj;
  return 2.0 * lambda * xj / (q * q);
}

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_grad_cols(LogisticData ld, const float* __restrict__ x,
                                                       float* __restrict__ grads, int64_t d, int rows_per_chunk) {
  constexpr int CPL = VEC ? 4 : 1;                 // columns per lane
  __shared__ double part[4][64 * CPL];
  __shared__ int s_flag;
  const int node = blockIdx.z, rc = blockIdx.y, w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t j0 = ((int64_t)blockIdx.x * 64 + lane) * CPL;
  const bool live = j0 < d;
  const int64_t r_begin = ld.offsets[node] + (int64_t)rc * rows_per_chunk;
  const int64_t r_end = min(ld.offsets[node + 1], r_begin + rows_per_chunk);
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  if (live) {
    const float* __restrict__ a = ld.A + (size_t)(r_begin + w) * d + j0;
#pragma unroll 4
    for (int64_t l = r_begin + w; l < r_end; l += 4, a += 4 * d) {
      const double s = ld.margins[l];
      if (VEC) {
        const float4 av = *reinterpret_cast<const float4*>(a);
        acc[0] = fma(s, (double)av.x, acc[0]);
        acc[1] = fma(s, (double)av.y, acc[1]);
        acc[2] = fma(s, (double)av.z, acc[2]);
        acc[3] = fma(s, (double)av.w, acc[3]);
      } else {
        acc[0] = fma(s, (double)a[0], acc[0]);
      }
    }
  }
#pragma unroll
  for (int c = 0; c < CPL; ++c) part[w][lane * CPL + c] = acc[c];
  __syncthreads();
  double t[4];
#pragma unroll
  for (int c = 0; c < CPL; ++c)
    t[c] = ((part[0][lane * CPL + c] + part[1][lane * CPL + c]) + part[2][lane * CPL + c]) + part[3][lane * CPL + c];
  if (ld.row_chunks > 1) {
    // several blocks share the shard's rows: each leaves its sums, the last to arrive adds them in chunk order
    if (w == 0 && live) {
#pragma unroll
      for (int c = 0; c < CPL; ++c) st_coherent(&ld.part[((size_t)node * ld.row_chunks + rc) * d + j0 + c], t[c]);
    }
    if (!arrive_last_few(&ld.col_done[(size_t)node * gridDim.x + blockIdx.x], (uint32_t)ld.row_chunks, &s_flag)) return;
#pragma unroll
    for (int c = 0; c < CPL; ++c) t[c] = 0.0;
    if (w == 0 && live) {
      for (int r0 = 0; r0 < ld.row_chunks; r0 += 8) {        // eight chunks' loads in flight, added in chunk order
        double v[8][4];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int c = 0; c < CPL; ++c)
            v[u][c] = r0 + u < ld.row_chunks ? ld_coherent(&ld.part[((size_t)node * ld.row_chunks + r0 + u) * d + j0 + c]) : 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int c = 0; c < CPL; ++c) t[c] += v[u][c];
      }
    }
  }
  if (w != 0 || !live) return;
#pragma unroll
  for (int c = 0; c < CPL; ++c) grads[(size_t)node * d + j0 + c] = (float)(t[c] + reg_grad(ld.lambda, (double)x[j0 + c]));
}

// ---------------------------------------------------------------------------
// The same gradient for sparse features (rows in CSR form, and per worker by column).
// margins: LPR lanes per row (a power of two) sum the row's stored entries in fp64.
// cols   : 1, 16 or 64 lanes per (worker, column) sum s_l a_lj over the column's entries of that
//          worker's shard in a fixed order, then add the regulariser and round once.
// ---------------------------------------------------------------------------
template <int LPR>
__global__ __launch_bounds__(kBlock) void k_csr_margins(LogisticData ld, const float* __restrict__ x) {
  const int64_t l = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / LPR;
  const int sub = threadIdx.x % LPR;
  const bool live = l < ld.rows;
  const int64_t b = live ? ld.rp[l] : 0, e = live ? ld.rp[l + 1] : 0;
  double acc = 0.0;
  int64_t k = b + sub;
  for (; k + 3 * LPR < e; k += 4 * LPR) {          // four entries at a time: their gathers overlap
    int32_t c[4];
    float a[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      c[u] = ld.ci[k + u * LPR];
      a[u] = ld.binary ? 1.f : ld.cv[k + u * LPR];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) acc = fma((double)a[u], (double)x[c[u]], acc);
  }
  for (; k < e; k += LPR) {
    const double a = ld.binary ? 1.0 : (double)ld.cv[k];
    acc = fma(a, (double)x[ld.ci[k]], acc);
  }
#pragma unroll
  for (int o = LPR >> 1; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if (live && sub == 0) {
    const int node = ld.row_node[l];
    const double N = (double)(ld.offsets[node + 1] - ld.offsets[node]);
    const double yl = (double)ld.labels[l];
    ld.margins[l] = -yl / (1.0 + exp(yl * acc)) / N;
  }
}

template <int LPC>   // lanes per column, a power of two: long columns are shared by 16 or 64 lanes
__global__ __launch_bounds__(kBlock) void k_csr_cols(LogisticData ld, const float* __restrict__ x,
                                                      float* __restrict__ grads, int64_t d) {
  const int node = blockIdx.y;
  const int64_t j = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / LPC;
  const int sub = threadIdx.x % LPC;
  const bool live = j < d;
  const uint32_t* __restrict__ cp = ld.cptr + (size_t)node * (size_t)(d + 1);
  const int64_t w0 = ld.wbase[node];
  const int64_t b = live ? w0 + cp[j] : 0, e = live ? w0 + cp[j + 1] : 0;
  double acc = 0.0;
  for (int64_t k = b + sub; k < e; k += LPC) {
    const double a = ld.binary ? 1.0 : (double)ld.tval[k];
    acc = fma(ld.margins[ld.trow[k]], a, acc);
  }
#pragma unroll
  for (int o = LPC >> 1; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if (live && sub == 0) grads[(size_t)node * d + j] = (float)(acc + reg_grad(ld.lambda, (double)x[j]));
}

// Short columns (a few entries per worker-column): one thread owns four columns, 64 apart, and walks
// them side by side, so that four independent chains of gathers (row of the entry, then its margin)
// are in flight instead of one.  Same order of summation per column as k_csr_cols<1>.
__global__ __launch_bounds__(kBlock) void k_csr_cols4(LogisticData ld, const float* __restrict__ x,
                                                       float* __restrict__ grads, int64_t d) {
  const int node = blockIdx.y, w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t j0 = ((int64_t)blockIdx.x * 4 + w) * 256 + lane;      // columns j0, j0+64, j0+128, j0+192
  const uint32_t* __restrict__ cp = ld.cptr + (size_t)node * (size_t)(d + 1);
  const int64_t w0 = ld.wbase[node];
  int64_t b[4], e[4];
  double acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int64_t j = j0 + 64 * c;
    const bool live = j < d;
    b[c] = live ? w0 + cp[j] : 0;
    e[c] = live ? w0 + cp[j + 1] : 0;
    acc[c] = 0.0;
  }
  int64_t longest = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) longest = max(longest, e[c] - b[c]);
  for (int64_t t = 0; t < longest; ++t) {
    int32_t r[4];
    float a[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool on = b[c] + t < e[c];
      r[c] = on ? ld.trow[b[c] + t] : -1;
      a[c] = (on && !ld.binary) ? ld.tval[b[c] + t] : 1.f;
    }
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (r[c] >= 0) acc[c] = fma(ld.margins[r[c]], (double)a[c], acc[c]);
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int64_t j = j0 + 64 * c;
    if (j < d) grads[(size_t)node * d + j] = (float)(acc[c] + reg_grad(ld.lambda, (double)x[j]));
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
static inline unsigned blocks_for(size_t count, unsigned cap = 65535u * 16u) {
  size_t b = (count + kBlock - 1) / kBlock;
  if (b < 1) b = 1;
  return (unsigned)(b > cap ? cap : b);
}

hipError_t launch_xupdate(float* x, const float* g, double gamma, int64_t d, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  hipLaunchKernelGGL(k_xupdate, dim3((unsigned)((d + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, x, g, gamma, d);
  return hipGetLastError();
}

hipError_t launch_mean(const float* gi, float* o0, float* o1, float* o2, int n, int64_t d, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  hipLaunchKernelGGL(k_mean, dim3((unsigned)((d + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, gi, o0, o1, o2, n, d);
  return hipGetLastError();
}

hipError_t launch_aggregate(const NodeSet& ws, const float* gt_old, float* gt_new, const IterateUpdate& xu,
                            hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  if (ws.lv.nq == 0 && ws.lv.nr == 0) {
    if (ws.nn <= kOrderedMax)
      hipLaunchKernelGGL(k_aggregate_ordered, dim3(ws.groups), dim3(kBlock), 0, st, ws, gt_old, gt_new, xu);
    else
      hipLaunchKernelGGL((k_aggregate<false>), dim3(ws.groups, ws.AS), dim3(kBlock), 0, st, ws, gt_old, gt_new, xu);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((k_aggregate<true>), dim3(ws.groups, ws.AS), dim3(kBlock), 0, st, ws, gt_old, gt_new, IterateUpdate{});
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_aggregate_dense, dim3((unsigned)((ws.d + kDenseCols - 1) / kDenseCols)), dim3(64 * kDenseWaves), 0, st, ws,
                     gt_old, gt_new, xu);
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, uint32_t v, size_t count, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(k_fill_u32, dim3(blocks_for(count, 4096)), dim3(kBlock), 0, st, p, v, count);
  return hipGetLastError();
}

hipError_t launch_copy_f32(float* dst, const float* src, size_t count, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(k_copy_f32, dim3(blocks_for(count, 8192)), dim3(kBlock), 0, st, dst, src, count);
  return hipGetLastError();
}

hipError_t launch_grad_margins(const LogisticData& ld, const float* x, int64_t d, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  if (ld.csr) {
    const int64_t per_row = ld.nnz / (ld.rows > 0 ? ld.rows : 1);
    const int lpr = per_row >= 128 ? 64 : per_row >= 16 ? 16 : 4;
    const unsigned grid = (unsigned)((ld.rows * lpr + kBlock - 1) / kBlock);
    if (lpr == 64) hipLaunchKernelGGL((k_csr_margins<64>), dim3(grid), dim3(kBlock), 0, st, ld, x);
    else if (lpr == 16) hipLaunchKernelGGL((k_csr_margins<16>), dim3(grid), dim3(kBlock), 0, st, ld, x);
    else hipLaunchKernelGGL((k_csr_margins<4>), dim3(grid), dim3(kBlock), 0, st, ld, x);
    return hipGetLastError();
  }
  const bool vec = (d % 4 == 0) && ((reinterpret_cast<uintptr_t>(ld.A) & 15u) == 0) &&
                   ((reinterpret_cast<uintptr_t>(x) & 15u) == 0);
  const int lpr = d >= 1024 ? 64 : 16;
  const dim3 grid((unsigned)((ld.rows * lpr + kBlock - 1) / kBlock));
  if (lpr == 64) {
    if (vec) hipLaunchKernelGGL((k_grad_margins<64, true>), grid, dim3(kBlock), 0, st, ld, x, d);
    else hipLaunchKernelGGL((k_grad_margins<64, false>), grid, dim3(kBlock), 0, st, ld, x, d);
  } else {
    if (vec) hipLaunchKernelGGL((k_grad_margins<16, true>), grid, dim3(kBlock), 0, st, ld, x, d);
    else hipLaunchKernelGGL((k_grad_margins<16, false>), grid, dim3(kBlock), 0, st, ld, x, d);
  }
  return hipGetLastError();
}

hipError_t launch_grad_cols(const LogisticData& ld, const float* x, float* grads, int n, int64_t d, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  if (ld.csr) {
    const int64_t per_col = ld.nnz / ((int64_t)n * d);
    const int lpc = per_col >= 256 ? 64 : per_col >= 16 ? 16 : 1;
    const dim3 grid((unsigned)((d * lpc + kBlock - 1) / kBlock), n);
    if (lpc == 64) hipLaunchKernelGGL((k_csr_cols<64>), grid, dim3(kBlock), 0, st, ld, x, grads, d);
    else if (lpc == 16) hipLaunchKernelGGL((k_csr_cols<16>), grid, dim3(kBlock), 0, st, ld, x, grads, d);
    else hipLaunchKernelGGL(k_csr_cols4, dim3((unsigned)((d + 1023) / 1024), n), dim3(kBlock), 0, st, ld, x, grads, d);
    return hipGetLastError();
  }
  const bool vec = (d % 4 == 0) && ((reinterpret_cast<uintptr_t>(ld.A) & 15u) == 0);
  const int rpc = (int)((ld.max_rows + ld.row_chunks - 1) / ld.row_chunks);
  const int64_t cols_per_block = 64 * (vec ? 4 : 1);
  const dim3 grid((unsigned)((d + cols_per_block - 1) / cols_per_block), ld.row_chunks, n);
  if (vec) hipLaunchKernelGGL((k_grad_cols<true>), grid, dim3(kBlock), 0, st, ld, x, grads, d, rpc);
  else hipLaunchKernelGGL((k_grad_cols<false>), grid, dim3(kBlock), 0, st, ld, x, grads, d, rpc);
  return hipGetLastError();
}

}  // namespace adacgd
