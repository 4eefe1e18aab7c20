// Rank-K levels of the AdaCGD cascade (Section 2.1 names Rank-K beside Top-K as a contractive
// compressor for matrix-shaped arguments): the compressor's argument v = x - h, read row-major as a
// matrix X of r = d/c rows and c columns, is replaced by its best rank-K approximation X_K = X P_K,
// P_K the projector onto the K leading right singular vectors.  Per node:
//   gram      : G = X^T X (c x c, fp64: products of fp32 values are exact, sums in fp64), block partial
//               sums added in block order by the node's last block
//   eig       : one block diagonalises G by cyclic Jacobi rotations in a parallel (round-robin) order, all in
//               LDS, sorts the eigenvalues (squared singular values) and forms P_K for every Rank-K level
//   rank_err  : realised error || v - fl32(X P_K) ||^2 of every Rank-K level (left side of the trigger,
//               Eq. (10), evaluated on the rounded message like every other level's)
//   rank_apply: for nodes whose chosen level is a Rank-K level: C(v) = fl32(X P_K), h <- h + C(v)
//               (Eq. (7)) and the dense message the aggregation adds
// All Rank-K levels of a level set share c (16, 32 or 64), so one decomposition serves them all.
// The two projection kernels are dense contractions with a c x c matrix, run as fp64 FMAs on register
// tiles (the fp64 matrix and vector peaks of the device coincide, and the arithmetic has to be fp64 for
// the realised errors to meet the 1e-12 bar of the other reductions).
#include "devutil.h"
#include "engine.h"

namespace adacgd {

constexpr int kRankRows = 64;        // rows of X staged in LDS at a time

// Loads kRankRows rows (starting at row r0) of X = (x - h) into LDS, zero beyond the last row.
template <bool DIFF, int C>
__device__ __forceinline__ void stage_rows(const float* __restrict__ x, const float* __restrict__ h, int64_t r0,
                                           int64_t rows, float (*tile)[C]) {
  const int64_t base = r0 * C, end = rows * C;
  for (int e = threadIdx.x; e < kRankRows * C; e += kBlock) {
    const int64_t l = base + e;
    float v = 0.f;
    if (l < end) v = DIFF ? x[l] : x[l] - h[l];
    tile[e / C][e % C] = v;
  }
}

// ---------------------------------------------------------------------------
// gram
// ---------------------------------------------------------------------------
template <bool DIFF, int C>
__global__ __launch_bounds__(kBlock) void k_gram(NodeSet ns, PassArgs a) {
  constexpr int TS = C / 16;           // every thread owns a TS x TS tile of G
  __shared__ float tile[kRankRows][C];
  __shared__ int s_flag;
  const int node = blockIdx.y, tid = threadIdx.x;
  if (ns.skip[node] != 0) return;
  const int64_t d = ns.d, rows = d / C;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  const float* __restrict__ h = a.h + row;
  const int ty = tid / 16, tx = tid % 16;
  double acc[TS][TS];
#pragma unroll
  for (int i = 0; i < TS; ++i)
#pragma unroll
    for (int j = 0; j < TS; ++j) acc[i][j] = 0.0;
  const int64_t per = (rows + gridDim.x - 1) / gridDim.x;
  const int64_t rlo = (int64_t)blockIdx.x * per, rhi = min(rows, rlo + per);
  for (int64_t r0 = rlo; r0 < rhi; r0 += kRankRows) {
    __syncthreads();
    stage_rows<DIFF, C>(x, h, r0, rhi, tile);
    __syncthreads();
    for (int rr = 0; rr < kRankRows; ++rr) {
      double u[TS], w[TS];
#pragma unroll
      for (int i = 0; i < TS; ++i) {
        u[i] = (double)tile[rr][ty * TS + i];
        w[i] = (double)tile[rr][tx * TS + i];
      }
#pragma unroll
      for (int i = 0; i < TS; ++i)
#pragma unroll
        for (int j = 0; j < TS; ++j) acc[i][j] = fma(u[i], w[j], acc[i][j]);
    }
  }
  double* part = ns.gram_part + ((size_t)node * ns.GR + blockIdx.x) * (C * C);
#pragma unroll
  for (int i = 0; i < TS; ++i)
#pragma unroll
    for (int j = 0; j < TS; ++j) st_coherent(&part[(ty * TS + i) * C + tx * TS + j], acc[i][j]);
  if (!arrive_last_few(&ns.done[(size_t)node * (kArriveFan + 1) * kCounterStride], gridDim.x, &s_flag)) return;
  double* G = ns.gram + (size_t)node * (C * C);
  for (int e = tid; e < C * C; e += kBlock) {
    double t = 0.0;
    for (int b = 0; b < (int)gridDim.x; ++b)
      t += ld_coherent(&ns.gram_part[((size_t)node * ns.GR + b) * (C * C) + e]);
    G[e] = t;
  }
}

// ---------------------------------------------------------------------------
// eig: cyclic Jacobi on the c x c Gram matrix, one block per node.  A round rotates c/2 disjoint
// index pairs at once (round-robin order: c - 1 rounds visit every pair once); a sweep is c - 1
// rounds.  Sweeps stop when the off-diagonal mass has reached its rounding floor, at most kMaxSweeps.
// ---------------------------------------------------------------------------
constexpr int kMaxSweeps = 40;

// one work item per thread in the matrix update of a round: (c/2)^2 threads, at least one block of 256
template <int C>
constexpr int eig_threads() { return (C / 2) * (C / 2) > kBlock ? (C / 2) * (C / 2) : kBlock; }

template <int C>
__global__ __launch_bounds__(eig_threads<C>()) void k_eig(NodeSet ns) {
  constexpr int NT = eig_threads<C>();
  // Two copies of the matrix (a round reads one and writes the other: every new entry is a combination of
  // four old ones, so no barrier is needed between the row and the column half of the rotation) and the
  // eigenvector matrix, rows padded by one entry so that walking a column touches every LDS bank.
  __shared__ double Abuf[2][C][C + 1];
  __shared__ double V[C][C + 1];
  __shared__ double s_cs[C / 2], s_sn[C / 2];
  __shared__ int s_p[C / 2], s_q[C / 2];
  __shared__ double red[2][NT / 64];
  __shared__ int s_rank[C];
  __shared__ int s_stop;
  const int node = blockIdx.x, tid = threadIdx.x;
  if (ns.skip[node] != 0) return;
  const double* __restrict__ G = ns.gram + (size_t)node * (C * C);
  for (int e = tid; e < C * C; e += NT) {
    Abuf[0][e / C][e % C] = G[e];
    V[e / C][e % C] = (e / C == e % C) ? 1.0 : 0.0;
  }
  int cur = 0;
  double off_prev = 0.0;
  __syncthreads();
  for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
    // off-diagonal against diagonal mass
    double off = 0.0, dia = 0.0;
    for (int e = tid; e < C * C; e += NT) {
      const double v = Abuf[cur][e / C][e % C];
      if (e / C == e % C) dia = fma(v, v, dia); else off = fma(v, v, off);
    }
    off = wave_sum(off);
    dia = wave_sum(dia);
    if ((tid & 63) == 0) { red[0][tid >> 6] = off; red[1][tid >> 6] = dia; }
    __syncthreads();
    // Convergence is quadratic until the rounding floor is reached: stop when the off-diagonal mass is
    // negligible, or when a sweep no longer reduces it fourfold (the floor).
    if (tid == 0) {
      off = dia = 0.0;
      for (int i = 0; i < NT / 64; ++i) { off += red[0][i]; dia += red[1][i]; }
      s_stop = (off <= 1e-34 * dia || (sweep >= 3 && off >= 0.25 * off_prev)) ? 1 : 0;
      off_prev = off;
    }
    __syncthreads();
    if (s_stop) break;                            // (the same in every thread)
    for (int m = 0; m < C - 1; ++m) {
      double (*A)[C + 1] = Abuf[cur];
      double (*B)[C + 1] = Abuf[cur ^ 1];
      if (tid < C / 2) {
        int p, q;
        if (tid == 0) { p = C - 1; q = m; }
        else { p = (m + tid) % (C - 1); q = (m - tid + (C - 1)) % (C - 1); }
        if (p > q) { const int t = p; p = q; q = t; }
        const double app = A[p][p], aqq = A[q][q], apq = A[p][q];
        double cs = 1.0, sn = 0.0;
        if (apq != 0.0) {
          const double theta = (aqq - app) / (2.0 * apq);
          const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
          cs = 1.0 / sqrt(t * t + 1.0);
          sn = t * cs;
        }
        s_p[tid] = p; s_q[tid] = q; s_cs[tid] = cs; s_sn[tid] = sn;
      }
      __syncthreads();
      // B = J^T A J, one 2 x 2 block (rows of pair ka, columns of pair kb) per work item
      for (int e = tid; e < (C / 2) * (C / 2); e += NT) {
        const int ka = e / (C / 2), kb = e % (C / 2);
        const int p = s_p[ka], q = s_q[ka], r = s_p[kb], u = s_q[kb];
        const double ca = s_cs[ka], sa = s_sn[ka], cb = s_cs[kb], sb = s_sn[kb];
        const double apr = A[p][r], apu = A[p][u], aqr = A[q][r], aqu = A[q][u];
        // rows first (J^T A) ...
        const double tpr = ca * apr - sa * aqr, tpu = ca * apu - sa * aqu;
        const double tqr = sa * apr + ca * aqr, tqu = sa * apu + ca * aqu;
        // ... then columns
        B[p][r] = cb * tpr - sb * tpu;
        B[p][u] = sb * tpr + cb * tpu;
        B[q][r] = cb * tqr - sb * tqu;
        B[q][u] = sb * tqr + cb * tqu;
      }
      for (int e = tid; e < (C / 2) * C; e += NT) {       // V <- V J: columns p, q of every pair
        const int k = e / C, i = e % C;
        const int p = s_p[k], q = s_q[k];
        const double cs = s_cs[k], sn = s_sn[k];
        const double vp = V[i][p], vq = V[i][q];
        V[i][p] = cs * vp - sn * vq;
        V[i][q] = sn * vp + cs * vq;
      }
      cur ^= 1;
      __syncthreads();
    }
  }
  __syncthreads();
  double (*A)[C + 1] = Abuf[cur];
  // eigenvalues in descending order (ties by index): position of each, then the sorted list
  if (tid < C) {
    const double li = A[tid][tid];
    int rk = 0;
    for (int j = 0; j < C; ++j) {
      const double lj = A[j][j];
      rk += (lj > li || (lj == li && j < tid)) ? 1 : 0;
    }
    s_rank[tid] = rk;
    ns.rk_lambda[(size_t)node * C + rk] = li;
  }
  __syncthreads();
  // projector onto the K leading eigenvectors, for every Rank-K level
  for (int r = 0; r < ns.lv.nr; ++r) {
    const int K = ns.lv.rK[r];
    double* __restrict__ P = ns.rk_P + ((size_t)node * ns.lv.nr + r) * (C * C);
    for (int e = tid; e < C * C; e += NT) {
      const int i = e / C, j = e % C;
      double t = 0.0;
      for (int k = 0; k < C; ++k)
        if (s_rank[k] < K) t = fma(V[i][k], V[j][k], t);
      P[e] = t;
    }
  }
}

// ---------------------------------------------------------------------------
// projection X P: every thread owns 4 rows x TS columns of a 64-row chunk
// ---------------------------------------------------------------------------
template <int C>
__device__ __forceinline__ void project_chunk(const float (*tile)[C], const double (*P)[C], int ty, int tx,
                                              double (&out)[4][C / 16]) {
  constexpr int TS = C / 16;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TS; ++j) out[i][j] = 0.0;
  for (int k = 0; k < C; ++k) {
    double u[4], w[TS];
#pragma unroll
    for (int i = 0; i < 4; ++i) u[i] = (double)tile[ty * 4 + i][k];
#pragma unroll
    for (int j = 0; j < TS; ++j) w[j] = P[k][tx * TS + j];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TS; ++j) out[i][j] = fma(u[i], w[j], out[i][j]);
  }
}

template <bool DIFF, int C>
__global__ __launch_bounds__(kBlock) void k_rank_err(NodeSet ns, PassArgs a) {
  constexpr int TS = C / 16;
  __shared__ float tile[kRankRows][C];
  __shared__ double P[C][C];
  __shared__ double red[4];
  __shared__ int s_flag;
  const int node = blockIdx.y, tid = threadIdx.x;
  if (ns.skip[node] != 0) return;
  const int64_t d = ns.d, rows = d / C;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  const float* __restrict__ h = a.h + row;
  const int ty = tid / 16, tx = tid % 16;
  const int nr = ns.lv.nr;
  const int64_t per = (rows + gridDim.x - 1) / gridDim.x;
  const int64_t rlo = (int64_t)blockIdx.x * per, rhi = min(rows, rlo + per);
  for (int r = 0; r < nr; ++r) {
    __syncthreads();
    const double* __restrict__ Pg = ns.rk_P + ((size_t)node * nr + r) * (C * C);
    for (int e = tid; e < C * C; e += kBlock) P[e / C][e % C] = Pg[e];
    double err = 0.0;
    for (int64_t r0 = rlo; r0 < rhi; r0 += kRankRows) {
      __syncthreads();
      stage_rows<DIFF, C>(x, h, r0, rhi, tile);
      __syncthreads();
      double out[4][TS];
      project_chunk<C>(tile, P, ty, tx, out);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TS; ++j) {
          const float c32 = (float)out[i][j];                       // the message is fp32
          const double e = (double)tile[ty * 4 + i][tx * TS + j] - (double)c32;
          err = fma(e, e, err);
        }
    }
    err = block_sum(err, red);
    if (tid == 0) st_coherent(&ns.rk_part[((size_t)node * ns.GR + blockIdx.x) * nr + r], err);
  }
  if (!arrive_last_few(&ns.done[(size_t)node * (kArriveFan + 1) * kCounterStride], gridDim.x, &s_flag)) return;
  if (tid < nr) {
    double t = 0.0;
    for (int b = 0; b < (int)gridDim.x; ++b) t += ld_coherent(&ns.rk_part[((size_t)node * ns.GR + b) * nr + tid]);
    ns.rk_err[(size_t)node * nr + tid] = t;
  }
}

template <bool DIFF, int C>
__global__ __launch_bounds__(kBlock) void k_rank_apply(NodeSet ns, PassArgs a) {
  constexpr int TS = C / 16;
  __shared__ float tile[kRankRows][C];
  __shared__ double P[C][C];
  const int node = blockIdx.y, tid = threadIdx.x;
  const int r = ns.sel_rk[node];
  if (r < 0) return;
  const int64_t d = ns.d, rows = d / C;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  float* __restrict__ h = a.h + row;
  float* __restrict__ dense = ns.rdense + row;
  const int ty = tid / 16, tx = tid % 16;
  const double* __restrict__ Pg = ns.rk_P + ((size_t)node * ns.lv.nr + r) * (C * C);
  for (int e = tid; e < C * C; e += kBlock) P[e / C][e % C] = Pg[e];
  const int64_t per = (rows + gridDim.x - 1) / gridDim.x;
  const int64_t rlo = (int64_t)blockIdx.x * per, rhi = min(rows, rlo + per);
  for (int64_t r0 = rlo; r0 < rhi; r0 += kRankRows) {
    __syncthreads();
    stage_rows<DIFF, C>(x, h, r0, rhi, tile);
    __syncthreads();
    double out[4][TS];
    project_chunk<C>(tile, P, ty, tx, out);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t rr = r0 + ty * 4 + i;
      if (rr < rhi) {
#pragma unroll
        for (int j = 0; j < TS; ++j) {
          const int64_t l = rr * C + tx * TS + j;
          const float c32 = (float)out[i][j];
          dense[l] = c32;
          h[l] = h[l] + c32;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
template <int C>
static hipError_t launch_rank_c(int which, const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  const dim3 grid(ns.GR, ns.nn), block(kBlock);
  switch (which) {
    case 0:
      if (a.diff) hipLaunchKernelGGL((k_gram<true, C>), grid, block, 0, st, ns, a);
      else hipLaunchKernelGGL((k_gram<false, C>), grid, block, 0, st, ns, a);
      break;
    case 1:
      hipLaunchKernelGGL((k_eig<C>), dim3(ns.nn), dim3(eig_threads<C>()), 0, st, ns);
      break;
    case 2:
      if (a.diff) hipLaunchKernelGGL((k_rank_err<true, C>), grid, block, 0, st, ns, a);
      else hipLaunchKernelGGL((k_rank_err<false, C>), grid, block, 0, st, ns, a);
      break;
    default:
      if (a.diff) hipLaunchKernelGGL((k_rank_apply<true, C>), grid, block, 0, st, ns, a);
      else hipLaunchKernelGGL((k_rank_apply<false, C>), grid, block, 0, st, ns, a);
      break;
  }
  return hipGetLastError();
}

static hipError_t launch_rank(int which, const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  (void)hipGetLastError();
  switch (ns.lv.rcols) {
    case 16: return launch_rank_c<16>(which, ns, a, st);
    case 32: return launch_rank_c<32>(which, ns, a, st);
    case 64: return launch_rank_c<64>(which, ns, a, st);
    default: return hipErrorInvalidValue;
  }
}

// Gram matrix, its eigen-decomposition and the realised error of every Rank-K level (before the level choice)
hipError_t launch_rank_errors(const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  hipError_t e = launch_rank(0, ns, a, st);
  if (e != hipSuccess) return e;
  e = launch_rank(1, ns, a, st);
  if (e != hipSuccess) return e;
  return launch_rank(2, ns, a, st);
}

// Estimator update and dense message of the nodes whose chosen level is a Rank-K level
hipError_t launch_rank_apply(const NodeSet& ns, const PassArgs& a, hipStream_t st) { return launch_rank(3, ns, a, st); }

}  // namespace adacgd
