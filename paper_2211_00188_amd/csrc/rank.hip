// Rank-K levels of the AdaCGD cascade (Section 2.1 names Rank-K beside Top-K as a contractive
// compressor for matrix-shaped arguments): the compressor's argument v = x - h, read row-major as a
// matrix X of r = d/c rows and c columns, is replaced by its best rank-K approximation
// X_K = (X V_K) V_K^T, V_K the K leading right singular vectors.  Per node:
//   gram      : G = X^T X (c x c, fp64: products of fp32 values are exact, sums in fp64), the upper
//               triangle as 16 x 16 tiles on the fp64 matrix cores, one partial sum per block
//   eig       : one block adds the partial sums in block order and diagonalises G by cyclic Jacobi
//               rotations in a parallel (round-robin) order, all in
//               LDS, and leaves the eigenvalues (squared singular values) in descending order with their
//               eigenvectors
//   rank_err  : realised error || v - fl32(X_K) ||^2 of every Rank-K level (left side of the trigger,
//               Eq. (10), evaluated on the rounded message like every other level's)
//   rank_apply: for nodes whose chosen level is a Rank-K level: C(v) = fl32(X_K), h <- h + C(v)
//               (Eq. (7)) and the dense message the aggregation adds
// All Rank-K levels of a level set share c (16, 32 or 64), so one decomposition serves them all.
// Gram matrix and projections are dense fp64 contractions and run as 16 x 16 x 4 matrix instructions
// (the arithmetic has to be fp64 for the realised errors to meet the 1e-12 bar of the other reductions;
// the device's fp64 matrix and vector peaks coincide, what the matrix cores save is operand delivery:
// two LDS reads per 1024 multiply-adds instead of one per two).
#include "devutil.h"
#include "engine.h"

namespace adacgd {

typedef double d4 __attribute__((ext_vector_type(4)));

constexpr int kRankRows = 64;        // rows of X staged in LDS at a time: 16 per wavefront
constexpr int kRowPad = 4;           // floats of padding per staged row: 16 rows x 4 columns hit 64 different banks

// D += A B for A (16 x 4) and B (4 x 16): lane l passes A[l % 16][l / 16] and B[l / 16][l % 16];
// register v of lane l holds D[l / 16 + 4 v][l % 16].
__device__ __forceinline__ d4 mma(double a, double b, d4 c) { return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0); }

// kRankRows rows of X = (x - h) on their way into LDS: `fetch` loads a thread's share (16-byte loads; rows
// are 64-byte aligned because d is a multiple of c >= 16 and the vectors are 16-byte aligned) into registers,
// zero beyond row `rows`; `store` puts it into the tile.  Fetching the next chunk before working on the
// current one keeps the loads in flight during the matrix instructions.
template <bool DIFF, int C>
struct Stager {
  static constexpr int NV = kRankRows * C / 4 / kBlock;        // 16-byte pieces per thread: c / 16
  float4 v[NV];
  __device__ __forceinline__ void fetch(const float* __restrict__ x, const float* __restrict__ h, int64_t r0, int64_t rows) {
    const int64_t base = r0 * C, end = rows * C;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int64_t l = base + (int64_t)(u * kBlock + threadIdx.x) * 4;
      float4 xv = make_float4(0.f, 0.f, 0.f, 0.f), hv = xv;
      if (l < end) {                                           // (l and end are multiples of four)
        xv = *reinterpret_cast<const float4*>(x + l);
        if (!DIFF) hv = *reinterpret_cast<const float4*>(h + l);
      }
      v[u] = make_float4(xv.x - hv.x, xv.y - hv.y, xv.z - hv.z, xv.w - hv.w);
    }
  }
  __device__ __forceinline__ void store(float (*tile)[C + kRowPad]) const {
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int e = (u * kBlock + threadIdx.x) * 4;
      *reinterpret_cast<float4*>(&tile[e / C][e % C]) = v[u];   // (a padded row is a whole number of 16 bytes)
    }
  }
};

// ---------------------------------------------------------------------------
// gram: every wavefront owns 16 rows of a staged chunk and all tiles of the upper triangle
// ---------------------------------------------------------------------------
template <bool DIFF, int C>
__global__ __launch_bounds__(kBlock) void k_gram(NodeSet ns, PassArgs a) {
  constexpr int NB = C / 16, NT = NB * (NB + 1) / 2;      // column blocks, tiles (ci <= cj)
  __shared__ __align__(16) float tile[kRankRows][C + kRowPad];
  __shared__ double red[NT * 256];                        // a tile as [lane][register]
  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  if (ns.skip[node] != 0) return;
  const int64_t d = ns.d, rows = d / C;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  const float* __restrict__ h = a.h + row;
  d4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = d4{0.0, 0.0, 0.0, 0.0};
  const int64_t per = (rows + gridDim.x - 1) / gridDim.x;
  const int64_t rlo = (int64_t)blockIdx.x * per, rhi = min(rows, rlo + per);
  Stager<DIFF, C> stg;
  if (rlo < rhi) stg.fetch(x, h, rlo, rhi);
  for (int64_t r0 = rlo; r0 < rhi; r0 += kRankRows) {
    __syncthreads();
    stg.store(tile);
    __syncthreads();
    if (r0 + kRankRows < rhi) stg.fetch(x, h, r0 + kRankRows, rhi);
#pragma unroll
    for (int s = 0; s < 4; ++s) {                          // four rows per instruction
      const int r = 16 * w + 4 * s + (l >> 4);
      double val[NB];
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) val[cb] = (double)tile[r][cb * 16 + (l & 15)];
      int t = 0;
#pragma unroll
      for (int ci = 0; ci < NB; ++ci)
#pragma unroll
        for (int cj = ci; cj < NB; ++cj) { acc[t] = mma(val[ci], val[cj], acc[t]); ++t; }
    }
  }
  // the four wavefronts' sums, added in wavefront order
  for (int ww = 0; ww < 4; ++ww) {
    if (w == ww) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          double* slot = &red[(t * 64 + l) * 4 + v];
          *slot = (ww == 0 ? 0.0 : *slot) + acc[t][v];
        }
    }
    __syncthreads();
  }
  // the block's partial sums, tile by tile as [lane][register] (NT * 256 <= c * c entries); eig adds the blocks up
  double* part = ns.gram_part + ((size_t)node * ns.GR + blockIdx.x) * (C * C);
  for (int e = tid; e < NT * 256; e += kBlock) part[e] = red[e];
}

// ---------------------------------------------------------------------------
// eig: cyclic Jacobi on the c x c Gram matrix, one block per node.  A round rotates c/2 disjoint
// index pairs at once; a sweep is c - 1 rounds in the round-robin (tournament) order, which visits every
// pair once.  The schedule is kept in the data, not in indices: the matrix lives in c "positions", position k
// (top) always paired with position c/2 + k (bottom), and every round ends by moving rows and columns one
// place along the tournament's cycle while they are written back.  Every thread therefore reads and writes
// the same LDS addresses in every round (unit stride across lanes, no index arithmetic in the loop), and the
// eigenvector matrix stays in registers: a thread owns two rows of one position pair, and the cyclic move is
// a shift by one lane.  Which original index sits where never matters: rows of V are coordinates, its columns
// travel with the positions, and the eigenvalues are sorted at the end.
// Sweeps stop when the off-diagonal mass is negligible, or is below 1e-22 of the diagonal mass and a sweep no
// longer reduces it fourfold (the rounding floor, about c^2 2^-106 of the diagonal; convergence is quadratic
// on the way there, while the first sweeps may well gain less than a factor of four), at most kMaxSweeps.
// ---------------------------------------------------------------------------
constexpr int kMaxSweeps = 40;

// one 2 x 2 block per thread in the matrix update of a round: (c/2)^2 threads, at least one block of 256
template <int C>
constexpr int eig_threads() { return (C / 2) * (C / 2) > kBlock ? (C / 2) * (C / 2) : kBlock; }

// 1/x and 1/sqrt(x) for normal x > 0 from the hardware's approximations and STEPS Newton steps (every step
// squares the relative error; the approximations start with well over ten good bits, so three steps are
// exact to rounding and one is good to a few parts in a million at worst).
template <int STEPS>
__device__ __forceinline__ double newton_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
#pragma unroll
  for (int i = 0; i < STEPS; ++i) r = fma(fma(-x, r, 1.0), r, r);
  return r;
}
template <int STEPS>
__device__ __forceinline__ double newton_rsq(double x) {
  double r = __builtin_amdgcn_rsq(x);
#pragma unroll
  for (int i = 0; i < STEPS; ++i) r = fma(0.5 * r, fma(-x * r, r, 1.0), r);
  return r;
}

// The value of the lane below (up = true) or above (up = false) in the wavefront, by two data-parallel moves
// (no LDS traffic); the first and the last lane of the wavefront get their own value back.
template <bool UP>
__device__ __forceinline__ double lane_shift(double x) {
  constexpr int ctrl = UP ? 0x138 : 0x130;             // wave_shr:1 / wave_shl:1
  const int lo = __double2loint(x), hi = __double2hiint(x);
  const int nlo = __builtin_amdgcn_update_dpp(lo, lo, ctrl, 0xf, 0xf, false);
  const int nhi = __builtin_amdgcn_update_dpp(hi, hi, ctrl, 0xf, 0xf, false);
  return __hiloint2double(nhi, nlo);
}

// where the row / column at position `pos` goes at the end of a round (H = c/2 pairs; positions 0 .. H-1 are
// the tops, H .. 2H-1 the bottoms): top 0 stays, the other tops move up by one, the last top becomes the last
// bottom, the bottoms move down by one and bottom 0 becomes top 1
template <int H>
__device__ __forceinline__ int next_pos(int pos) {
  if (pos == 0) return 0;
  if (pos < H - 1) return pos + 1;
  if (pos == H - 1) return 2 * H - 1;
  if (pos == H) return 1;
  return pos - 1;
}

template <int C>
__global__ __launch_bounds__(eig_threads<C>()) void k_eig(NodeSet ns) {
  constexpr int NT = eig_threads<C>();
  constexpr int H = C / 2;
  constexpr int GROUPS = NT / H;                         // threads with the same pair index
  constexpr int RPT = C / GROUPS > 0 ? C / GROUPS : 1;    // rows of V per thread (2, 2, 1 for c = 64, 32, 16)
  // Two copies of the matrix: a round reads one and writes the other (every new entry is a combination of
  // four old ones, so no barrier is needed between the row and the column half of the rotation).
  __shared__ double Abuf[2][C][C + 1];
  __shared__ double V[C][C + 1];                         // the eigenvectors, once the sweeps are over
  __shared__ double2 s_rot[H];                           // (cos, sin) of the round's rotations
  __shared__ double red[2][NT / 64];
  __shared__ int s_rank[C];
  __shared__ int s_stop;
  const int node = blockIdx.x, tid = threadIdx.x;
  if (ns.skip[node] != 0) return;
  // G from the partial sums of the Gram kernel's blocks, added in block order (16 loads in flight), its tiles
  // unpacked into the full symmetric matrix (inside a diagonal tile both halves were computed, from the same
  // products in the same order)
  constexpr int NB = C / 16, NTL = NB * (NB + 1) / 2;
  const double* __restrict__ part = ns.gram_part + (size_t)node * ns.GR * (C * C);
  for (int e = tid; e < NTL * 256; e += NT) {
    double t = 0.0;
    for (int b0 = 0; b0 < ns.GR; b0 += 16) {
      double pv[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) pv[u] = b0 + u < ns.GR ? part[(size_t)(b0 + u) * (C * C) + e] : 0.0;
#pragma unroll
      for (int u = 0; u < 16; ++u) t += pv[u];
    }
    int ci = 0, rem = e / 256;
    while (rem >= NB - ci) { rem -= NB - ci; ++ci; }
    const int cj = ci + rem, ll = (e % 256) / 4, v = e % 4;
    const int i = ci * 16 + (ll >> 4) + 4 * v, j = cj * 16 + (ll & 15);
    Abuf[0][i][j] = t;
    if (ci != cj) Abuf[0][j][i] = t;
  }
  // This thread's 2 x 2 block of the matrix update: rows (top ka, bottom ka), columns (top kb, bottom kb).
  // (Updating only the blocks with ka <= kb and writing their transposes along was slower: the saving only
  // counts where whole wavefronts drop out, and those that remain then carry the round.)
  const bool item = tid < H * H;
  const int rT = item ? tid / H : 0, rB = H + rT, cT = tid % H, cB = H + cT;
  const int wrT = next_pos<H>(rT), wrB = next_pos<H>(rB), wcT = next_pos<H>(cT), wcB = next_pos<H>(cB);
  // ... and its rows of V: pair kv, rows vrow .. vrow + RPT - 1; V = I to start with
  const int kv = tid % H;
  const int vrow = (tid / H) * RPT;
  const bool vitem = vrow < C;
  double vt[RPT], vb[RPT];
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    vt[r] = (vrow + r == kv) ? 1.0 : 0.0;
    vb[r] = (vrow + r == H + kv) ? 1.0 : 0.0;
  }
  // V <- V J, columns moved along the cycle: the new top of pair k is the old top of pair k - 1 (pair 1: the
  // old bottom of pair 0; pair 0 keeps its top), the new bottom the old bottom of pair k + 1 (the last pair:
  // its own old top).  Lanes with the same rows are H neighbours; what crosses from one such group to the
  // next is not used: pair 0 ignores `up`, the last pair ignores `down`.
  auto rotate_v = [&](const double2 rk) {
    const double cs = rk.x, sn = rk.y;
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      const double nt = fma(cs, vt[r], -(sn * vb[r]));
      const double nb = fma(sn, vt[r], cs * vb[r]);
      const double up = lane_shift<true>(kv == 0 ? nb : nt);
      const double down = lane_shift<false>(nb);
      vt[r] = kv == 0 ? nt : up;
      vb[r] = kv == H - 1 ? nt : down;
    }
  };
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
    if (tid == 0) {
      off = dia = 0.0;
      for (int i = 0; i < NT / 64; ++i) { off += red[0][i]; dia += red[1][i]; }
      s_stop = (off <= 1e-34 * dia || (sweep >= 1 && off <= 1e-22 * dia && off >= 0.25 * off_prev)) ? 1 : 0;
      off_prev = off;
    }
    __syncthreads();
    if (s_stop) break;                            // (the same in every thread)
    for (int m = 0; m < C - 1; ++m) {
      double (*A)[C + 1] = Abuf[cur];
      double (*B)[C + 1] = Abuf[cur ^ 1];
      if (tid < H) {
        // Rotation that annihilates A[p][q], p = top tid, q = bottom tid: with a = A[q][q] - A[p][p] and
        // b = 2 A[p][q] the tangent is t = sign(a b) |b| / (|a| + sqrt(a^2 + b^2)), the smaller root (no division
        // by b: the denominator is at least |b|).  (cs, sn) = (1, t) / sqrt(1 + t^2) is orthogonal to rounding
        // whatever t is, and that is all the decomposition needs of it; an inexact t only leaves a smaller
        // A[p][q] for the next sweep.
        const double app = A[tid][tid], aqq = A[H + tid][H + tid], apq = A[tid][H + tid];
        double cs = 1.0, sn = 0.0;
        const double ga = aqq - app, gb = 2.0 * apq;
        const double hyp2 = fma(ga, ga, gb * gb);
        // (an element so small that its square leaves the normal range is as good as annihilated; the bounds
        // also keep the approximations below away from zero, infinity and NaN)
        if (apq != 0.0 && hyp2 >= 1e-290 && hyp2 <= 1e290) {
          const double hyp = hyp2 * newton_rsq<1>(hyp2);          // (the tangent need not be exact, see above)
          double t = fabs(gb) * newton_rcp<1>(fabs(ga) + hyp);
          if ((ga < 0.0) != (gb < 0.0)) t = -t;
          cs = newton_rsq<3>(fma(t, t, 1.0));                     // (the normalisation has to be)
          sn = t * cs;
        }
        s_rot[tid] = make_double2(cs, sn);
      }
      __syncthreads();
      // B = J^T A J, moved along the cycle
      if (item) {
        const double2 ra = s_rot[rT], rb = s_rot[cT];
        const double ca = ra.x, sa = ra.y, cb = rb.x, sb = rb.y;
        const double att = A[rT][cT], atb = A[rT][cB], abt = A[rB][cT], abb = A[rB][cB];
        // rows first (J^T A) ...
        const double ttt = fma(ca, att, -(sa * abt)), ttb = fma(ca, atb, -(sa * abb));
        const double tbt = fma(sa, att, ca * abt), tbb = fma(sa, atb, ca * abb);
        // ... then columns
        const double ntt = fma(cb, ttt, -(sb * ttb)), ntb = fma(sb, ttt, cb * ttb);
        const double nbt = fma(cb, tbt, -(sb * tbb)), nbb = fma(sb, tbt, cb * tbb);
        B[wrT][wcT] = ntt; B[wrT][wcB] = ntb; B[wrB][wcT] = nbt; B[wrB][wcB] = nbb;
      }
      // (The eigenvector update is registers only and fills the waits of the matrix update; moving it
      // under the rotation phase of the next round, where most wavefronts idle, was slower: it then
      // lengthens the one wavefront everybody waits for.)
      rotate_v(s_rot[kv]);
      cur ^= 1;
      __syncthreads();
    }
  }
  if (vitem) {
#pragma unroll
    for (int r = 0; r < RPT; ++r) { V[vrow + r][kv] = vt[r]; V[vrow + r][H + kv] = vb[r]; }
  }
  __syncthreads();
  double (*A)[C + 1] = Abuf[cur];
  // eigenvalues in descending order (ties by position): rank of each, then the sorted list
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
  // eigenvectors as the columns of a row-major c x c matrix, in the order of their eigenvalues
  double* __restrict__ Vout = ns.rk_V + (size_t)node * (C * C);
  for (int e = tid; e < C * C; e += NT) Vout[(e / C) * C + s_rank[e % C]] = V[e / C][e % C];
}

// ---------------------------------------------------------------------------
// Projection of a staged chunk onto the leading eigenvectors.  LDS (dynamic): the first KP eigenvectors
// Vs[j][k], per wavefront its 16 rows of Y = X V, and the staged rows (fp32).  The leading dimension of Vs
// and Ys is 2 modulo 32 doubles, so that the 16 rows x 2 columns a half-wavefront reads for a transposed
// operand fall into 32 different bank pairs.
// ---------------------------------------------------------------------------
__host__ __device__ inline int proj_ld(int kp) { return ((kp + 31) / 32) * 32 + 2; }

template <int C>
struct ProjLds {
  float (*tile)[C + kRowPad];
  double* Vs;        // [C][ld]
  double* Ys;        // [4][16][ld]
  int KP, ld;
  __device__ ProjLds(unsigned char* base, int kp) {
    KP = kp; ld = proj_ld(kp);
    Vs = reinterpret_cast<double*>(base);
    Ys = Vs + (size_t)C * ld;
    tile = reinterpret_cast<float (*)[C + kRowPad]>(Ys + (size_t)4 * 16 * ld);
  }
  static size_t bytes(int kp) {
    return sizeof(double) * ((size_t)C + 4 * 16) * proj_ld(kp) + sizeof(float) * kRankRows * (C + kRowPad);
  }
  __device__ void load_vectors(const double* __restrict__ Vg) {       // Vg[j][k], row-major c x c
    for (int e = threadIdx.x; e < C * KP; e += kBlock) Vs[(e / KP) * ld + e % KP] = Vg[(e / KP) * C + e % KP];
  }
  // Y = X V for the wavefront's 16 staged rows, all KP columns, left in Ys (rows x KP)
  __device__ void project(int w, int l) {
    for (int kb = 0; kb < KP / 16; ++kb) {
      d4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
      for (int j0 = 0; j0 < C; j0 += 4)
        acc = mma((double)tile[16 * w + (l & 15)][j0 + (l >> 4)], Vs[(j0 + (l >> 4)) * ld + kb * 16 + (l & 15)], acc);
#pragma unroll
      for (int v = 0; v < 4; ++v) Ys[(w * 16 + (l >> 4) + 4 * v) * ld + kb * 16 + (l & 15)] = acc[v];
    }
  }
  // the wavefront's 16 rows of X_K = Y V_K^T, one 16 x 16 tile per column block (independent accumulators:
  // the matrix instructions of the c / 16 tiles follow each other without waiting)
  __device__ void expand(int w, int l, int K, d4 (&out)[C / 16]) const {
#pragma unroll
    for (int cb = 0; cb < C / 16; ++cb) out[cb] = d4{0.0, 0.0, 0.0, 0.0};
    for (int kk = 0; kk < K; kk += 4) {
      const int k = kk + (l >> 4);                                     // < KP: a whole number of 16-column blocks
      const double y = Ys[(w * 16 + (l & 15)) * ld + k];
      double b[C / 16];
#pragma unroll
      for (int cb = 0; cb < C / 16; ++cb) b[cb] = k < K ? Vs[(cb * 16 + (l & 15)) * ld + k] : 0.0;
#pragma unroll
      for (int cb = 0; cb < C / 16; ++cb) out[cb] = mma(y, b[cb], out[cb]);
    }
  }
};

// number of eigenvectors the projections need, rounded up to whole 16-column blocks
__host__ __device__ inline int proj_columns(const LevelTable& lv, int only) {
  int k = 0;
  for (int r = 0; r < lv.nr; ++r)
    if (only < 0 || r == only) k = lv.rK[r] > k ? lv.rK[r] : k;
  return (k + 15) & ~15;
}

template <bool DIFF, int C>
__global__ __launch_bounds__(kBlock) void k_rank_err(NodeSet ns, PassArgs a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ double s_err[4][kMaxLevels];                  // per wavefront and level
  __shared__ int s_flag;
  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  if (ns.skip[node] != 0) return;
  const int nr = ns.lv.nr;
  if (tid < 4 * kMaxLevels) s_err[tid / kMaxLevels][tid % kMaxLevels] = 0.0;
  ProjLds<C> L(lds_raw, proj_columns(ns.lv, -1));
  const int64_t d = ns.d, rows = d / C;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  const float* __restrict__ h = a.h + row;
  L.load_vectors(ns.rk_V + (size_t)node * (C * C));
  const int64_t per = (rows + gridDim.x - 1) / gridDim.x;
  const int64_t rlo = (int64_t)blockIdx.x * per, rhi = min(rows, rlo + per);
  Stager<DIFF, C> stg;
  if (rlo < rhi) stg.fetch(x, h, rlo, rhi);
  for (int64_t r0 = rlo; r0 < rhi; r0 += kRankRows) {
    __syncthreads();
    stg.store(L.tile);
    __syncthreads();
    if (r0 + kRankRows < rhi) stg.fetch(x, h, r0 + kRankRows, rhi);
    L.project(w, l);          // (a wavefront reads back only its own rows of Ys, in program order)
    double xt[C / 16][4];     // this lane's entries of X in the layout the tiles come out in
#pragma unroll
    for (int cb = 0; cb < C / 16; ++cb)
#pragma unroll
      for (int v = 0; v < 4; ++v) xt[cb][v] = (double)L.tile[16 * w + (l >> 4) + 4 * v][cb * 16 + (l & 15)];
    for (int r = 0; r < nr; ++r) {
      d4 out[C / 16];
      L.expand(w, l, ns.lv.rK[r], out);
      double e2 = 0.0;
#pragma unroll
      for (int cb = 0; cb < C / 16; ++cb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const double e = xt[cb][v] - (double)(float)out[cb][v];     // the message is fp32
          e2 = fma(e, e, e2);
        }
      e2 = wave_sum(e2);
      if (l == 0) s_err[w][r] += e2;        // (only this wavefront touches its row of s_err)
    }
  }
  __syncthreads();
  if (tid < nr) {
    const double e = ((s_err[0][tid] + s_err[1][tid]) + s_err[2][tid]) + s_err[3][tid];
    st_coherent(&ns.rk_part[((size_t)node * ns.GR + blockIdx.x) * nr + tid], e);
  }
  if (!arrive_last_few(&ns.done[(size_t)node * (kArriveFan + 1) * kCounterStride], gridDim.x, &s_flag)) return;
  // last block of the node: all partial errors in one round trip, then each level's sum in block order
  double* stash = reinterpret_cast<double*>(lds_raw);
  const int np = (int)gridDim.x * nr;                      // <= 64 * 16 entries: far below the LDS the kernel was given
  for (int e = tid; e < np; e += kBlock) stash[e] = ld_coherent(&ns.rk_part[(size_t)node * ns.GR * nr + e]);
  __syncthreads();
  if (tid < nr) {
    double t = 0.0;
    for (int b = 0; b < (int)gridDim.x; ++b) t += stash[b * nr + tid];
    ns.rk_err[(size_t)node * nr + tid] = t;
  }
}

template <bool DIFF, int C>
__global__ __launch_bounds__(kBlock) void k_rank_apply(NodeSet ns, PassArgs a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const int r = ns.sel_rk[node];
  if (r < 0) return;
  const int K = ns.lv.rK[r];
  ProjLds<C> L(lds_raw, proj_columns(ns.lv, r));
  const int64_t d = ns.d, rows = d / C;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  float* __restrict__ h = a.h + row;
  float* __restrict__ dense = ns.rdense + row;
  L.load_vectors(ns.rk_V + (size_t)node * (C * C));
  const int64_t per = (rows + gridDim.x - 1) / gridDim.x;
  const int64_t rlo = (int64_t)blockIdx.x * per, rhi = min(rows, rlo + per);
  Stager<DIFF, C> stg;
  if (rlo < rhi) stg.fetch(x, h, rlo, rhi);
  for (int64_t r0 = rlo; r0 < rhi; r0 += kRankRows) {
    __syncthreads();
    stg.store(L.tile);
    __syncthreads();
    // (the next chunk's rows of h are other addresses than the ones written below)
    if (r0 + kRankRows < rhi) stg.fetch(x, h, r0 + kRankRows, rhi);
    L.project(w, l);
    d4 out[C / 16];
    L.expand(w, l, K, out);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int64_t rr = r0 + 16 * w + (l >> 4) + 4 * v;
      if (rr < rhi) {
        float hv[C / 16];
#pragma unroll
        for (int cb = 0; cb < C / 16; ++cb) hv[cb] = h[rr * C + cb * 16 + (l & 15)];
#pragma unroll
        for (int cb = 0; cb < C / 16; ++cb) {
          const int64_t g = rr * C + cb * 16 + (l & 15);
          const float c32 = (float)out[cb][v];
          dense[g] = c32;
          h[g] = hv[cb] + c32;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
// Launch with `lds` bytes of dynamic LDS; sizes above 64 KB are announced to the runtime first (for the
// current device: a host-side setting, no allocation).
template <typename Kern>
static hipError_t launch_lds(Kern kern, size_t lds, dim3 grid, hipStream_t st, const NodeSet& ns, const PassArgs& a) {
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, grid, dim3(kBlock), lds, st, ns, a);
  return hipGetLastError();
}

template <int C>
static hipError_t launch_rank_c(int which, const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  const dim3 grid(ns.GR, ns.nn), block(kBlock);
  const size_t lds = ProjLds<C>::bytes(proj_columns(ns.lv, -1));      // (the apply kernel needs at most this)
  switch (which) {
    case 0:
      if (a.diff) hipLaunchKernelGGL((k_gram<true, C>), grid, block, 0, st, ns, a);
      else hipLaunchKernelGGL((k_gram<false, C>), grid, block, 0, st, ns, a);
      break;
    case 1:
      hipLaunchKernelGGL((k_eig<C>), dim3(ns.nn), dim3(eig_threads<C>()), 0, st, ns);
      break;
    case 2:
      if (a.diff) return launch_lds(k_rank_err<true, C>, lds, grid, st, ns, a);
      return launch_lds(k_rank_err<false, C>, lds, grid, st, ns, a);
    default:
      if (a.diff) return launch_lds(k_rank_apply<true, C>, lds, grid, st, ns, a);
      return launch_lds(k_rank_apply<false, C>, lds, grid, st, ns, a);
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

// Gram matrix, its eigen-decomposition and the realised error of every Rank-K level, in this order (before the
// level choice)
hipError_t launch_rank_gram(const NodeSet& ns, const PassArgs& a, hipStream_t st) { return launch_rank(0, ns, a, st); }
hipError_t launch_rank_eig(const NodeSet& ns, const PassArgs& a, hipStream_t st) { return launch_rank(1, ns, a, st); }
hipError_t launch_rank_errors(const NodeSet& ns, const PassArgs& a, hipStream_t st) { return launch_rank(2, ns, a, st); }

// Estimator update and dense message of the nodes whose chosen level is a Rank-K level
hipError_t launch_rank_apply(const NodeSet& ns, const PassArgs& a, hipStream_t st) { return launch_rank(3, ns, a, st); }

}  // namespace adacgd
