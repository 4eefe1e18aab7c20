// Worker / master compression step of AdaCGD (Section 4.3) for a set of nodes:
// multi-level exact Top-K selection by radix select on the magnitude key, the
// realised error of every level (left side of the trigger, Eq. (10)), the level
// cascade of the AdaCGD definition, and the EF21 update h <- h + C_j(x - h) (Eq. (7))
// with the sparse message.
//
// Every vector is cut into groups of 2048 consecutive coordinates (one wavefront's share of
// an 8192-coordinate tile).  The candidates of group g -- the coordinates that can belong to
// the largest Top-K set -- are stored at the fixed offset g * 2048 of the node's candidate
// list, in coordinate order, so all later stages keep that order without sorting.
//
// Kernel sequences per node set.  Kernels that need a reduction over the node end with a
// "last block of the node" epilogue (an arrival counter; nobody waits), so the small serial
// parts need no extra launches.
//
// One-pass sequence (Top-K levels only, long vectors):
//   sample  : one block per node histograms a sample of the vector and derives a
//             conservative candidate cut (a key) for the largest Top-K size
//   scanx   : v = x - h, S = ||v||^2, D = ||x - y||^2, candidates with key >= cut (staged in
//             LDS, written out when the block has finished its tiles), their first-digit
//             histogram and count, the energy below the cut
//             epilogue: first digit (bin) and in-bin rank of each Top-K size; marks the node
//             for repair if fewer candidates than the largest K were found, and as skipping
//             if the first trigger holds, S <= zeta D in the AdaCGD definition (then every
//             later kernel returns at once for that node)
//   scanx (repair variant): idle unless a node is marked; then it redoes the node with the
//             cut at zero (every coordinate a candidate)
// Two-pass sequence (level sets with quantisers, short vectors):
//   scan    : v, S, D, full first-digit histogram, max |v|
//             epilogue: bin and in-bin rank of each Top-K size, candidate cut-off bin, skip mark
//   filter  : re-forms v, candidates = keys in bins >= cut-off, energy below, realised
//             error of every quantiser level (Philox dither)
// Then, both sequences:
//   gather  : keys of the candidates inside some Top-K size's bin -> one list per node
//   select  : one block per (Top-K size, node) finishes the radix select on that list:
//             exact threshold key T_s, ties to take r_s, count of keys equal to T_s
//   tally   : per group counts of keys > T_s and == T_s, energy strictly below T_s
//             epilogue: err of every level, the cascade, message layout per block
//   compact : writes the chosen level's message in ascending coordinate and updates h
//   qapply  : dense update and codes for nodes whose chosen level is a quantiser
// Short vectors (d <= 4096): k_small, one block per node, does all of the above in one launch and,
// when asked, the server aggregation (its last block) and the next iterate update.
//
// What one block leaves for another block of the same launch (partial sums, its largest key, its
// candidate count, histogram counts) goes through agent-scope atomic accesses on distinct
// addresses.  Read-modify-writes by many blocks on one address are served one after the other, so
// only two things are accumulated that way: the first-digit histogram (spread over 4096 bins) and
// the gather cursor (one reservation per block).
#include <type_traits>

#include "devutil.h"
#include "engine.h"

namespace adacgd {

// ---------------------------------------------------------------------------
// element mapping of a tile: wavefront w owns coordinates [w*2048, (w+1)*2048) of the
// tile.  Vector path (d % 4 == 0): iteration k, lane l holds 4 consecutive coordinates
// starting at w*2048 + k*256 + 4l.  Scalar path: component c of iteration k is
// coordinate w*2048 + k*256 + 64c + l.
// ---------------------------------------------------------------------------
// Right side of the trigger that guards cascade position j (0 = keep h, j = level j):
// zeta_j ||x-y||^2 + eta_j ||x-h||^2.  Both products and the sum are rounded separately (no fused
// multiply-add), so the bound is the same number wherever it is evaluated; with eta_j = 0 it is
// exactly zeta_j ||x-y||^2, the trigger of Eq. (10).
__device__ __forceinline__ double trigger_bound(const LevelTable& lv, int j, double S, double D) {
  return __dadd_rn(__dmul_rn(lv.tz[j], D), __dmul_rn(lv.te[j], S));
}

template <bool VEC>
__device__ __forceinline__ int64_t comp0(int64_t base, int w, int lane, int k) {
  return VEC ? base + w * kWaveTile + k * 256 + lane * 4 : base + w * kWaveTile + k * 256 + lane;
}
template <bool VEC>
__device__ __forceinline__ int64_t comp_index(int64_t l0, int c) {
  return VEC ? l0 + c : l0 + 64 * c;
}
// The vectors are streamed once per pass: non-temporal loads keep them from displacing the
// candidate lists and histograms in L2 (measured: 8-10 % faster scans).
typedef float vfloat4 __attribute__((ext_vector_type(4)));
template <bool VEC>
__device__ __forceinline__ void load4(const float* __restrict__ p, int64_t l0, int64_t d, float (&o)[4]) {
  if (VEC) {
    if (l0 < d) {
      const vfloat4 q = __builtin_nontemporal_load(reinterpret_cast<const vfloat4*>(p + l0));
      o[0] = q.x; o[1] = q.y; o[2] = q.z; o[3] = q.w;
    } else {
      o[0] = o[1] = o[2] = o[3] = 0.f;
    }
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) o[c] = (l0 + 64 * c < d) ? __builtin_nontemporal_load(p + l0 + 64 * c) : 0.f;
  }
}
template <bool VEC>
__device__ __forceinline__ void store4(float* __restrict__ p, int64_t l0, int64_t d, const float (&o)[4]) {
  if (VEC) {
    if (l0 < d) *reinterpret_cast<float4*>(p + l0) = make_float4(o[0], o[1], o[2], o[3]);
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (l0 + 64 * c < d) p[l0 + 64 * c] = o[c];
  }
}

// Walks a histogram of this launch from its top bin down and finds, for each of nr
// ranks, the bin where the running count reaches the rank.  Zeroes the histogram.
__device__ __forceinline__ uint32_t hist0_slot(uint32_t bin) { return ((bin & 31u) << 7) | (bin >> 5); }
template <int NB>
__device__ void locate(uint32_t* hist, int nr, const uint32_t* rank, uint32_t* out_bin, uint32_t* out_rank,
                       uint32_t* out_cnt, uint32_t* lds4) {
  constexpr int PER = NB / kBlock;
  uint32_t loc[PER];
  uint32_t sum = 0;
  const int top = NB - 1 - (int)threadIdx.x * PER;
#pragma unroll
  for (int q = 0; q < PER; ++q) loc[q] = ld_coherent(&hist[hist0_slot((uint32_t)(top - q))]);
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    hist[hist0_slot((uint32_t)(top - q))] = 0;
    sum += loc[q];
  }
  uint32_t total;
  uint32_t cum = block_excl_scan(sum, lds4, &total);
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const uint32_t c = loc[q];
    if (c) {
      for (int r = 0; r < nr; ++r) {
        const uint32_t rk = rank[r];
        if (cum < rk && rk <= cum + c) {
          out_bin[r] = (uint32_t)(top - q);
          out_rank[r] = rk - cum;
          out_cnt[r] = c;
        }
      }
    }
    cum += c;
  }
  __syncthreads();
}

// Entry e of group g's candidate slot sits at position (e + group_rot(g)) mod 2048 of the
// slot.  Typical groups fill only the first few hundred entries; without the rotation those
// writes would all fall on the same few address bits (slot stride 8 KB) and so on a fraction of
// the memory channels.  Rotations are multiples of 64 entries, so 64-entry chunks stay
// contiguous.  A trailing partial group is not rotated (its slot is shorter than 2048).
__device__ __forceinline__ uint32_t group_rot(int g, int64_t d) {
  if (((int64_t)g + 1) * kWaveTile > d) return 0u;
  return (((uint32_t)g * 2654435761u) >> 21) & (uint32_t)(kWaveTile - 64);
}

// ---------------------------------------------------------------------------
// ordered extraction: the wavefront appends the flagged components of one iteration (4 per
// lane, flag bit c <-> component c) to its group's slot of the candidate list, keeping
// coordinate order.  A candidate is stored as its value bits (sval) and, in a separate array,
// its 11-bit offset inside the group (soff); o0 is the offset of the lane's component 0.
// `running` is the number of candidates the group holds so far.  Must be called by all 64 lanes.
// ---------------------------------------------------------------------------
template <bool VEC>
__device__ __forceinline__ void emit4(uint32_t f, const float (&vv)[4], uint32_t o0, uint32_t* __restrict__ sval,
                                      uint16_t* __restrict__ soff, uint32_t rot, uint32_t& running) {
  if (VEC) {      // order: lane, then component
    const uint64_t b0 = ballot(f & 1u), b1 = ballot(f & 2u), b2 = ballot(f & 4u), b3 = ballot(f & 8u);
    if ((b0 | b1 | b2 | b3) != 0) {
      uint32_t pos = running + below(b0) + below(b1) + below(b2) + below(b3);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if ((f >> c) & 1u) {
          const uint32_t at = (pos + rot) & (uint32_t)(kWaveTile - 1);
          sval[at] = fbits(vv[c]);
          soff[at] = (uint16_t)(o0 + c);
          ++pos;
        }
      running += popc64(b0) + popc64(b1) + popc64(b2) + popc64(b3);
    }
  } else {        // order: component, then lane
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool fc = (f >> c) & 1u;
      const uint64_t b = ballot(fc);
      if (fc) {
        const uint32_t at = (running + below(b) + rot) & (uint32_t)(kWaveTile - 1);
        sval[at] = fbits(vv[c]);
        soff[at] = (uint16_t)(o0 + 64 * c);
      }
      running += popc64(b);
    }
  }
}

// ---------------------------------------------------------------------------
// scan
// ---------------------------------------------------------------------------
template <bool DIFF, bool VEC>
__global__ __launch_bounds__(kBlock) void k_scan(NodeSet ns, PassArgs a) {
  __shared__ uint32_t hist[kBins0];
  __shared__ double red[4];
  __shared__ uint32_t lds4[4];
  __shared__ int s_flag;
  __shared__ uint32_t s_rank[kMaxLevels], s_bin[kMaxLevels], s_rk[kMaxLevels], s_cnt[kMaxLevels];
  __shared__ uint32_t s_kmax;

  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int64_t d = ns.d;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  const float* __restrict__ h = a.h + row;
  const float* __restrict__ y = DIFF ? nullptr : a.y + row;
  float* __restrict__ yc = a.ycopy ? a.ycopy + row : nullptr;

  for (int b = tid; b < kBins0; b += kBlock) hist[b] = 0;
  __syncthreads();

  // block-wise quantiser levels: the largest key of every 64-coordinate segment (a block's scale is the
  // maximum over its segments, so the result does not depend on how the blocks fall on the wavefronts)
  uint32_t* __restrict__ segm = ns.segmax ? ns.segmax + (size_t)node * ns.nseg : nullptr;
  double S = 0.0, D = 0.0;
  uint32_t kmax = 0;
  for (int t = blockIdx.x; t < ns.tiles; t += gridDim.x) {
    const int64_t base = (int64_t)t * kTile;
#pragma unroll
    for (int k = 0; k < kIter; ++k) {
      const int64_t l0 = comp0<VEC>(base, w, lane, k);
      float xv[4], hv[4], yv[4];
      load4<VEC>(x, l0, d, xv);
      if (!DIFF) {
        load4<VEC>(h, l0, d, hv);
        load4<VEC>(y, l0, d, yv);
        if (yc) store4<VEC>(yc, l0, d, xv);
      }
      uint32_t kc[4] = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (comp_index<VEC>(l0, c) < d) {
          const float v = DIFF ? xv[c] : xv[c] - hv[c];
          const double dv = (double)v;
          S = fma(dv, dv, S);
          if (!DIFF) {
            const double dw = (double)(xv[c] - yv[c]);
            D = fma(dw, dw, D);
          }
          const uint32_t key = magkey(v);
          kc[c] = key;
          kmax = key > kmax ? key : kmax;
          hist_add(hist, key >> kShift0);
        }
      }
      if (segm) {
        if (VEC) {        // 16 lanes x 4 consecutive coordinates = one segment
          uint32_t m = max(max(kc[0], kc[1]), max(kc[2], kc[3]));
#pragma unroll
          for (int o = 1; o < 16; o <<= 1) m = max(m, (uint32_t)__shfl_xor(m, o, 64));
          if ((lane & 15) == 0 && l0 < d) segm[l0 >> 6] = m;
        } else {          // component c over the 64 lanes = one segment
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t m = wave_max(kc[c]);
            const int64_t start = l0 - lane + 64 * c;
            if (lane == 0 && start < d) segm[start >> 6] = m;
          }
        }
      }
    }
  }
  S = block_sum(S, red);
  D = block_sum(D, red);
  if (tid == 0) {
    st_coherent(&ns.partS[(size_t)node * ns.G + blockIdx.x], S);
    st_coherent(&ns.partD[(size_t)node * ns.G + blockIdx.x], D);
  }
  if (ns.lv.nq > 0) {       // the block's largest key, as one more partial result (no shared counter)
    kmax = wave_max(kmax);
    if (lane == 0) lds4[w] = kmax;
    __syncthreads();
    if (tid == 0) {
      const uint32_t a01 = lds4[0] > lds4[1] ? lds4[0] : lds4[1], a23 = lds4[2] > lds4[3] ? lds4[2] : lds4[3];
      st_coherent(&ns.partU[(size_t)node * ns.G + blockIdx.x], a01 > a23 ? a01 : a23);
    }
  }
  __syncthreads();
  uint32_t* gh = ns.hist0 + (size_t)node * kBins0;
  for (int b = tid; b < kBins0; b += kBlock) {
    const uint32_t c = hist[b];
    if (c) atomicAdd(&gh[hist0_slot((uint32_t)b)], c);
  }

  if (!arrive_last(&ns.done[(size_t)node * (kArriveFan + 1) * kCounterStride], gridDim.x, blockIdx.x, &s_flag)) return;

  // ---- epilogue: one block per node ----
  const int p = ns.lv.p;
  double s = 0.0, dd = 0.0;
  for (int b = tid; b < (int)gridDim.x; b += kBlock) {
    s += ld_coherent(&ns.partS[(size_t)node * ns.G + b]);
    dd += ld_coherent(&ns.partD[(size_t)node * ns.G + b]);
  }
  s = block_sum(s, red);
  dd = block_sum(dd, red);
  if (ns.lv.nq > 0) {
    uint32_t km = 0;
    for (int b = tid; b < (int)gridDim.x; b += kBlock) {
      const uint32_t v = ld_coherent(&ns.partU[(size_t)node * ns.G + b]);
      km = v > km ? v : km;
    }
    km = wave_max(km);
    __syncthreads();
    if (lane == 0) lds4[w] = km;
    __syncthreads();
    if (tid == 0) {
      const uint32_t a01 = lds4[0] > lds4[1] ? lds4[0] : lds4[1], a23 = lds4[2] > lds4[3] ? lds4[2] : lds4[3];
      s_kmax = a01 > a23 ? a01 : a23;
    }
  }
  if (tid < kMaxLevels) {
    s_rank[tid] = tid < p ? ns.lv.K[tid] : 0;
    s_bin[tid] = 0; s_rk[tid] = 1; s_cnt[tid] = 0;
  }
  __syncthreads();
  locate<kBins0>(gh, p, s_rank, s_bin, s_rk, s_cnt, lds4);
  if (tid < p) {
    ns.prefix[node * p + tid] = s_bin[tid];
    ns.rank[node * p + tid] = s_rk[tid];
  }
  if (tid == 0) {
    ns.S[node] = s;
    const double dnode = DIFF ? a.extD[node] : dd;
    ns.D[node] = dnode;
    // first condition of the cascade: the trigger keeps h, and nothing after this kernel has work
    // to do for the node (the tally kernel takes the same decision from the same two numbers)
    // (the compressed start applies its one level unconditionally: a zero gradient still selects K zeros, signs kept)
    ns.skip[node] = (!a.assign && s <= trigger_bound(ns.lv, 0, s, dnode)) ? 1u : 0u;
    ns.bmin[node] = p > 0 ? s_bin[p - 1] : (uint32_t)kBins0;   // largest K reaches lowest
    if (ns.lv.nq > 0) ns.amax[node] = s_kmax;
  }
}

// ---------------------------------------------------------------------------
// sample: one block per node histograms (top 13 key bits) a sample of R = min(tiles, 256)
// rows of 256 consecutive coordinates, one row from each of R evenly spaced tiles (row = hash
// of the tile index), each row read by one wavefront as a single 16-byte load per lane.
// Result: the candidate cut = the key at the sample's rank ceil(m K/d) + 6 sqrt(m K/d) + 8 from
// the top (interpolated inside the histogram bin that holds that rank), K the largest Top-K size
// and m the sample size, so that with overwhelming probability at least K coordinates of the
// full vector have keys >= cut.  scanx counts them and the repair passes cover a miss.
// ---------------------------------------------------------------------------
constexpr int kSampleShift = 18, kSampleBins = 8192, kSampleBlock = 1024, kSampleRows = 256;
__device__ __forceinline__ int sample_row(int t) { return (int)(((uint32_t)t * 2654435761u) >> 27); }

template <bool DIFF>
__global__ __launch_bounds__(kSampleBlock) void k_sample(NodeSet ns, PassArgs a) {
  __shared__ uint32_t hist[kSampleBins];
  __shared__ uint32_t wsum16[16];
  __shared__ uint32_t res[3];
  const int node = blockIdx.x, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int64_t d = ns.d;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  const float* __restrict__ h = a.h + row;
  for (int b = tid; b < kSampleBins; b += kSampleBlock) hist[b] = 0;
  if (tid < 3) res[tid] = tid == 1 ? 1u : 0u;
  __syncthreads();
  const int R = ns.tiles < kSampleRows ? ns.tiles : kSampleRows;
  constexpr int U = kSampleRows / 16;        // rows per wavefront
  constexpr int UB = U / 2;                  // ... read in two batches of UB rows, each batch in flight at once
  uint32_t mine = 0;
  for (int b = 0; b < 2; ++b) {
    float4 xv[UB], hv[UB];
    bool ok[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int r = w * U + b * UB + u;
      const int t = (int)(((int64_t)r * ns.tiles) / R);          // evenly spaced tiles
      const int64_t l0 = (int64_t)t * kTile + sample_row(t) * 256 + lane * 4;
      ok[u] = r < R && l0 < d;
      xv[u] = hv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (ok[u]) {
        xv[u] = *reinterpret_cast<const float4*>(x + l0);
        if (!DIFF) hv[u] = *reinterpret_cast<const float4*>(h + l0);
      }
    }
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      if (ok[u]) {
        hist_add(hist, magkey(xv[u].x - hv[u].x) >> kSampleShift);
        hist_add(hist, magkey(xv[u].y - hv[u].y) >> kSampleShift);
        hist_add(hist, magkey(xv[u].z - hv[u].z) >> kSampleShift);
        hist_add(hist, magkey(xv[u].w - hv[u].w) >> kSampleShift);
        mine += 4;
      }
    }
  }
  // sample size m
  mine = wave_sum(mine);
  __syncthreads();
  if (lane == 0) wsum16[w] = mine;
  __syncthreads();
  uint32_t m = 0;
  for (int i = 0; i < 16; ++i) m += wsum16[i];
  const double mq = (double)m * (double)ns.lv.K[ns.lv.p - 1] / (double)d;
  double rk = ceil(mq) + 6.0 * sqrt(mq) + 8.0;
  if (rk > (double)m) rk = (double)m;
  const uint32_t rank = (uint32_t)rk;
  // walk the histogram from the top: thread t owns bins [top - 8 t - 7, top - 8 t]
  constexpr int PER = kSampleBins / kSampleBlock;
  uint32_t loc[PER], sum = 0;
  const int top = kSampleBins - 1 - tid * PER;
#pragma unroll
  for (int q = 0; q < PER; ++q) { loc[q] = hist[top - q]; sum += loc[q]; }
  uint32_t inc = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) wsum16[w] = inc;
  __syncthreads();
  uint32_t cum = inc - sum;
  for (int i = 0; i < w; ++i) cum += wsum16[i];
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    if (loc[q] && cum < rank && rank <= cum + loc[q]) {
      // The rank falls inside this bin, `need` of its `loc` samples from the top.  The cut is placed
      // at that fraction of the bin's key range (samples taken as evenly spread inside one bin, whose
      // width is 3 % of the value), rounded down.  It only has to be good, not safe: scanx counts the
      // candidates and the repair pass covers a cut that turns out too high.
      const uint32_t need = rank - cum;
      const uint32_t span = 1u << kSampleShift;
      const uint32_t down = (uint32_t)(((uint64_t)span * need) / loc[q]);       // <= span
      res[0] = (((uint32_t)(top - q) + 1u) << kSampleShift) - down;
    }
    cum += loc[q];
  }
  __syncthreads();
  if (tid == 0) ns.best[node] = res[0];
}

// ---------------------------------------------------------------------------
// scanx: scan fused with the candidate extraction at the estimated cut-off bin
// (16-byte vector path only)
// ---------------------------------------------------------------------------
// REPAIR: second attempt, only for nodes marked in ns.redo (the sampled cut left fewer
// candidates than the largest K): the same pass with the cut at zero, i.e. every coordinate
// becomes a candidate and the histogram is the full one.
template <bool DIFF, bool REPAIR>
__global__ __launch_bounds__(kBlock) void k_scanx(NodeSet ns, PassArgs a) {
  constexpr bool VEC = true;
  __shared__ uint32_t hist[kBins0];
  __shared__ double red[4];
  __shared__ uint32_t lds4[4];
  __shared__ int s_flag;
  __shared__ uint32_t s_rank[kMaxLevels], s_bin[kMaxLevels], s_rk[kMaxLevels], s_cnt[kMaxLevels];
  // Candidates are staged in LDS per wavefront and written to memory when the block has finished
  // its tiles (earlier only if the stage fills up): a store issued between the loads makes the
  // next wait for a load wait for everything outstanding, which drains the wavefront's pipeline.
  constexpr int kStage = 768;            // staged candidates per wavefront (an iteration adds at most 256)
  constexpr int kSeg = 8;                // ... belonging to at most kSeg groups
  __shared__ uint32_t st_val[4][kStage];
  __shared__ uint16_t st_off[4][kStage];
  __shared__ uint32_t sg_grp[4][kSeg], sg_end[4][kSeg], sg_base[4][kSeg];

  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  if (REPAIR && (ns.redo[node] == 0 || ns.skip[node] != 0)) return;
  const int64_t d = ns.d;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  const float* __restrict__ h = a.h + row;
  const float* __restrict__ y = DIFF ? nullptr : a.y + row;
  float* __restrict__ yc = (a.ycopy && !REPAIR) ? a.ycopy + row : nullptr;
  uint32_t* __restrict__ cval = ns.cand_val + row;
  uint16_t* __restrict__ coff = ns.cand_off + row;
  const uint32_t cut = REPAIR ? 0u : ns.best[node];

  for (int b = tid; b < kBins0; b += kBlock) hist[b] = 0;
  __syncthreads();

  double S = 0.0, D = 0.0, El = 0.0;
  uint32_t ncand = 0;
  // stage bookkeeping (all values are the same in every lane of the wavefront; every lane writes
  // and reads the segment table itself, so no lane depends on another's LDS write)
  uint32_t held = 0;        // entries in the stage
  uint32_t nseg = 0;        // closed segments: group sg_grp, entries [previous end, sg_end), first entry
                            // is the group's entry number sg_base
  uint32_t open_base = 0;   // entries of the open group that were written out already
  uint32_t open_begin = 0;  // stage index where the open group's entries start
  // writes segments [0, nseg) and, if `open_grp` >= 0, the open group's staged entries
  auto flush = [&](int open_grp) {
    uint32_t begin = 0;
    const uint32_t total = nseg + (open_grp >= 0 ? 1u : 0u);
    for (uint32_t sgi = 0; sgi < total; ++sgi) {
      const bool closed = sgi < nseg;
      const uint32_t grp = closed ? sg_grp[w][sgi] : (uint32_t)open_grp;
      const uint32_t end = closed ? sg_end[w][sgi] : held;
      const uint32_t gbase = closed ? sg_base[w][sgi] : open_base;
      uint32_t* __restrict__ sval = cval + (size_t)grp * kWaveTile;
      uint16_t* __restrict__ soff = coff + (size_t)grp * kWaveTile;
      const uint32_t rot = group_rot((int)grp, d);
      for (uint32_t e = begin + lane; e < end; e += 64) {
        const uint32_t at = (gbase + (e - begin) + rot) & (uint32_t)(kWaveTile - 1);
        __builtin_nontemporal_store(st_val[w][e], &sval[at]);
        __builtin_nontemporal_store(st_off[w][e], &soff[at]);
      }
      if (closed && lane == 0 && (int)grp < ns.groups) ns.grp_count[(size_t)node * ns.groups + grp] = gbase + (end - begin);
      if (!closed) open_base = gbase + (end - begin);
      begin = end;
    }
    nseg = 0;
    held = 0;
    open_begin = 0;
  };
  for (int t = blockIdx.x; t < ns.tiles; t += gridDim.x) {
    const int64_t base = (int64_t)t * kTile;
    const int grp = t * 4 + w;
    open_base = 0;
    open_begin = held;
#pragma unroll
    for (int k = 0; k < kIter; ++k) {
      const int64_t l0 = comp0<VEC>(base, w, lane, k);
      float xv[4], hv[4], yv[4], vv[4];
      load4<VEC>(x, l0, d, xv);
      if (!DIFF) {
        load4<VEC>(h, l0, d, hv);
        load4<VEC>(y, l0, d, yv);
        if (yc) store4<VEC>(yc, l0, d, xv);
      }
      uint32_t f = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        vv[c] = DIFF ? xv[c] : xv[c] - hv[c];
        if (l0 < d) {
          const double dv = (double)vv[c];
          const double e = dv * dv;
          S += e;
          if (!DIFF) {
            const double dw = (double)(xv[c] - yv[c]);
            D = fma(dw, dw, D);
          }
          const uint32_t key = magkey(vv[c]);
          if (key >= cut) {
            f |= 1u << c;
            atomicAdd(&hist[key >> kShift0], 1u);     // every threshold lies among the candidates
          } else {
            El += e;
          }
        }
      }
      if (held > (uint32_t)(kStage - 256)) flush(grp);         // rare: dense groups
      emit4<VEC>(f, vv, (uint32_t)(l0 - base) - (uint32_t)w * kWaveTile, st_val[w], st_off[w], 0u, held);
    }
    // close the group's segment
    sg_grp[w][nseg] = (uint32_t)grp;
    sg_end[w][nseg] = held;
    sg_base[w][nseg] = open_base;
    ncand += open_base + (held - open_begin);
    ++nseg;
    if (nseg == (uint32_t)kSeg) flush(-1);
  }
  flush(-1);
  S = block_sum(S, red);
  D = block_sum(D, red);
  El = block_sum(El, red);
  ncand = __builtin_amdgcn_readfirstlane(ncand);      // (the same in every lane of a wavefront)
  __syncthreads();
  if (lane == 0) lds4[w] = ncand;
  __syncthreads();
  if (tid == 0) {
    st_coherent(&ns.partU[(size_t)node * ns.G + blockIdx.x], (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]));
    st_coherent(&ns.partS[(size_t)node * ns.G + blockIdx.x], S);
    st_coherent(&ns.partD[(size_t)node * ns.G + blockIdx.x], D);
    st_coherent(&ns.partEb[(size_t)node * ns.G + blockIdx.x], El);
  }
  __syncthreads();
  uint32_t* gh = ns.hist0 + (size_t)node * kBins0;
  for (int b = tid; b < kBins0; b += kBlock) {
    const uint32_t c = hist[b];
    if (c) atomicAdd(&gh[hist0_slot((uint32_t)b)], c);
  }

  if (!arrive_last(&ns.done[(size_t)node * (kArriveFan + 1) * kCounterStride], gridDim.x, blockIdx.x, &s_flag)) return;

  const int p = ns.lv.p;
  double s = 0.0, dd = 0.0, el = 0.0;
  uint32_t found = 0;
  for (int b = tid; b < (int)gridDim.x; b += kBlock) {
    s += ld_coherent(&ns.partS[(size_t)node * ns.G + b]);
    dd += ld_coherent(&ns.partD[(size_t)node * ns.G + b]);
    el += ld_coherent(&ns.partEb[(size_t)node * ns.G + b]);
    found += ld_coherent(&ns.partU[(size_t)node * ns.G + b]);
  }
  s = block_sum(s, red);
  dd = block_sum(dd, red);
  el = block_sum(el, red);
  found = wave_sum(found);
  __syncthreads();
  if (lane == 0) lds4[w] = found;
  __syncthreads();
  found = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
  if (tid < kMaxLevels) {
    s_rank[tid] = tid < p ? ns.lv.K[tid] : 0;
    s_bin[tid] = 0; s_rk[tid] = 1; s_cnt[tid] = 0;
  }
  __syncthreads();
  locate<kBins0>(gh, p, s_rank, s_bin, s_rk, s_cnt, lds4);
  if (tid < p) {
    ns.prefix[node * p + tid] = s_bin[tid];
    ns.rank[node * p + tid] = s_rk[tid];
  }
  if (tid == 0) {
    ns.S[node] = s;
    const double dnode = DIFF ? a.extD[node] : dd;
    ns.D[node] = dnode;
    // first condition of the cascade: the trigger keeps h, and nothing after this kernel has work
    // to do for the node (the tally kernel takes the same decision from the same two numbers)
    const bool skip = !a.assign && s <= trigger_bound(ns.lv, 0, s, dnode);       // (see the two-pass scan)
    ns.skip[node] = skip ? 1u : 0u;
    ns.Eb[node] = el;
    // the K largest all have keys >= cut  <=>  at least K candidates were found
    const uint32_t total = found;
    const bool redo = total < ns.lv.K[p - 1];           // estimate too high: the repair pass runs
    ns.redo[node] = redo ? 1u : 0u;
    if (redo && !skip) atomicAdd(ns.repairs, 1ull);
  }
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1) -> 4 words
// ---------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c0 = n0; c1 = (uint32_t)p1; c2 = n2; c3 = (uint32_t)p0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// dither u in [0,1) of coordinate l: word l%4 of the block l/4, top 24 bits
__device__ __forceinline__ float dither_of(uint32_t word) { return (float)(word >> 8) * 5.9604644775390625e-8f; }

// b-bit stochastic quantiser of one coordinate from t = fl(|v| / a): the magnitude code xi (as a float) and
// the decoded magnitude fl(xi c).  s = magnitude levels, c = fl(a / (s (1+omega))).
__device__ __forceinline__ float quant_mag(float t, float s, float c, float u, float* xi_out) {
  const float r = t * s;              // the second of the two rounded fp32 operations
  const float fl = floorf(r);
  const float pfrac = r - fl;
  const float xi = fl + ((u < pfrac) ? 1.f : 0.f);
  *xi_out = xi;
  return xi * c;
}

// ... with the sign of v: returns the signed code and the decoded value.
__device__ __forceinline__ float quant_ratio(float v, float t, float s, float c, float u, int* code) {
  float xi;
  const float mag = quant_mag(t, s, c, u, &xi);
  *code = (__float_as_uint(v) >> 31) ? -(int)xi : (int)xi;
  return copysignf(mag, v);
}

// The same with a = max |v| (> 0) given.
__device__ __forceinline__ float quant_one(float v, float a, float s, float c, float u, int* code) {
  return quant_ratio(v, fabsf(v) / a, s, c, u, code);
}

// Block-wise quantiser scales of one group of 2048 coordinates (one wavefront's share of a tile).
// Lane j < 32 loads the largest key of the group's segment j; a block of B coordinates is B/64
// neighbouring segments (blocks are aligned: B and the group length are powers of two), so its largest
// key is a maximum over B/64 neighbouring lanes.  On return lane j holds, for the block that contains
// segment j, the scale a (as a key) and c = fl(a / (s (1 + omega_B))).  Called by all 64 lanes.
__device__ __forceinline__ void block_scales(const uint32_t* __restrict__ segm, int nseg, int grp, int B, double qdenom,
                                             uint32_t lane, uint32_t* akey, float* c) {
  const int64_t seg = (int64_t)grp * kSegPerGroup + lane;
  uint32_t m = (lane < (uint32_t)kSegPerGroup && seg < nseg) ? segm[seg] : 0u;
  for (int o = 1; o < B / kSeg; o <<= 1) m = max(m, (uint32_t)__shfl_xor(m, o, 64));
  const float a = __uint_as_float(m);
  *akey = m;
  *c = a > 0.f ? (float)((double)a / qdenom) : 0.f;
}

// ---------------------------------------------------------------------------
// filter
// ---------------------------------------------------------------------------
// NQ: 0 = no quantiser level; 1..3 = exactly that many (the loops over them carry no run-time test);
// kMaxLevels = any number.  BLK: some of them are block-wise (their scales come from the segment maxima).
template <bool DIFF, bool VEC, int NQ, bool BLK>
__global__ __launch_bounds__(kBlock) void k_filter(NodeSet ns, PassArgs a) {
  constexpr bool QUANT = NQ > 0;
  constexpr bool EXACT = NQ < kMaxLevels;          // ns.lv.nq == NQ
  constexpr int NQA = NQ > 0 ? NQ : 1;
  __shared__ double red[4];
  __shared__ int s_flag;

  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  if (ns.skip[node] != 0) return;   // skipping nodes need no candidates
  const int64_t d = ns.d;
  const int nq = ns.lv.nq;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  const float* __restrict__ h = a.h + row;
  uint32_t* __restrict__ cval = ns.cand_val + row;
  uint16_t* __restrict__ coff = ns.cand_off + row;

  const uint32_t bmin = ns.bmin[node];

  // quantiser constants of this node
  float qa = 0.f;
  float qc[NQA];
  double qacc[NQA];
  if (QUANT) {
    qa = __uint_as_float(ns.amax[node]);
#pragma unroll
    for (int q = 0; q < NQA; ++q) {
      qc[q] = ((EXACT || q < nq) && qa > 0.f) ? (float)((double)qa / ns.lv.qdenom[q]) : 0.f;
      qacc[q] = 0.0;
    }
  }
  const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
  const uint32_t ctr1 = (uint32_t)node | a.node_flag;

  double Eb = 0.0;
  for (int t = blockIdx.x; t < ns.tiles; t += gridDim.x) {
    const int64_t base = (int64_t)t * kTile;
    const int grp = t * 4 + w;
    uint32_t* __restrict__ sval = cval + (size_t)grp * kWaveTile;
    uint16_t* __restrict__ soff = coff + (size_t)grp * kWaveTile;
    const uint32_t rot = group_rot(grp, d);
    uint32_t running = 0;
    uint32_t bkey[NQA];       // block-wise levels: per lane < 32, scale (as a key) and c of the block of segment `lane`
    float bcq[NQA];
    if (BLK) {
#pragma unroll
      for (int q = 0; q < NQA; ++q) {
        bkey[q] = 0u;
        bcq[q] = 0.f;
        if ((EXACT || q < nq) && ns.lv.qblock[q])
          block_scales(ns.segmax + (size_t)node * ns.nseg, ns.nseg, grp, ns.lv.qblock[q], ns.lv.qdenom[q], lane, &bkey[q], &bcq[q]);
      }
    }
#pragma unroll
    for (int k = 0; k < kIter; ++k) {
      const int64_t l0 = comp0<VEC>(base, w, lane, k);
      float xv[4], hv[4], vv[4];
      load4<VEC>(x, l0, d, xv);
      if (!DIFF) load4<VEC>(h, l0, d, hv);
      uint32_t rnd[4];
      if (QUANT && VEC) philox4x32_10((uint32_t)(l0 >> 2), ctr1, a.step, 0u, k0, k1, rnd);
      uint32_t f = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        vv[c] = DIFF ? xv[c] : xv[c] - hv[c];
        const int64_t l = comp_index<VEC>(l0, c);
        // scale and c of every quantiser level at this coordinate (all lanes take part in the shuffles)
        float qa_l[NQA], qc_l[NQA];
        if (QUANT) {
          const int sg = k * 4 + (VEC ? (int)(lane >> 4) : c);       // segment of the group this coordinate is in
#pragma unroll
          for (int q = 0; q < NQA; ++q) {
            qa_l[q] = qa;
            qc_l[q] = qc[q];
            if (BLK && (EXACT || q < nq) && ns.lv.qblock[q]) {
              qa_l[q] = __uint_as_float((uint32_t)__shfl(bkey[q], sg, 64));
              qc_l[q] = __shfl(bcq[q], sg, 64);
            }
          }
        }
        if (l < d) {
          const uint32_t key = magkey(vv[c]);
          const uint32_t bin = key >> kShift0;
          const double dv = (double)vv[c];
          if (bin >= bmin) {
            f |= 1u << c;
          } else {
            Eb = fma(dv, dv, Eb);
          }
          if (QUANT) {
            uint32_t word;
            if (VEC) {
              word = rnd[c];
            } else {
              uint32_t r4[4];
              philox4x32_10((uint32_t)(l >> 2), ctr1, a.step, 0u, k0, k1, r4);
              word = r4[l & 3];
            }
            const float u = dither_of(word);
            // |v| / a once for all levels that share the whole-vector scale (a division is a dozen
            // instructions, and the compiler does not merge the divisions of separately guarded levels)
            const float av = fabsf(vv[c]);
            const float tg = qa > 0.f ? av / qa : 0.f;
            float tb = 0.f;
#pragma unroll
            for (int q = 0; q < NQA; ++q) {
              if (EXACT || q < nq) {
                float xi, t = tg;
                if (BLK && ns.lv.qblock[q]) {
                  // (levels with the same block length share the scale, hence the quotient)
                  if (q == 0 || ns.lv.qblock[q] != ns.lv.qblock[q > 0 ? q - 1 : 0]) tb = qa_l[q] > 0.f ? av / qa_l[q] : 0.f;
                  t = tb;
                }
                // the error of a coordinate is | |v| - decoded magnitude |: the sign is common to both
                const float mag = qa_l[q] > 0.f ? quant_mag(t, ns.lv.qs[q], qc_l[q], u, &xi) : 0.f;
                const double e = (double)av - (double)mag;
                qacc[q] = fma(e, e, qacc[q]);
              }
            }
          }
        }
      }
      emit4<VEC>(f, vv, (uint32_t)(l0 - base) - (uint32_t)w * kWaveTile, sval, soff, rot, running);
    }
    if (lane == 0 && grp < ns.groups) ns.grp_count[(size_t)node * ns.groups + grp] = running;
  }

  Eb = block_sum(Eb, red);
  if (tid == 0) st_coherent(&ns.partEb[(size_t)node * ns.G + blockIdx.x], Eb);
  if (QUANT) {
#pragma unroll
    for (int q = 0; q < NQA; ++q) {
      if (EXACT || q < nq) {
        const double e = block_sum(qacc[q], red);
        if (tid == 0) st_coherent(&ns.partQ[((size_t)node * ns.G + blockIdx.x) * nq + q], e);
      }
    }
  }
  if (!arrive_last(&ns.done[(size_t)node * (kArriveFan + 1) * kCounterStride], gridDim.x, blockIdx.x, &s_flag)) return;

  // ---- epilogue ----
  double e = 0.0;
  for (int b = tid; b < (int)gridDim.x; b += kBlock) e += ld_coherent(&ns.partEb[(size_t)node * ns.G + b]);
  e = block_sum(e, red);
  if (tid == 0) ns.Eb[node] = e;
  if (QUANT) {
    for (int q = 0; q < nq; ++q) {
      double s = 0.0;
      for (int b = tid; b < (int)gridDim.x; b += kBlock)
        s += ld_coherent(&ns.partQ[((size_t)node * ns.G + b) * nq + q]);
      s = block_sum(s, red);
      if (tid == 0) ns.qerr[node * nq + q] = s;
    }
  }
}

// ---------------------------------------------------------------------------
// Reading the candidates of a group, in order, 64 at a time.  group_load issues the loads of
// the group's count and of its first 192 entries together, so that a typical group (one or two
// hundred candidates) costs one memory round trip.  group_visit then calls
// f(value bits, offset in group, valid) in all lanes for each 64 entries (offsets are read only
// when OFF).  Entries past the count are stale data inside the group's own slot, flagged invalid.
// ---------------------------------------------------------------------------
constexpr int kPre = 3;
struct GroupHead {
  uint32_t start, rot, cnt;
  uint32_t pv[kPre], po[kPre];
};

template <bool OFF>
__device__ __forceinline__ GroupHead group_load(const uint32_t* __restrict__ cval, const uint16_t* __restrict__ coff,
                                                const uint32_t* __restrict__ counts, int g, int64_t d, uint32_t lane) {
  GroupHead gh;
  gh.start = (uint32_t)g * kWaveTile;
  gh.rot = group_rot(g, d);
  const uint32_t slen = (uint32_t)min((int64_t)kWaveTile, d - (int64_t)gh.start);
  gh.cnt = counts[g];
#pragma unroll
  for (int j = 0; j < kPre; ++j) {      // unconditional loads (entries past a short slot read its first one)
    const uint32_t e = lane + 64 * j;
    const uint32_t at = gh.start + (e < slen ? ((e + gh.rot) & (uint32_t)(kWaveTile - 1)) : 0u);
    gh.pv[j] = cval[at];
    gh.po[j] = OFF ? (uint32_t)coff[at] : 0u;
  }
  return gh;
}

// Calls body(head, g) for g = g0, g0 + gstep, ... < gend with the loads of the following group
// already issued.  Two heads alternate so that no register copy (which would have to wait for
// the loads) sits between one group and the next, and the last group has a call site of its
// own so that no path merges with loads that may or may not have been issued.
template <bool OFF, typename Body>
__device__ __forceinline__ void for_groups(const uint32_t* __restrict__ cval, const uint16_t* __restrict__ coff,
                                           const uint32_t* __restrict__ counts, int g0, int gend, int gstep, int64_t d,
                                           uint32_t lane, Body&& body) {
  if (g0 >= gend) return;
  int g = g0;
  GroupHead a = group_load<OFF>(cval, coff, counts, g, d, lane);
  for (;;) {
    if (g + gstep >= gend) { body(a, g); break; }
    const GroupHead b = group_load<OFF>(cval, coff, counts, g + gstep, d, lane);
    body(a, g);
    g += gstep;
    if (g + gstep >= gend) { body(b, g); break; }
    a = group_load<OFF>(cval, coff, counts, g + gstep, d, lane);
    body(b, g);
    g += gstep;
  }
}

template <bool OFF, typename F>
__device__ __forceinline__ void group_visit(const GroupHead& gh, const uint32_t* __restrict__ cval,
                                            const uint16_t* __restrict__ coff, uint32_t lane, F&& f) {
#pragma unroll
  for (int j = 0; j < kPre; ++j) {
    if (64u * j < gh.cnt) f(gh.pv[j], gh.po[j], lane + 64 * j < gh.cnt);
  }
  for (uint32_t e0 = 64 * kPre; e0 < gh.cnt; e0 += 64) {
    const uint32_t e = e0 + lane;
    const bool valid = e < gh.cnt;
    const uint32_t at = gh.start + ((e + gh.rot) & (uint32_t)(kWaveTile - 1));
    f(valid ? cval[at] : 0u, (OFF && valid) ? (uint32_t)coff[at] : 0u, valid);
  }
}

// ---------------------------------------------------------------------------
// gather: the keys of all candidates that lie in some slot's first-digit bin are appended
// to one list per node (order is irrelevant for what follows).  Each wavefront buffers up to
// kGatherCap keys in LDS and appends them with one reservation on the node's cursor.
// ---------------------------------------------------------------------------
constexpr int kGatherCap = 1024;
constexpr int kCurStride = 64;    // one cursor per 256 bytes: read-modify-writes on one cache line serialise

template <int P>
__global__ __launch_bounds__(kBlock) void k_gather(NodeSet ns) {
  __shared__ uint32_t buf[4][kGatherCap];
  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6;
  if (ns.skip[node] != 0) return;
  const uint32_t lane = tid & 63;
  const int p = ns.lv.p;
  const size_t row = (size_t)node * (size_t)ns.d;
  const uint32_t* __restrict__ cval = ns.cand_val + row;
  const uint16_t* __restrict__ coff = ns.cand_off + row;
  uint32_t* __restrict__ list = ns.glist + row;
  const uint32_t* __restrict__ counts = ns.grp_count + (size_t)node * ns.groups;
  uint32_t pre[P];
#pragma unroll
  for (int s = 0; s < P; ++s) pre[s] = s < p ? ns.prefix[node * p + s] : 0xFFFFFFFFu;
  __shared__ uint32_t s_held[4];
  __shared__ uint32_t s_base;
  uint32_t held = 0;
  auto flush_to = [&](uint32_t base) {
    for (uint32_t i = lane; i < held; i += 64) list[base + i] = buf[w][i];
    held = 0;
  };
  for_groups<false>(cval, coff, counts, blockIdx.x * 4 + w, ns.groups, gridDim.x * 4, ns.d, lane, [&](const GroupHead& cur, int) {
    group_visit<false>(cur, cval, coff, lane, [&](uint32_t vbits, uint32_t, bool valid) {
      const uint32_t key = vbits & 0x7FFFFFFFu;
      const uint32_t bin = key >> kShift0;
      bool hit = false;
#pragma unroll
      for (int s = 0; s < P; ++s) hit = hit || bin == pre[s];
      hit = hit && valid;
      const uint64_t b = ballot(hit);
      if (b != 0) {
        const uint32_t nhit = popc64(b);
        if (held + nhit > (uint32_t)kGatherCap) {       // rare: the wavefront appends on its own
          uint32_t base = 0;
          if (lane == 0) base = atomicAdd(&ns.gcur[(size_t)node * kCurStride], held);
          flush_to(__builtin_amdgcn_readfirstlane(base));
        }
        if (hit) buf[w][held + below(b)] = key;
        held += nhit;
      }
    });
  });
  // one reservation per block for what the four wavefronts still hold
  if (lane == 0) s_held[w] = held;
  __syncthreads();
  if (tid == 0) {
    const uint32_t tot = s_held[0] + s_held[1] + s_held[2] + s_held[3];
    s_base = tot ? atomicAdd(&ns.gcur[(size_t)node * kCurStride], tot) : 0u;
  }
  __syncthreads();
  uint32_t base = s_base;
  for (int i = 0; i < w; ++i) base += s_held[i];
  flush_to(base);
}

// ---------------------------------------------------------------------------
// select: one block per (slot, node) finishes the radix select of that slot's threshold on
// the node's gathered keys: second digit (10 bits), third digit (9 bits) -> exact T_s, the
// number of ties to take r_s, and the number of keys equal to T_s.
// ---------------------------------------------------------------------------
constexpr int kSelBlock = 1024;
constexpr uint32_t kSelSmall = 1u << 15;   // lists up to this length are finished by one block
constexpr int kSelUnroll = 8;

// counts, into an LDS histogram, the keys of list[begin, end) whose bits above `shift_hi`
// equal `prefix`, binned by the nb-bin digit at `shift_lo` (16-byte loads when `vec`)
__device__ __forceinline__ void select_count(const uint32_t* __restrict__ list, uint32_t begin, uint32_t end, bool vec,
                                             uint32_t prefix, int shift_hi, int shift_lo, int nb, uint32_t* hist) {
  const uint32_t tid = threadIdx.x;
  // consecutive keys of a thread that fall into the same bin are counted with one atomic: lists
  // made of one repeated key (all zeros, say) would otherwise serialise on a single LDS word
  uint32_t run_bin = 0, run_len = 0;
  auto count = [&](uint32_t key, bool ok) {
    if (ok && (key >> shift_hi) == prefix) {
      const uint32_t b = (key >> shift_lo) & (nb - 1);
      if (b != run_bin && run_len) {
        atomicAdd(&hist[run_bin], run_len);
        run_len = 0;
      }
      run_bin = b;
      ++run_len;
    }
  };
  if (vec) {        // begin is a multiple of 4 and the row start is 16-byte aligned
    const uint4* __restrict__ l4 = reinterpret_cast<const uint4*>(list);
    const uint32_t e4 = (end + 3) / 4;
    auto sweep = [&](uint32_t i0, auto unroll) {      // unroll 16-byte loads in flight per thread
      constexpr int U = decltype(unroll)::value;
      uint4 k[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t i = i0 + u * kSelBlock + tid;
        k[u] = i < e4 ? l4[i] : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t i = i0 + u * kSelBlock + tid;
        count(k[u].x, 4 * i + 0 < end); count(k[u].y, 4 * i + 1 < end); count(k[u].z, 4 * i + 2 < end); count(k[u].w, 4 * i + 3 < end);
      }
    };
    uint32_t i0 = begin / 4;
    for (; i0 + (kSelUnroll - 2) * kSelBlock < e4; i0 += kSelUnroll * kSelBlock) sweep(i0, std::integral_constant<int, kSelUnroll>());
    for (; i0 < e4; i0 += 2 * kSelBlock) sweep(i0, std::integral_constant<int, 2>());
  } else {
    for (uint32_t i = begin + tid; i < end; i += kSelBlock) count(list[i], true);
  }
  if (run_len) atomicAdd(&hist[run_bin], run_len);
}

// walks nb <= 1024 bin counts from the top (thread t holds the count of bin nb-1-t) and finds
// the bin where the running count reaches `rank`; res = {bin, rank inside the bin, bin count}
__device__ __forceinline__ void select_walk(uint32_t c, int nb, uint32_t rank, uint32_t* res, uint32_t* wsum16) {
  const uint32_t tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  uint32_t inc = c;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(inc, o, 64);
    if (lane >= (uint32_t)o) inc += t;
  }
  __syncthreads();
  if (lane == 63) wsum16[w] = inc;
  __syncthreads();
  uint32_t cum = inc - c;
  for (uint32_t i = 0; i < w; ++i) cum += wsum16[i];
  if (c && cum < rank && rank <= cum + c) {
    res[0] = nb - 1 - tid;
    res[1] = rank - cum;
    res[2] = c;
  }
  __syncthreads();
}

// Lists of up to kSelSmall keys: block z = 0 of the first launch does both digits on its own and
// the second launch has nothing to do.  Longer lists (up to the whole vector when a threshold
// bin holds most of it, e.g. many equal magnitudes): every launch does one digit; one block per
// kSelSmall keys (at most gridDim.z) of a (slot, node) shares the list, the blocks add their LDS
// histograms into a global one, and the block that arrives last walks it.  Blocks without a
// share exit at once.
template <int STAGE>
__global__ __launch_bounds__(kSelBlock) void k_select(NodeSet ns) {
  __shared__ uint32_t hist[kBins1];
  __shared__ uint32_t wsum16[16];
  __shared__ uint32_t res[3];
  __shared__ int s_flag;
  const int s = blockIdx.x, node = blockIdx.y, z = blockIdx.z, tid = threadIdx.x;
  if (ns.skip[node] != 0) return;
  const int p = ns.lv.p;
  const uint32_t* __restrict__ list = ns.glist + (size_t)node * (size_t)ns.d;
  const uint32_t L = ns.gcur[(size_t)node * kCurStride];
  const bool vec = (ns.d % 4) == 0;
  const bool small = L <= kSelSmall;
  if (small && (STAGE == 2 || z != 0)) return;
  // longer lists are shared by one block per kSelSmall keys, as far as the launch has blocks
  const uint32_t zn = min((uint32_t)gridDim.z, (L + kSelSmall - 1) / kSelSmall);
  if (!small && (uint32_t)z >= zn) return;
  uint32_t prefix = ns.prefix[node * p + s];   // 12 bits known before stage 1, 22 before stage 2
  uint32_t rank = ns.rank[node * p + s];
  if (small) {
    for (int stage = 0; stage < 2; ++stage) {
      const int nb = stage == 0 ? kBins1 : kBins2;
      for (int b = tid; b < kBins1; b += kSelBlock) hist[b] = 0;
      if (tid < 3) res[tid] = tid == 1 ? 1u : 0u;
      __syncthreads();
      select_count(list, 0, L, vec, prefix, stage == 0 ? kShift0 : kShift1, stage == 0 ? kShift1 : 0, nb, hist);
      __syncthreads();
      select_walk(tid < nb ? hist[nb - 1 - tid] : 0u, nb, rank, res, wsum16);
      prefix = (prefix << (stage == 0 ? 10 : 9)) | res[0];
      rank = res[1];
      __syncthreads();
    }
  } else {
    constexpr int nb = STAGE == 1 ? kBins1 : kBins2;
    for (int b = tid; b < kBins1; b += kSelBlock) hist[b] = 0;
    if (tid < 3) res[tid] = tid == 1 ? 1u : 0u;
    __syncthreads();
    // this block's share of the list, in whole 16-byte words
    const uint32_t per = ((L + zn - 1) / zn + 3) & ~3u;
    const uint32_t begin = min(L, (uint32_t)z * per), end = min(L, begin + per);
    select_count(list, begin, end, vec, prefix, STAGE == 1 ? kShift0 : kShift1, STAGE == 1 ? kShift1 : 0, nb, hist);
    __syncthreads();
    uint32_t* gh = ns.sel_hist + ((size_t)node * p + s) * kBins1;
    if (tid < nb && hist[tid]) atomicAdd(&gh[tid], hist[tid]);
    if (!arrive_last(&ns.sel_done[((size_t)node * p + s) * (kArriveFan + 1) * kCounterStride], zn, z, &s_flag))
      return;
    uint32_t c = 0;
    if (tid < nb) {
      c = ld_coherent(&gh[nb - 1 - tid]);
      gh[nb - 1 - tid] = 0;
    }
    select_walk(c, nb, rank, res, wsum16);
    prefix = (prefix << (STAGE == 1 ? 10 : 9)) | res[0];
    rank = res[1];
  }
  if (tid == 0) {
    ns.prefix[node * p + s] = prefix;   // after the last digit: exact threshold key T_s
    ns.rank[node * p + s] = rank;       // ... ties to take
    ns.eqcnt[node * p + s] = res[2];    // ... keys equal to T_s
  }
}

// ---------------------------------------------------------------------------
// tally: counts and band energies against the exact thresholds; epilogue = level choice.
// Block b owns the contiguous group range [b*GB, (b+1)*GB), GB = ceil(groups / G2); the
// compact kernel uses the same mapping.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, uint32_t lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(v, o, 64);
    if (lane >= (uint32_t)o) v += t;
  }
  return v;
}

template <int P>
__global__ __launch_bounds__(kBlock) void k_tally(NodeSet ns) {
  __shared__ double red[4];
  __shared__ uint32_t lds4[4];
  __shared__ int s_flag;
  __shared__ double s_strict[kMaxLevels];
  __shared__ uint32_t s_tg[4][P], s_te[4][P];
  __shared__ int s_slot;
  __shared__ uint32_t s_r;
  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int p = ns.lv.p;
  const int groups = ns.groups;
  const int GB = (groups + ns.G2 - 1) / ns.G2;
  const int lo = blockIdx.x * GB, hi = min(groups, lo + GB);
  const size_t row = (size_t)node * (size_t)ns.d;
  const uint32_t* __restrict__ cval = ns.cand_val + row;
  const uint16_t* __restrict__ coff = ns.cand_off + row;
  uint32_t T[P], tg[P], te[P];
  double strict[P];
#pragma unroll
  for (int s = 0; s < P; ++s) {
    T[s] = s < p ? ns.prefix[node * p + s] : 0u;
    strict[s] = 0.0;
    tg[s] = te[s] = 0;
  }
  const uint32_t* __restrict__ counts = ns.grp_count + (size_t)node * groups;
  const bool skip = ns.skip[node] != 0;         // the node keeps h: no candidates were extracted
  // (a level set without any Top-K level has no candidate arrays at all: nothing to read either)
  for (int g = lo + w; g < ((skip || p == 0) ? lo : hi); g += 4) {
    const GroupHead cur = group_load<false>(cval, coff, counts, g, ns.d, lane);
    uint32_t cg[P], ce[P];
#pragma unroll
    for (int s = 0; s < P; ++s) cg[s] = ce[s] = 0;
    group_visit<false>(cur, cval, coff, lane, [&](uint32_t vbits, uint32_t, bool valid) {
      const uint32_t key = vbits & 0x7FFFFFFFu;
      const double dv = (double)__uint_as_float(vbits);
      const double ev = dv * dv;
#pragma unroll
      for (int s = 0; s < P; ++s) {
        if (s < p) {
          cg[s] += popc64(ballot(valid && key > T[s]));
          ce[s] += popc64(ballot(valid && key == T[s]));
          if (valid && key < T[s]) strict[s] += ev;
        }
      }
    });
#pragma unroll
    for (int s = 0; s < P; ++s) {
      if (s < p) {
        if (lane == 0) {
          ns.cnt_gt[((size_t)node * p + s) * groups + g] = cg[s];
          ns.cnt_eq[((size_t)node * p + s) * groups + g] = ce[s];
        }
        tg[s] += cg[s];
        te[s] += ce[s];
      }
    }
  }
  if (lane == 0) {
#pragma unroll
    for (int s = 0; s < P; ++s) { s_tg[w][s] = tg[s]; s_te[w][s] = te[s]; }
  }
#pragma unroll
  for (int s = 0; s < P; ++s) {
    if (s < p) {
      const double e = block_sum(strict[s], red);     // (contains the barriers that publish s_tg / s_te)
      if (tid == 0) st_coherent(&ns.partStrict[((size_t)node * ns.G2 + blockIdx.x) * p + s], e);
    }
  }
  __syncthreads();
  if (tid < p) {
    const size_t o = ((size_t)node * p + tid) * ns.G2 + blockIdx.x;
    st_coherent(&ns.blk_gt[o], s_tg[0][tid] + s_tg[1][tid] + s_tg[2][tid] + s_tg[3][tid]);
    st_coherent(&ns.blk_eq[o], s_te[0][tid] + s_te[1][tid] + s_te[2][tid] + s_te[3][tid]);
  }
  if (!arrive_last(&ns.done[(size_t)node * (kArriveFan + 1) * kCounterStride], gridDim.x, blockIdx.x, &s_flag)) return;

  // ---- epilogue: realised errors, the AdaCGD cascade, message layout per block ----
  for (int s = 0; s < p; ++s) {
    double e = 0.0;
    for (int b = tid; b < (int)gridDim.x; b += kBlock)
      e += ld_coherent(&ns.partStrict[((size_t)node * ns.G2 + b) * p + s]);
    e = block_sum(e, red);
    if (tid == 0) s_strict[s] = e;
  }
  __syncthreads();
  if (tid == 0) {
    const LevelTable& lv = ns.lv;
    const double S = ns.S[node], D = ns.D[node], Eb = ns.Eb[node];
    double err[kMaxLevels];
    for (int j = 0; j < lv.m; ++j) {
      if (skip) {
        err[j] = __longlong_as_double(0x7FF8000000000000ll);    // not evaluated: the cascade stopped before
      } else if (lv.kind[j] == kTopK) {
        const int s = lv.ref[j];
        const double tv = (double)__uint_as_float(ns.prefix[node * p + s]);
        const double left = (double)(ns.eqcnt[node * p + s] - ns.rank[node * p + s]);   // ties not taken
        err[j] = Eb + s_strict[s] + left * (tv * tv);
      } else if (lv.kind[j] == kRank) {
        err[j] = ns.rk_err[node * lv.nr + lv.ref[j]];
      } else {
        err[j] = ns.qerr[node * lv.nq + lv.ref[j]];
      }
      ns.err[node * lv.m + j] = err[j];
    }
    int jstar;
    if (skip) {                                    // (the scan took this decision: S <= bound of position 0)
      jstar = 0;                                   // keep h: communication skipped
    } else {
      jstar = lv.m;
      for (int j = 1; j < lv.m; ++j)
        if (err[j - 1] <= trigger_bound(lv, j, S, D)) { jstar = j; break; }
    }
    ns.level[node] = jstar;
    atomicAdd(&ns.level_hist[jstar], 1ull);
    if (p > 0) ns.gcur[(size_t)node * kCurStride] = 0;
    int slot = -1, q = -1, rk = -1;
    if (jstar > 0) {
      if (lv.kind[jstar - 1] == kTopK) slot = lv.ref[jstar - 1];
      else if (lv.kind[jstar - 1] == kRank) rk = lv.ref[jstar - 1];
      else q = lv.ref[jstar - 1];
    }
    ns.sel_slot[node] = slot;
    ns.sel_q[node] = q;
    if (lv.nr > 0) ns.sel_rk[node] = rk;
    ns.msg_count[node] = slot >= 0 ? lv.K[slot] : 0u;
    // (the message tables, this scale among them, are read by the previous step's aggregation: the first
    // kernel that may write them is this one, which in overlap mode is ordered behind that aggregation)
    if (lv.nq > 0) ns.qscale[node] = 0.f;       // the apply kernel sets it if the chosen level is a quantiser
    if (slot >= 0) {
      ns.sel_T[node] = ns.prefix[node * p + slot];
      ns.sel_r[node] = ns.rank[node * p + slot];
      s_r = ns.rank[node * p + slot];
      ns.grp_off[(size_t)node * (groups + 1) + groups] = lv.K[slot];
    }
    s_slot = slot;
  }
  __syncthreads();
  const int slot = s_slot;
  if (slot < 0) return;
  // ties are taken in coordinate order: block b takes clamp(r - ties before b, 0, ties in b)
  const uint32_t r = s_r;
  const uint32_t* bgt = ns.blk_gt + ((size_t)node * p + slot) * ns.G2;
  const uint32_t* beq = ns.blk_eq + ((size_t)node * p + slot) * ns.G2;
  uint32_t eq_carry = 0, out_carry = 0;
  for (int b0 = 0; b0 < (int)gridDim.x; b0 += kBlock) {
    const int b = b0 + tid;
    const bool in = b < (int)gridDim.x;
    const uint32_t ce = in ? ld_coherent(&beq[b]) : 0u;
    const uint32_t cg = in ? ld_coherent(&bgt[b]) : 0u;
    uint32_t tot_e, tot_o;
    const uint32_t eqb = eq_carry + block_excl_scan(ce, lds4, &tot_e);
    const uint32_t take = eqb >= r ? 0u : min(ce, r - eqb);
    const uint32_t outb = out_carry + block_excl_scan(cg + take, lds4, &tot_o);
    if (in) {
      ns.blk_eqb[(size_t)node * ns.G2 + b] = eqb;
      ns.blk_out[(size_t)node * ns.G2 + b] = outb;
    }
    eq_carry += tot_e;
    out_carry += tot_o;
  }
}

// ---------------------------------------------------------------------------
// compact: message of the chosen Top-K level, h <- h + C_j(v)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_compact(NodeSet ns, PassArgs a) {
  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int slot = ns.sel_slot[node];
  if (slot < 0) return;
  const uint32_t T = ns.sel_T[node], r = ns.sel_r[node];
  const int groups = ns.groups, p = ns.lv.p;
  const int GB = (groups + ns.G2 - 1) / ns.G2;
  const int lo = blockIdx.x * GB, hi = min(groups, lo + GB);
  if (lo >= hi) return;
  const size_t row = (size_t)node * (size_t)ns.d;
  const uint32_t* __restrict__ cval = ns.cand_val + row;
  const uint16_t* __restrict__ coff = ns.cand_off + row;
  float* __restrict__ h = a.h + row;
  int32_t* __restrict__ midx = ns.msg_idx + (size_t)node * ns.Kcap;
  float* __restrict__ mval = ns.msg_val + (size_t)node * ns.Kcap;
  const uint32_t* cgt = ns.cnt_gt + ((size_t)node * p + slot) * groups;
  const uint32_t* ceq = ns.cnt_eq + ((size_t)node * p + slot) * groups;
  const uint32_t* __restrict__ counts = ns.grp_count + (size_t)node * groups;
  uint32_t eq_base = ns.blk_eqb[(size_t)node * ns.G2 + blockIdx.x];
  uint32_t out_base = ns.blk_out[(size_t)node * ns.G2 + blockIdx.x];
  // every wavefront scans the block's groups 64 at a time (lane i <-> group c0 + i) to get each
  // group's message offset and tie rank, then handles the groups with (g - lo) % 4 == w
  for (int c0 = lo; c0 < hi; c0 += 64) {
    const int gi = c0 + (int)lane;
    const uint32_t ce = gi < hi ? ceq[gi] : 0u;
    const uint32_t cg = gi < hi ? cgt[gi] : 0u;
    const uint32_t eq_inc = wave_incl_scan(ce, lane);
    const uint32_t eqb_l = eq_base + eq_inc - ce;
    const uint32_t take = eqb_l >= r ? 0u : min(ce, r - eqb_l);
    const uint32_t out_inc = wave_incl_scan(cg + take, lane);
    const uint32_t out_l = out_base + out_inc - (cg + take);
    const int nchunk = min(64, hi - c0);
    for (int i = w; i < nchunk; i += 4) {
      const int g = c0 + i;
      const GroupHead cur = group_load<true>(cval, coff, counts, g, ns.d, lane);
      uint32_t eqb = __shfl(eqb_l, i, 64);
      uint32_t out = __shfl(out_l, i, 64);
      if (lane == 0) ns.grp_off[(size_t)node * (groups + 1) + g] = out;
      const uint32_t gbase = (uint32_t)g * kWaveTile;
      group_visit<true>(cur, cval, coff, lane, [&](uint32_t vbits, uint32_t off, bool valid) {
        const uint32_t key = vbits & 0x7FFFFFFFu;
        const bool eq = valid && key == T;
        const uint64_t beq = ballot(eq);
        const bool tk = valid && (key > T || (eq && eqb + below(beq) < r));
        const uint64_t bt = ballot(tk);
        if (tk) {
          const uint32_t pos = out + below(bt);
          const float val = __uint_as_float(vbits);
          const uint32_t l = gbase + off;
          midx[pos] = (int32_t)l;
          mval[pos] = val;
          h[l] = a.assign ? val : h[l] + val;
        }
        eqb += popc64(beq);
        out += popc64(bt);
      });
    }
    eq_base += __shfl(eq_inc, 63, 64);
    out_base += __shfl(out_inc, 63, 64);
  }
}

// ---------------------------------------------------------------------------
// qapply: dense update h <- h + C_b(v) and codes, for nodes whose chosen level is a quantiser
// ---------------------------------------------------------------------------
template <bool DIFF, bool VEC>
__global__ __launch_bounds__(kBlock) void k_qapply(NodeSet ns, PassArgs a) {
  const int node = blockIdx.y, tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int q = ns.sel_q[node];
  if (q < 0) return;
  const int64_t d = ns.d;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  float* __restrict__ h = a.h + row;
  int16_t* __restrict__ codes = ns.qcodes + row;
  const int B = ns.lv.qblock[q];                    // 0: one scale for the whole vector
  const float qs = ns.lv.qs[q];
  const float qa_node = B ? 0.f : __uint_as_float(ns.amax[node]);
  const float qc_node = qa_node > 0.f ? (float)((double)qa_node / ns.lv.qdenom[q]) : 0.f;
  if (blockIdx.x == 0 && tid == 0) ns.qscale[node] = qc_node;
  const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
  const uint32_t ctr1 = (uint32_t)node | a.node_flag;
  for (int t = blockIdx.x; t < ns.tiles; t += gridDim.x) {
    const int64_t base = (int64_t)t * kTile;
    uint32_t bkey = 0u;
    float bcq = 0.f;
    if (B) {          // scales of this group's blocks; the first lane of every block stores the block's c
      const int grp = t * 4 + w;
      block_scales(ns.segmax + (size_t)node * ns.nseg, ns.nseg, grp, B, ns.lv.qdenom[q], lane, &bkey, &bcq);
      const int64_t seg = (int64_t)grp * kSegPerGroup + lane;
      const int per = B / kSeg;
      if (lane < (uint32_t)kSegPerGroup && seg < ns.nseg && (lane % per) == 0)
        ns.qbscale[(size_t)node * ns.nseg + seg / per] = bcq;
    }
#pragma unroll
    for (int k = 0; k < kIter; ++k) {
      const int64_t l0 = comp0<VEC>(base, w, lane, k);
      float xv[4], hv[4];
      load4<VEC>(x, l0, d, xv);
      load4<VEC>(h, l0, d, hv);
      uint32_t rnd[4];
      if (VEC) philox4x32_10((uint32_t)(l0 >> 2), ctr1, a.step, 0u, k0, k1, rnd);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int64_t l = comp_index<VEC>(l0, c);
        float qa = qa_node, qc = qc_node;
        if (B) {
          const int sg = k * 4 + (VEC ? (int)(lane >> 4) : c);
          qa = __uint_as_float((uint32_t)__shfl(bkey, sg, 64));
          qc = __shfl(bcq, sg, 64);
        }
        if (l < d) {
          const float vv = DIFF ? xv[c] : xv[c] - hv[c];
          uint32_t word;
          if (VEC) {
            word = rnd[c];
          } else {
            uint32_t r4[4];
            philox4x32_10((uint32_t)(l >> 2), ctr1, a.step, 0u, k0, k1, r4);
            word = r4[l & 3];
          }
          int code = 0;
          const float cq = qa > 0.f ? quant_one(vv, qa, qs, qc, dither_of(word), &code) : 0.f;
          h[l] = hv[c] + cq;
          codes[l] = (int16_t)code;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// small: the whole compression step of a node in one block, for d <= kSmallMax (the scale of the
// paper's own experiments, where a step of the general sequence is a dozen launches of a few
// microseconds each).  The coordinates are sorted in LDS by the total order of Top-K -- key
// descending, index ascending -- so every Top-K size is a prefix of the sorted order; errors are
// sums over the rest; then the cascade, and the message in ascending coordinate by a scan over a
// flag per coordinate.  Same arithmetic per element as the general kernels.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double small_sum(double v, double* red, int nw) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

template <bool DIFF, bool QUANT>      // QUANT: the level set holds quantisers (otherwise their code is left out)
__global__ __launch_bounds__(1024) void k_small(NodeSet ns, PassArgs a) {
  __shared__ uint64_t ck[kSmallMax];       // (key << 32) | ~index, sorted descending
  __shared__ float sv[kSmallMax];          // v by coordinate
  __shared__ uint8_t flag[kSmallMax];      // 1 = coordinate belongs to the message
  __shared__ double red[16];
  __shared__ uint32_t redu[16];
  __shared__ double s_slot_err[kMaxLevels], s_qerr[kMaxLevels];
  __shared__ uint32_t segk[kSmallMax / kSeg];   // largest key of every 64-coordinate segment (block-wise quantiser scales)
  __shared__ int s_slot, s_q;
  __shared__ int s_flag;
  const bool serve = a.agg_new != nullptr;     // what the aggregation reads goes through coherent accesses
  const int node = blockIdx.x, tid = threadIdx.x, NT = blockDim.x, nw = NT >> 6;
  const int lane = tid & 63, w = tid >> 6;
  const int d = (int)ns.d;
  const LevelTable& lv = ns.lv;
  const int p = lv.p, nq = lv.nq;
  const size_t row = (size_t)node * (size_t)d;
  const float* __restrict__ x = a.x + row;
  float* __restrict__ h = a.h + row;
  const float* __restrict__ y = DIFF ? nullptr : a.y + row;
  float* __restrict__ yc = a.ycopy ? a.ycopy + row : nullptr;
  int dp = 64;
  while (dp < d) dp <<= 1;

  // ---- v, ||v||^2, ||x - y||^2, max |v|, sort keys ----
  double S = 0.0, D = 0.0;
  uint32_t kmax = 0;
  const bool blockwise = QUANT && lv.nqb > 0;
  if (blockwise) {
    for (int i = tid; i < kSmallMax / kSeg; i += NT) segk[i] = 0u;
    __syncthreads();
  }
  // scale a (as a float) of the block of B coordinates that holds coordinate i: the maximum over its segments
  auto block_max = [&](int i, int B) {
    const int per = B / kSeg, s0 = (i / B) * per;
    uint32_t m = 0u;
    for (int j = 0; j < per && (s0 + j) * kSeg < d; ++j) m = max(m, segk[s0 + j]);
    return __uint_as_float(m);
  };
  for (int i = tid; i < dp; i += NT) {
    if (i < d) {
      const float xv = x[i];
      const float v = DIFF ? xv : xv - h[i];
      if (!DIFF) {
        const double dw = (double)(xv - y[i]);
        D = fma(dw, dw, D);
        if (yc) yc[i] = xv;
      }
      const double dv = (double)v;
      S = fma(dv, dv, S);
      const uint32_t key = magkey(v);
      kmax = key > kmax ? key : kmax;
      if (blockwise) atomicMax(&segk[i >> 6], key);
      sv[i] = v;
      ck[i] = ((uint64_t)key << 32) | (uint64_t)(~(uint32_t)i);
    } else {
      ck[i] = 0;                     // sorts behind every coordinate
    }
  }
  S = small_sum(S, red, nw);
  D = small_sum(D, red, nw);
  kmax = wave_max(kmax);
  __syncthreads();
  if (lane == 0) redu[w] = kmax;
  __syncthreads();
  for (int i = 0; i < nw; ++i) kmax = redu[i] > kmax ? redu[i] : kmax;
  const double Dn = DIFF ? a.extD[node] : D;
  // first condition of the cascade: nothing else is evaluated (the compressed start applies its level unconditionally)
  const bool skip = !a.assign && S <= trigger_bound(lv, 0, S, Dn);

  if (!skip) {
    // ---- bitonic sort, descending ----
    for (int k = 2; k <= dp; k <<= 1) {
      for (int j = k >> 1; j > 0; j >>= 1) {
        __syncthreads();
        for (int t = tid; t < (dp >> 1); t += NT) {
          const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
          const int l = i | j;
          const uint64_t ai = ck[i], al = ck[l];
          const bool desc = (i & k) == 0;
          if (desc ? ai < al : ai > al) {
            ck[i] = al;
            ck[l] = ai;
          }
        }
      }
    }
    __syncthreads();
    // ---- realised error of every Top-K size: energy of the ranks behind it ----
    for (int s = 0; s < p; ++s) {
      const int K = (int)lv.K[s];
      double e = 0.0;
      for (int r = K + tid; r < d; r += NT) {
        const double f = (double)__uint_as_float((uint32_t)(ck[r] >> 32));
        e = fma(f, f, e);
      }
      e = small_sum(e, red, nw);
      if (tid == 0) s_slot_err[s] = e;
    }
    // ---- realised error of every quantiser level ----
    if (QUANT && nq > 0) {
      const float qa = __uint_as_float(kmax);
      const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
      const uint32_t ctr1 = (uint32_t)node | a.node_flag;
      double qacc[kMaxLevels];
#pragma unroll
      for (int q = 0; q < kMaxLevels; ++q) qacc[q] = 0.0;
      for (int i = tid; i < d; i += NT) {
        uint32_t r4[4];
        philox4x32_10((uint32_t)(i >> 2), ctr1, a.step, 0u, k0, k1, r4);
        const float u = dither_of(r4[i & 3]);
        const float v = sv[i];
#pragma unroll
        for (int q = 0; q < kMaxLevels; ++q) {
          if (q < nq) {
            const float aq = lv.qblock[q] ? block_max(i, lv.qblock[q]) : qa;
            const float qc = aq > 0.f ? (float)((double)aq / lv.qdenom[q]) : 0.f;
            int code;
            const float cq = aq > 0.f ? quant_one(v, aq, lv.qs[q], qc, u, &code) : 0.f;
            const double e = (double)v - (double)cq;
            qacc[q] = fma(e, e, qacc[q]);
          }
        }
      }
#pragma unroll
      for (int q = 0; q < kMaxLevels; ++q) {
        if (q < nq) {
          const double e = small_sum(qacc[q], red, nw);
          if (tid == 0) s_qerr[q] = e;
        }
      }
    }
  }
  __syncthreads();

  // ---- the cascade ----
  if (tid == 0) {
    double err[kMaxLevels];
    for (int j = 0; j < lv.m; ++j) {
      if (skip) err[j] = __longlong_as_double(0x7FF8000000000000ll);
      else err[j] = lv.kind[j] == kTopK ? s_slot_err[lv.ref[j]] : s_qerr[lv.ref[j]];
      ns.err[node * lv.m + j] = err[j];
    }
    int jstar;
    if (skip) {
      jstar = 0;
    } else {
      jstar = lv.m;
      for (int j = 1; j < lv.m; ++j)
        if (err[j - 1] <= trigger_bound(lv, j, S, Dn)) { jstar = j; break; }
    }
    int slot = -1, q = -1;
    if (jstar > 0) {
      if (lv.kind[jstar - 1] == kTopK) slot = lv.ref[jstar - 1];
      else q = lv.ref[jstar - 1];
    }
    ns.S[node] = S;
    ns.D[node] = Dn;
    ns.level[node] = jstar;
    atomicAdd(&ns.level_hist[jstar], 1ull);
    if (serve) st_coherent(&ns.sel_slot[node], slot);
    else ns.sel_slot[node] = slot;
    ns.sel_q[node] = q;
    ns.msg_count[node] = slot >= 0 ? lv.K[slot] : 0u;
    ns.qscale[node] = 0.f;
    s_slot = slot;
    s_q = q;
  }
  __syncthreads();
  const int slot = s_slot, q = s_q;

  if (slot >= 0) {
    // ---- message of the chosen Top-K size in ascending coordinate, h <- h + C(v) ----
    const int K = (int)lv.K[slot];
    for (int i = tid; i < d; i += NT) flag[i] = 0;
    __syncthreads();
    for (int r = tid; r < K; r += NT) flag[~(uint32_t)ck[r]] = 1;
    __syncthreads();
    const int E = (d + NT - 1) / NT;               // consecutive coordinates per thread
    const int lo = min(d, tid * E), hi = min(d, lo + E);
    uint32_t cnt = 0, low = 0;
    for (int i = lo; i < hi; ++i) {
      cnt += flag[i];
      if (i < kWaveTile) low += flag[i];
    }
    // exclusive prefix of cnt over the threads
    uint32_t inc = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    if (lane == 63) redu[w] = inc;
    __syncthreads();
    uint32_t pos = inc - cnt;
    for (int i = 0; i < w; ++i) pos += redu[i];
    __syncthreads();
    int32_t* __restrict__ midx = ns.msg_idx + (size_t)node * ns.Kcap;
    float* __restrict__ mval = ns.msg_val + (size_t)node * ns.Kcap;
    for (int i = lo; i < hi; ++i) {
      if (flag[i]) {
        const float v = sv[i];
        if (serve) {
          st_coherent(&midx[pos], (int32_t)i);
          st_coherent(&mval[pos], v);
        } else {
          midx[pos] = i;
          mval[pos] = v;
        }
        h[i] = a.assign ? v : h[i] + v;
        ++pos;
      }
    }
    // message offsets of the groups of 2048 coordinates (the aggregation reads them)
    const double lowsum = small_sum((double)low, red, nw);
    if (tid == 0) {
      uint32_t* go = ns.grp_off + (size_t)node * (ns.groups + 1);
      go[0] = 0;
      if (ns.groups == 2) go[1] = (uint32_t)lowsum;
      go[ns.groups] = (uint32_t)K;
    }
  } else if (QUANT && q >= 0) {
    // ---- dense update and codes of the chosen quantiser level ----
    const int B = lv.qblock[q];
    const float qa_node = B ? 0.f : __uint_as_float(kmax);
    const float qs = lv.qs[q];
    const float qc_node = qa_node > 0.f ? (float)((double)qa_node / lv.qdenom[q]) : 0.f;
    const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
    const uint32_t ctr1 = (uint32_t)node | a.node_flag;
    int16_t* __restrict__ codes = ns.qcodes + row;
    if (tid == 0) ns.qscale[node] = qc_node;
    for (int i = tid; i < d; i += NT) {
      uint32_t r4[4];
      philox4x32_10((uint32_t)(i >> 2), ctr1, a.step, 0u, k0, k1, r4);
      float qa = qa_node, qc = qc_node;
      if (B) {
        qa = block_max(i, B);
        qc = qa > 0.f ? (float)((double)qa / lv.qdenom[q]) : 0.f;
        if (i % B == 0) ns.qbscale[(size_t)node * ns.nseg + i / B] = qc;
      }
      int code = 0;
      const float cq = qa > 0.f ? quant_one(sv[i], qa, qs, qc, dither_of(r4[i & 3]), &code) : 0.f;
      h[i] = h[i] + cq;
      codes[i] = (int16_t)code;
    }
  }

  // ---- iterate update that opens the next step, from this node's new estimator (the master) ----
  if (a.xu_out && !serve) {
    __syncthreads();                               // h is complete
    if (node == 0)
      for (int i = tid; i < d; i += NT) a.xu_out[i] = (float)((double)a.xu_x[i] - a.xu_gamma * (double)h[i]);
  }
  if (!serve) return;

  // ---- server aggregation, by the block that finishes last (Top-K messages only) ----
  if (!arrive_last(ns.done, (uint32_t)ns.nn, (uint32_t)node, &s_flag)) return;
  double* acc = reinterpret_cast<double*>(ck);     // the sort buffer is free now
  for (int i = tid; i < d; i += NT) acc[i] = 0.0;
  __syncthreads();
  for (int i = 0; i < ns.nn; ++i) {
    const int sl = ld_coherent(&ns.sel_slot[i]);
    if (sl < 0) continue;                          // same in every thread
    const int K = (int)lv.K[sl];
    const int32_t* __restrict__ mi = ns.msg_idx + (size_t)i * ns.Kcap;
    const float* __restrict__ mv = ns.msg_val + (size_t)i * ns.Kcap;
    for (int e = tid; e < K; e += NT) acc[ld_coherent(&mi[e])] += (double)ld_coherent(&mv[e]);   // distinct coordinates
    __syncthreads();
  }
  const double nn = (double)ns.nn;
  for (int i = tid; i < d; i += NT) {
    const float gn = (float)((double)a.agg_old[i] + acc[i] / nn);
    a.agg_new[i] = gn;
    if (a.xu_out) a.xu_out[i] = (float)((double)a.xu_x[i] - a.xu_gamma * (double)gn);
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
static inline bool vec_ok(const NodeSet& ns, const PassArgs& a) {
  auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  return (ns.d % 4 == 0) && al(a.x) && al(a.h) && (a.diff || al(a.y)) && (!a.ycopy || al(a.ycopy));
}

hipError_t launch_scan(const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  const dim3 grid(ns.G, ns.nn), block(kBlock);
  const bool v = vec_ok(ns, a);
  if (a.diff) {
    if (v) hipLaunchKernelGGL((k_scan<true, true>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_scan<true, false>), grid, block, 0, st, ns, a);
  } else {
    if (v) hipLaunchKernelGGL((k_scan<false, true>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_scan<false, false>), grid, block, 0, st, ns, a);
  }
  return hipGetLastError();
}

template <bool DIFF, bool VEC>
static void launch_filter_q(const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  const dim3 grid(ns.G, ns.nn), block(kBlock);
  const int nq = ns.lv.nq;
  if (ns.lv.nqb > 0) {       // some of the quantiser levels are block-wise
    if (VEC && nq == 1) hipLaunchKernelGGL((k_filter<DIFF, VEC, VEC ? 1 : kMaxLevels, true>), grid, block, 0, st, ns, a);
    else if (VEC && nq == 2) hipLaunchKernelGGL((k_filter<DIFF, VEC, VEC ? 2 : kMaxLevels, true>), grid, block, 0, st, ns, a);
    else if (VEC && nq == 3) hipLaunchKernelGGL((k_filter<DIFF, VEC, VEC ? 3 : kMaxLevels, true>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_filter<DIFF, VEC, kMaxLevels, true>), grid, block, 0, st, ns, a);
    return;
  }
  if (nq == 0) hipLaunchKernelGGL((k_filter<DIFF, VEC, 0, false>), grid, block, 0, st, ns, a);
  else if (VEC && nq == 1) hipLaunchKernelGGL((k_filter<DIFF, VEC, VEC ? 1 : kMaxLevels, false>), grid, block, 0, st, ns, a);
  else if (VEC && nq == 2) hipLaunchKernelGGL((k_filter<DIFF, VEC, VEC ? 2 : kMaxLevels, false>), grid, block, 0, st, ns, a);
  else if (VEC && nq == 3) hipLaunchKernelGGL((k_filter<DIFF, VEC, VEC ? 3 : kMaxLevels, false>), grid, block, 0, st, ns, a);
  else hipLaunchKernelGGL((k_filter<DIFF, VEC, kMaxLevels, false>), grid, block, 0, st, ns, a);
}

hipError_t launch_filter(const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  const bool v = vec_ok(ns, a);
  if (a.diff) {
    if (v) launch_filter_q<true, true>(ns, a, st);
    else launch_filter_q<true, false>(ns, a, st);
  } else {
    if (v) launch_filter_q<false, true>(ns, a, st);
    else launch_filter_q<false, false>(ns, a, st);
  }
  return hipGetLastError();
}

hipError_t launch_small(const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  (void)hipGetLastError();
  int dp = 64;
  while (dp < ns.d) dp <<= 1;
  int nt = dp / 2;                       // one compare-exchange per thread and sort stage
  nt = nt < 64 ? 64 : (nt > 1024 ? 1024 : nt);
  const dim3 grid(ns.nn), block(nt);
  if (ns.lv.nq > 0) {
    if (a.diff) hipLaunchKernelGGL((k_small<true, true>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_small<false, true>), grid, block, 0, st, ns, a);
  } else {
    if (a.diff) hipLaunchKernelGGL((k_small<true, false>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_small<false, false>), grid, block, 0, st, ns, a);
  }
  return hipGetLastError();
}

hipError_t launch_sample(const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  (void)hipGetLastError();
  const dim3 grid(ns.nn), block(kSampleBlock);
  if (a.diff) hipLaunchKernelGGL((k_sample<true>), grid, block, 0, st, ns, a);
  else hipLaunchKernelGGL((k_sample<false>), grid, block, 0, st, ns, a);
  return hipGetLastError();
}

hipError_t launch_scanx(const NodeSet& ns, const PassArgs& a, bool repair, hipStream_t st) {
  (void)hipGetLastError();
  // the repair pass almost never has work: a quarter of the blocks keeps its idle launch short
  const dim3 grid(repair ? (ns.G + 3) / 4 : ns.G, ns.nn), block(kBlock);
  if (repair) {
    if (a.diff) hipLaunchKernelGGL((k_scanx<true, true>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_scanx<false, true>), grid, block, 0, st, ns, a);
  } else {
    if (a.diff) hipLaunchKernelGGL((k_scanx<true, false>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_scanx<false, false>), grid, block, 0, st, ns, a);
  }
  return hipGetLastError();
}

hipError_t launch_gather(const NodeSet& ns, hipStream_t st) {
  (void)hipGetLastError();
  if (ns.lv.p == 0) return hipSuccess;
  const dim3 grid(ns.G2, ns.nn), block(kBlock);
  if (ns.lv.p <= 4) hipLaunchKernelGGL((k_gather<4>), grid, block, 0, st, ns);
  else if (ns.lv.p <= 8) hipLaunchKernelGGL((k_gather<8>), grid, block, 0, st, ns);
  else hipLaunchKernelGGL((k_gather<16>), grid, block, 0, st, ns);
  return hipGetLastError();
}

hipError_t launch_select(const NodeSet& ns, hipStream_t st) {
  (void)hipGetLastError();
  if (ns.lv.p == 0) return hipSuccess;
  const dim3 grid(ns.lv.p, ns.nn, ns.GZ);
  hipLaunchKernelGGL((k_select<1>), grid, dim3(kSelBlock), 0, st, ns);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((k_select<2>), grid, dim3(kSelBlock), 0, st, ns);
  return hipGetLastError();
}

hipError_t launch_tally(const NodeSet& ns, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  const dim3 grid(ns.G2, ns.nn), block(kBlock);
  if (ns.lv.p <= 4) hipLaunchKernelGGL((k_tally<4>), grid, block, 0, st, ns);
  else if (ns.lv.p <= 8) hipLaunchKernelGGL((k_tally<8>), grid, block, 0, st, ns);
  else hipLaunchKernelGGL((k_tally<16>), grid, block, 0, st, ns);
  return hipGetLastError();
}

hipError_t launch_compact(const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  if (ns.lv.p == 0) return hipSuccess;
  const dim3 grid(ns.G2, ns.nn), block(kBlock);
  hipLaunchKernelGGL(k_compact, grid, block, 0, st, ns, a);
  return hipGetLastError();
}

hipError_t launch_qapply(const NodeSet& ns, const PassArgs& a, hipStream_t st) {
  (void)hipGetLastError();   // drop a stale error left by earlier runtime calls of this thread
  if (ns.lv.nq == 0) return hipSuccess;
  // no per-block set-up or reduction here: about 8192 short blocks in all
  int gx = (8192 + ns.nn - 1) / ns.nn;
  if (gx > ns.tiles) gx = ns.tiles;
  const dim3 grid(gx, ns.nn), block(kBlock);
  const bool v = vec_ok(ns, a);
  if (a.diff) {
    if (v) hipLaunchKernelGGL((k_qapply<true, true>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_qapply<true, false>), grid, block, 0, st, ns, a);
  } else {
    if (v) hipLaunchKernelGGL((k_qapply<false, true>), grid, block, 0, st, ns, a);
    else hipLaunchKernelGGL((k_qapply<false, false>), grid, block, 0, st, ns, a);
  }
  return hipGetLastError();
}

}  // namespace adacgd
