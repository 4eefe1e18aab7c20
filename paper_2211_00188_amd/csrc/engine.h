// Internal interfaces of the AdaCGD engine: device-side data layout of one
// "node set" (the n workers, or the single master) and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adacgd {

// Tiling of a length-d vector.  A block works on tiles; each of its four wavefronts owns a
// contiguous quarter of the tile, a "group", whose candidates are stored together in
// ascending coordinate.
constexpr int kBlock = 256;             // threads per block (4 wavefronts of 64)
constexpr int kIter = 8;                // 16-byte loads per thread per tile
constexpr int kTile = kIter * kBlock * 4;   // 8192 coordinates
constexpr int kWaveTile = kTile / 4;    // coordinates per group

// Radix digits of the 31-bit magnitude key (bit pattern of |v|), most significant first.
constexpr int kShift0 = 19, kBins0 = 4096;  // sign-less exponent + 4 mantissa bits
constexpr int kShift1 = 9, kBins1 = 1024;
constexpr int kBins2 = 512;

constexpr int kMaxLevels = 16;
constexpr int kSmallMax = 4096;         // largest d handled by the one-block-per-node kernel
constexpr int kSmallServeMax = 64;      // ... which also aggregates when there are at most this many workers
constexpr int kSeg = 64;                // block-wise quantiser scales are built from maxima over segments of 64 coordinates
constexpr int kSegPerGroup = kWaveTile / kSeg;   // 32

enum { kTopK = 0, kQuant = 1, kRank = 2 };

// The ordered level set of one side, in the form the kernels use.
struct LevelTable {
  int m;                      // levels in cascade order (strongest compression first)
  int kind[kMaxLevels];       // kTopK / kQuant / kRank
  int ref[kMaxLevels];        // kTopK: slot index into K[]; kQuant: index into qs[]; kRank: index into rK[]
  int nr;                     // Rank-K levels (the vector read row-major as a (d / rcols) x rcols matrix)
  int rcols;                  // their common number of columns: 16, 32 or 64 (0 if there is none)
  int rK[kMaxLevels];         // their ranks
  int p;                      // distinct Top-K sizes ("slots")
  uint32_t K[kMaxLevels];     // ascending
  int nq;                     // quantiser levels
  int qbits[kMaxLevels];
  int qblock[kMaxLevels];     // 0: one scale for the whole vector; else block length B (a power of two, 64..2048):
                              // one scale per block of B consecutive coordinates
  int nqb;                    // how many of the nq quantisers are block-wise
  float qs[kMaxLevels];       // s = 2^(b-1) - 1 magnitude levels
  double qdenom[kMaxLevels];  // s (1 + omega), omega from d (whole vector) or from B (block-wise)
  // Trigger of cascade position j (0 = keep h, j = level j; the last level has none):
  //   err_j <= tz[j] ||x-y||^2 + te[j] ||x-h||^2,  err_0 = ||x-h||^2.  fp32 arguments widened.
  double tz[kMaxLevels];
  double te[kMaxLevels];
};

// Device arrays of one side.  nn nodes, each with a length-d vector.
struct NodeSet {
  int nn;
  int64_t d;
  int tiles;        // ceil(d / kTile)
  int groups;       // ceil(d / kWaveTile): candidate groups, one per wavefront share of a tile
  int G;            // blocks per node of the streaming kernels (scan, filter)
  int G2;           // blocks per node of the candidate kernels
  int GZ;           // blocks per (slot, node) of the select kernels
  int onepass;      // 1: sample + scanx sequence, 0: scan + filter sequence
  int small;        // 1: d <= kSmallMax: one kernel, one block per node, does the whole step
  uint32_t Kcap;    // message capacity per node = largest Top-K size (0 if none)
  LevelTable lv;

  uint32_t* hist0;      // [nn][kBins0]           first-digit counts; zero between launches
  uint32_t* sel_hist;   // [nn][p][kBins1]        digit counts of long gathered lists; zero between launches
  uint32_t* sel_done;   // [nn][p][kArriveFan+1]  arrival counters of the select kernels
  uint32_t* gcur;       // [nn]                   keys gathered so far; zero between steps
  uint32_t* glist;      // [nn][d]                keys of the candidates inside the slots' first-digit bins
  uint32_t* prefix;     // [nn][p]                known high bits of slot threshold T_s (12, 22, 31 bits)
  uint32_t* rank;       // [nn][p]                rank of the K_s-th element inside the prefix
  uint32_t* eqcnt;      // [nn][p]                count of keys equal to T_s
  uint32_t* bmin;       // [nn]                   lowest first-digit bin that holds candidates
  uint32_t* best;       // [nn]                   candidate cut (a key) estimated from the sample
  uint32_t* redo;       // [nn]                   1 = fewer candidates than the largest K: the repair passes run
  uint32_t* skip;       // [nn]                   1 = ||x-h||^2 <= zeta ||x-y||^2: h is kept, no selection work
  uint32_t* done;       // [nn][kArriveFan+1]     arrival counters of the last-block epilogues
  uint32_t* partU;      // [nn][G]                per block: largest key (two-pass scan) or candidates found (fused scan)
  uint32_t* amax;       // [nn]                   max magnitude key of the last scan (quantiser scale a)
  uint32_t* segmax;     // [nn][nseg]             max magnitude key of every 64-coordinate segment (only with block-wise
                        //                        quantiser levels): a block's scale is the max over its segments
  float* qbscale;       // [nn][nseg]             scales c_k of the last block-wise quantised message, entry k = block k
  int nseg;             // ceil(d / 64)
  double* partS;        // [nn][G]
  double* partD;        // [nn][G]
  double* partEb;       // [nn][G]
  double* partQ;        // [nn][G][nq]
  double* partStrict;   // [nn][G2][p]
  double* S;            // [nn]  ||x-h||^2
  double* D;            // [nn]  ||x-y||^2
  double* Eb;           // [nn]  energy below the candidate bins
  double* qerr;         // [nn][nq]
  double* err;          // [nn][m]
  uint32_t* grp_count;  // [nn][groups]
  uint32_t* cnt_gt;     // [nn][p][groups] candidates with key > T_s
  uint32_t* cnt_eq;     // [nn][p][groups] candidates with key == T_s
  uint32_t* blk_gt;     // [nn][p][G2]  per tally block: candidates with key > T_s
  uint32_t* blk_eq;     // [nn][p][G2]  per tally block: candidates with key == T_s
  uint32_t* blk_out;    // [nn][G2]     message offset of the block's first group, chosen level
  uint32_t* blk_eqb;    // [nn][G2]     ties before the block's first group, chosen level
  uint32_t* grp_off;    // [nn][groups+1] message offset of each group's first entry (last = total)
  uint32_t* cand_val;   // [nn][d]  value bits of the candidates; group g starts at g * kWaveTile
  uint16_t* cand_off;   // [nn][d]  their coordinate offsets inside the group, same layout
  int32_t* level;       // [nn]   0 = skip
  int32_t* sel_slot;    // [nn]   slot of the chosen Top-K level, -1 otherwise
  int32_t* sel_q;       // [nn]   quantiser index of the chosen level, -1 otherwise
  uint32_t* sel_T;      // [nn]
  uint32_t* sel_r;      // [nn]
  uint32_t* msg_count;  // [nn]
  int32_t* msg_idx;     // [nn][Kcap]
  float* msg_val;       // [nn][Kcap]
  unsigned long long* level_hist;  // [m+1]
  unsigned long long* repairs;     // [1] node-steps whose sampled cut was too high (second scan ran)
  int16_t* qcodes;      // [nn][d] (only with quantiser levels)
  float* qscale;        // [nn]
  double* accbuf;       // [d] fp64 sums of the sparse messages (only with quantiser levels)
  // Rank-K levels (allocated only when the level set has any; c = lv.rcols, nr = lv.nr)
  int GR;               // blocks per node of the Rank-K kernels
  double* gram_part;    // [nn][GR][c*c]  partial Gram matrices X^T X of the blocks (upper triangle, tile by tile)
  double* rk_lambda;    // [nn][c]        its eigenvalues (squared singular values of X), descending
  double* rk_V;         // [nn][c*c]      its eigenvectors (right singular vectors of X) as columns, in the same order
  double* rk_part;      // [nn][GR][nr]   partial realised errors
  double* rk_err;       // [nn][nr]       realised error of every Rank-K level
  float* rdense;        // [nn][d]        C(v) of the last Rank-K message (the aggregation adds it)
  int32_t* sel_rk;      // [nn]           Rank-K level (index into rK) of the chosen level, -1 otherwise
  int AS;               // aggregation: blocks that share one group's workers (1 = one block per group)
  double* agg_part;     // [AS][groups][kWaveTile] their partial sums (AS > 1)
  uint32_t* agg_done;   // [groups][kArriveFan+1] arrival counters (AS > 1); zero between launches
};

// Operands of one application of the compressor C_{h,y}(x) to every node of a set.
struct PassArgs {
  const float* x;      // [nn][d]  new point; in difference mode the difference vector itself
  float* h;            // [nn][d]  stored estimator, updated in place
  const float* y;      // [nn][d]  previous point (unused in difference mode)
  float* ycopy;        // optional [nn][d]: receives a copy of x
  const double* extD;  // difference mode: [nn] given ||x-y||^2
  int diff;            // 1 = difference mode
  uint64_t seed;       // Philox key
  uint32_t step;       // Philox counter word 2
  uint32_t node_flag;  // OR-ed into counter word 1 (0 for workers, 2^31 for the master)
  int assign;          // 1 = the compressed start g~_i^0 = C_m(grad f_i(x^0)) (Section 2.3): h holds zeros and receives
                       // the selected values themselves, h[l] = C(v)[l], instead of fl(h[l] + C(v)[l]) (Top-K only)
  // Server work that the one-block kernel for short vectors can take over (each part optional):
  // the block that finishes last adds every node's message to the server vector, g~_new =
  // fl(g~_old + sum / nn); and the iterate update that opens the next step, x_next = fl(x - gamma g),
  // with g = g~_new when it follows the aggregation, else g = the updated estimator of node 0 (the master).
  const float* agg_old;
  float* agg_new;
  const float* xu_x;
  float* xu_out;
  double xu_gamma;
};

struct LogisticData {
  const float* A;
  const float* labels;
  const int64_t* offsets;  // device [n+1]
  const int32_t* row_node; // device [rows]
  int64_t rows;
  int64_t max_rows;        // largest shard
  double lambda;
  double* margins;         // [rows]  s_l = -y_l / (1 + exp(y_l a_l^T x)) / N_i
  double* part;            // [n][row_chunks][d] when row_chunks > 1
  uint32_t* col_done;      // [n][column blocks] arrival counters when row_chunks > 1; zero between launches
  int row_chunks;
  // Sparse features (GRAD_LOGISTIC_CSR): device copies made at init.  The transposed copy holds
  // every worker's entries sorted by column, then by row, so that one thread sums a column of a
  // shard in a fixed order.
  int csr;                 // 1: the fields below are used instead of A
  int binary;              // 1: every stored entry is 1 (no value arrays)
  int64_t nnz;
  const int64_t* rp;       // [rows+1]
  const int32_t* ci;       // [nnz] column of each entry, ascending within a row
  const float* cv;         // [nnz]
  const int64_t* wbase;    // [n+1]  first entry of each worker = rp[offsets[i]]
  const uint32_t* cptr;    // [n][d+1]  start of column j of worker i in the transposed copy, relative to wbase[i]
  const int32_t* trow;     // [nnz] row (global) of each transposed entry
  const float* tval;       // [nnz]
};

// launchers (each enqueues on the stream and returns the launch status)
hipError_t launch_scan(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_filter(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_gather(const NodeSet& ns, hipStream_t st);
hipError_t launch_select(const NodeSet& ns, hipStream_t st);
hipError_t launch_small(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_sample(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_scanx(const NodeSet& ns, const PassArgs& a, bool repair, hipStream_t st);
hipError_t launch_tally(const NodeSet& ns, hipStream_t st);
hipError_t launch_compact(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_qapply(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_rank_gram(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_rank_eig(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_rank_errors(const NodeSet& ns, const PassArgs& a, hipStream_t st);
hipError_t launch_rank_apply(const NodeSet& ns, const PassArgs& a, hipStream_t st);

hipError_t launch_xupdate(float* x, const float* g, double gamma, int64_t d, hipStream_t st);
hipError_t launch_mean(const float* gi, float* out0, float* out1, float* out2, int n, int64_t d, hipStream_t st);
// optional extra of a kernel that finishes g: x_next = fl(x - gamma g) (out == nullptr: not asked for)
struct IterateUpdate {
  const float* x = nullptr;
  float* out = nullptr;
  double gamma = 0.0;
};
hipError_t launch_aggregate(const NodeSet& ws, const float* gt_old, float* gt_new, const IterateUpdate& xu,
                            hipStream_t st);
hipError_t launch_fill_u32(uint32_t* p, uint32_t v, size_t count, hipStream_t st);
hipError_t launch_copy_f32(float* dst, const float* src, size_t count, hipStream_t st);
hipError_t launch_grad_margins(const LogisticData& ld, const float* x, int64_t d, hipStream_t st);
hipError_t launch_grad_cols(const LogisticData& ld, const float* x, float* grads, int n, int64_t d, hipStream_t st);

}  // namespace adacgd
