// Damped Cholesky factor of the inverse Hessian:  U upper, U^T U = H_d^{-1}.
//
// Route.  With J the index reversal, G = J H_d J = L L^T (ordinary lower
// Cholesky) gives H_d = R R^T with R = J L J upper, hence H_d^{-1} = R^{-T} R^{-1}
// and U = R^{-1} = J L^{-1} J.  So one Cholesky factorization and one
// triangular inverse, both on the reversed matrix, and the result written back
// through the reversal.  Both are done by one recursion on the diagonal block
// [o, o+s) of G, which returns X = L^{-1} of that block:
//
//     split s = s1 + s2
//     X11           = rec(G11)
//     L21           = G21 X11^T                       (GEMM, X11 triangular)
//     G22          -= L21 L21^T                       (SYRK, lower tiles)  } one launch
//     T             = L21 X11                                              }
//     X22           = rec(G22)
//     X21           = -X22 T
//
// Every off-diagonal step is a float64 MFMA GEMM; only blocks of at most 128
// columns are factored and inverted inside one workgroup (in LDS).  L itself
// is never needed again, so only X is kept: it is stored directly in U through
// the reversal, X(i,j) = U[n-1-i][n-1-j].  L21^T is parked in the (otherwise
// unused) upper triangle of the work matrix, L21 X11 in the dead G21 block.
#include "dgemm.h"

#include <atomic>
#include <functional>
#include <mutex>

namespace ptq {
namespace {

constexpr int kLeaf = 128;          // largest block factored inside one workgroup

// ---- diagonal statistics: dead channels, mean of the fixed diagonal ---------
__global__ __launch_bounds__(1024) void diag_stats_kernel(const double* __restrict__ H, int64_t ldh,
                                                          int n, double damp, uint8_t* dead_mask,
                                                          double* scal, int32_t* info) {
  __shared__ double part[1024];
  double s = 0.0;
  for (int j = threadIdx.x; j < n; j += 1024) {
    double d = H[(int64_t)j * ldh + j];
    const bool dead = (d == 0.0);
    if (dead) d = 1.0;
    if (dead_mask) dead_mask[j] = dead ? 1 : 0;
    s += d;
  }
  part[threadIdx.x] = s;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    scal[0] = damp * (part[0] / (double)n);
    info[0] = PTQ_OK;
    info[1] = 0;
  }
}

// G = J H_d J (lower triangle, zeros above), and U cleared.
__global__ __launch_bounds__(256) void build_work_kernel(const double* __restrict__ H, int64_t ldh,
                                                         int n, const double* __restrict__ scal,
                                                         double* __restrict__ G, double* __restrict__ U,
                                                         int64_t ldu) {
  const int i = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  double g = 0.0;
  if (j <= i) {
    const int hi = n - 1 - i, hj = n - 1 - j;  // hi <= hj: upper triangle of H
    g = H[(int64_t)hi * ldh + hj];
    if (i == j) {
      if (g == 0.0) g = 1.0;
      g += scal[0];
    }
  }
  G[(int64_t)i * n + j] = g;
  U[(int64_t)i * ldu + j] = 0.0;
}

// ---- leaf: X = inverse of the Cholesky factor of G[o:o+s, o:o+s], s <= 128 ---
// The block lives in LDS and is processed in 16 x 16 sub-blocks, right-looking, by eight waves.
// The critical path is the chain of 128 pivots, so the pivots of block column d (a 16-column
// panel with all rows below it) are the only work that waits for anything:
//
//   A(d)  waves 0-3   panel d: factor the diagonal sub-block, invert its factor (X_dd) and form
//                     L_id for every i > d
//         waves 4-7   G_ij -= L_{i,d-1} L_{j,d-1}^T  for i >= j > d                    ("R(d-1)")
//                     T_ij += L_{i,d-2} X_{d-2,j}  for i > d-2, j <= d-2             ("C(d-2)")
//   B(d)  all waves   G_{i,d+1} -= L_id L_{d+1,d}^T  for i > d     (what panel d+1 waits for)
//                     X_{d-1,j} = -X_{d-1,d-1} T_{d-1,j}  for j < d-1               ("F(d-1)")
//
// and after the last panel  A': C(nb-2);  B': F(nb-1).  The off-diagonal part of the inverse
// therefore trails the factorization by two steps and is off the chain except for this tail.
//
// The panel: each of the four waves holds the 16 x 16 diagonal sub-block, one column per lane
// and replicated in its four rows of 16 lanes (register k = row k), plus a sixteenth of the rows
// below it (seven registers).  Eliminating pivot j is then  v -= bcast_j(v) * (D(j,c) / D(j,j))
// on every register, where bcast_j hands lane j's value to its row of 16 lanes (DPP
// row_newbcast, no LDS, no scalar round trip) and D(j,c) is the lane's own register j (the
// trailing block is kept symmetric): one multiply-add per register and pivot, all columns at
// once.  The columns stay unscaled until the end, so the chain per pivot is one broadcast, one
// reciprocal square root (hardware estimate + two Newton steps), two multiplications and the
// multiply-add of the next pivot's row.  The column operations that turn D into L, applied to
// the rows of the identity, give L^-T: four more registers per wave and the inverse of the
// diagonal factor needs no pass of its own.
//
// X_ij (i > j) and before it T_ij are parked in the unused upper sub-block (j, i); the
// inverses of the diagonal sub-blocks have a strip of their own.
constexpr int kLeafThreads = 512;
constexpr int kLeafP = kLeaf + 1;   // pitch of the LDS block
// LDS: the block [128][129]; the inverses of the diagonal sub-blocks side by side in a strip [16][129] of
// the same pitch; a dump slot per thread of the panel waves [256]
constexpr size_t kLeafLdsBytes = (size_t)(kLeaf * kLeafP + 16 * kLeafP + 256) * sizeof(double);

// The DPP forms below are written as assembly because the compiler neither folds a 64-bit DPP move
// into the multiply-add nor sees these instructions when it counts wait states: a DPP read needs two
// wait states (two instructions, or s_nop 1) after a vector write of the register it reads.  Every
// instruction of a wave costs an issue slot of four cycles, an s_nop included, so the statements
// below carry none: the caller keeps the distance.  Each multiply-add reads, through DPP, only the
// accumulator it updates, which in the panel was last written a whole pivot earlier; the one read
// that follows its producer closely (the broadcast of the next pivot) is placed two multiply-adds
// after it.  (That the compiler puts no copy of an accumulator in front of a statement is checked
// on the generated assembly when the library is built.)
template <int J>
__device__ __forceinline__ double row_bcast(double v) {
  double p;
  asm volatile("v_mov_b64_dpp %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf" : "=v"(p) : "v"(v), "n"(J));
  return p;
}
template <int J>
__device__ __forceinline__ void fmac_bcast1(double nc, double& a) {
  asm volatile("v_fmac_f64_dpp %0, %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf" : "+v"(a) : "v"(nc), "n"(J));
}
// (the same, naming a value that must exist before it: the statements keep their order, so whatever
// computes `before` cannot sink below this one, and unlike an in-out operand it costs no wait state)
template <int J>
__device__ __forceinline__ void fmac_bcast1_after(double nc, double& a, double before) {
  asm volatile("v_fmac_f64_dpp %0, %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf"
               : "+v"(a)
               : "v"(nc), "n"(J), "v"(before));
}
// r[LO .. HI) += bcast_J(r) * nc
template <int J, int LO, int HI, int N>
__device__ __forceinline__ void fmac_bcast_range(double nc, double (&r)[N]) {
  if constexpr (LO < HI) {
    fmac_bcast1<J>(nc, r[LO]);
    fmac_bcast_range<J, LO + 1, HI>(nc, r);
  }
}

constexpr int kPanelWaves = 2;                               // waves that factor the panel (each on a SIMD of its own)
static_assert(kPanelWaves == 2, "the work split below gives waves 2, 3, 6, 7 the products and 4, 5 the stores");
constexpr int kPanelSlots = 4 * kPanelWaves;                 // rows of 16 lanes among them
constexpr int kRowsPerBlock = 16 / kPanelSlots;              // rows of each sub-block that one of them holds
constexpr int kPanelRows = (kLeaf / 16 - 1) * kRowsPerBlock; // registers for the rows below the diagonal sub-block
constexpr int kIdentityRows = 16 / kPanelWaves;              // rows of the identity per wave: i = kPanelWaves m + wave

// The registers of a panel wave: the diagonal sub-block, its share of the rows below, and its four
// rows of the identity that the same column operations turn into the inverse of the factor.
struct PanelRegs {
  double Dg[16], A[kPanelRows], E[kIdentityRows];
};
// The I-th of the multiply-adds of pivot J that nothing waits for: rows J+2 .. 15 of the diagonal
// sub-block, then the rows below it, then the identity rows that can be non-zero in column J (row
// kPanelWaves m + wave is zero left of its own column, so m <= J / kPanelWaves).
template <int J, int I>
__device__ __forceinline__ void panel_pending(double nc, PanelRegs& R, double before) {
  constexpr int nd = 14 - J, ne = J / kPanelWaves + 1;
  if constexpr (I < nd)
    fmac_bcast1_after<J>(nc, R.Dg[J + 2 + I], before);
  else if constexpr (I < nd + kPanelRows)
    fmac_bcast1_after<J>(nc, R.A[I - nd], before);
  else if constexpr (I < nd + kPanelRows + ne)
    fmac_bcast1_after<J>(nc, R.E[I - nd - kPanelRows], before);
  else
    asm volatile("" : : "v"(before));
}
template <int J, int LO>
__device__ __forceinline__ void panel_pending_from(double nc, PanelRegs& R) {
  constexpr int nd = 14 - J, ne = J / kPanelWaves + 1;
  if constexpr (LO < nd + kPanelRows + ne) {
    panel_pending<J, LO>(nc, R, nc);
    panel_pending_from<J, LO + 1>(nc, R);
  }
}

// Stage J of the panel: the multiply-adds of pivot J (coefficients nc), written out interleaved with the
// chain that leads to pivot J+1's coefficients -- broadcast of D(J+1,J+1), reciprocal square root,
// r^2 D(J+1, c) -- one multiply-add in the shadow of each dependent operation.  The compiler does not know
// what the assembly costs and would sort the two apart again, so each operation of the chain is fenced:
// the multiply-add after it names its result (volatile statements keep their order, so the operation
// cannot sink below the statement), and a scheduling barrier on either side keeps the scheduler from
// moving it.  A pivot that is not positive makes r and everything after it non-finite; the caller finds
// it in rl.
#define PTQ_CHAIN(stmt, I, dep)                 \
  __builtin_amdgcn_sched_barrier(0);            \
  stmt;                                         \
  __builtin_amdgcn_sched_barrier(0);            \
  panel_pending<J, I>(nc, R, dep);

template <int J>
__device__ __forceinline__ void panel_stage(PanelRegs& R, double nc, double& rl, int c) {
  if constexpr (J == 15) {
    panel_pending_from<15, 0>(nc, R);
  } else {
    fmac_bcast1<J>(nc, R.Dg[J + 1]);  // the next pivot's row first
    panel_pending<J, 0>(nc, R, nc);   // (two statements, always there: the wait states of the
    panel_pending<J, 1>(nc, R, nc);   //  DPP read of the row just written)
    static_assert(kPanelRows >= 2, "the broadcast needs two statements between it and its producer");
    const double p = row_bcast<J + 1>(R.Dg[J + 1]);
    PTQ_CHAIN(double r = __builtin_amdgcn_rsq(p), 2, r)
    PTQ_CHAIN(const double h = -0.5 * p, 3, h)
    PTQ_CHAIN(const double dm = (c > J + 1) ? R.Dg[J + 1] : 0.0, 4, dm)   // D(J+1, c) for the columns still to come
    PTQ_CHAIN(double t = h * r, 5, t)
    PTQ_CHAIN(double u = fma(t, r, 1.5), 6, u)
    PTQ_CHAIN(r = r * u, 7, r)
    PTQ_CHAIN(t = h * r, 8, t)
    PTQ_CHAIN(u = fma(t, r, 1.5), 9, u)
    PTQ_CHAIN(r = r * u, 10, r)
    PTQ_CHAIN(const double rr = r * r, 11, rr)
    PTQ_CHAIN(const double next = -(rr * dm), 12, next)
    panel_pending_from<J, 13>(nc, R);
    rl = (c == J + 1) ? r : rl;
    panel_stage<J + 1>(R, next, rl, c);
  }
}
#undef PTQ_CHAIN

__global__ __launch_bounds__(kLeafThreads) void leaf_kernel(const double* __restrict__ G, int n, int o, int s,
                                                            double* __restrict__ U, int64_t ldu, int32_t* info) {
  extern __shared__ double lds[];
  double* S = lds;                                    // [128][129]
  double* XD = lds + kLeaf * kLeafP;                  // [16][129]: X_kk(i, j) at XD[i * 129 + 16 k + j]
  double* DUMP = XD + 16 * kLeafP;                    // [256]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps the work-list arithmetic scalar
  const int nb = (s + 15) >> 4, sp = nb << 4;
  const int l16 = lane & 15, lq = lane >> 4;

  // load the lower triangle: thread = (column j, row mod 4), all its loads in flight at once
  // (padding rows / columns beyond s: identity)
  {
    const int j = tid & 127, i0 = tid >> 7;
    double v[kLeaf / 4];
#pragma unroll
    for (int u = 0; u < kLeaf / 4; ++u) {
      const int i = i0 + 4 * u;
      const bool ld = (i < s) & (j <= i);
      v[u] = ld ? G[(int64_t)(o + i) * n + o + j] : ((i == j) ? 1.0 : 0.0);
    }
#pragma unroll
    for (int u = 0; u < kLeaf / 4; ++u) {
      const int i = i0 + 4 * u;
      if (i < sp && j < sp) S[i * kLeafP + j] = v[u];
    }
  }
  __syncthreads();

  // ---- the panel of block column d (waves 0-3).  Taken branches are what this wave can least afford
  // (each costs tens of cycles of instruction fetch), hence addresses chosen by selection, not code by branch.
  auto panel = [&](int d) {
    const int b0 = 16 * d, c = l16;
    const int below = nb - 1 - d;          // sub-blocks under the diagonal one
    const int rr = 4 * wave + lq;          // this lane's row of 16 lanes among the panel's
    PanelRegs R;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int hi = k > c ? k : c, lo = k > c ? c : k;
      R.Dg[k] = S[(b0 + hi) * kLeafP + b0 + lo];
    }
#pragma unroll
    for (int m = 0; m < kIdentityRows; ++m) {
      R.E[m] = (c == kPanelWaves * m + wave) ? 1.0 : 0.0;
      asm volatile("" : "+v"(R.E[m]));   // in a register of its own from here on, not copied into one at its first use
    }
    // rows that do not exist (t >= below) read some valid element and are never written back: what
    // they hold stays in their own register
    double* sub = S + (b0 + 16 + rr) * kLeafP + b0 + c;   // this lane's first element of the first sub-block below
    double* own = S + (b0 + c) * kLeafP + b0 + c;
    // register t: sub-block t / kRowsPerBlock, row (t % kRowsPerBlock) * kPanelSlots + rr of it
    auto row_of = [](int t) { return ((t / kRowsPerBlock) * 16 + (t % kRowsPerBlock) * kPanelSlots) * kLeafP; };
#pragma unroll
    for (int t = 0; t < kPanelRows; ++t) R.A[t] = *((t < below * kRowsPerBlock) ? sub + row_of(t) : own);
    // pivot 0's coefficients, then the sixteen stages
    double rl;
    {
      const double p = row_bcast<0>(R.Dg[0]);
      const double h = -0.5 * p;
      double r = __builtin_amdgcn_rsq(p);
      r = r * fma(h * r, r, 1.5);
      r = r * fma(h * r, r, 1.5);
      rl = r;
      const double nc = (c > 0) ? -((r * r) * R.Dg[0]) : 0.0;
      panel_stage<0>(R, nc, rl, c);
    }
    // scale column c by its reciprocal pivot; only now do the entries become those of L
    // (rows that do not exist go to a dump slot of the lane's own)
    double* dump = DUMP + tid;   // (tid < 64 kPanelWaves)
#pragma unroll
    for (int t = 0; t < kPanelRows; ++t) *((t < below * kRowsPerBlock) ? sub + row_of(t) : dump) = R.A[t] * rl;
    // the same column operations applied to the identity give the inverse factor transposed:
    // X_dd(c, i) = E_i(c) r_c, for this wave's rows i = kPanelWaves m + wave
    if (lq == 0) {
#pragma unroll
      for (int m = 0; m < kIdentityRows; ++m) XD[c * kLeafP + b0 + kPanelWaves * m + wave] = R.E[m] * rl;
    }
    // the diagonal sub-block, which both waves hold: each writes half of its rows
    // (rows above the diagonal get what the registers hold: nothing reads that triangle)
    if (lq == 0) {
      if (wave == 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) S[(b0 + k) * kLeafP + b0 + c] = R.Dg[k] * rl;
      } else {
#pragma unroll
        for (int k = 8; k < 16; ++k) S[(b0 + k) * kLeafP + b0 + c] = R.Dg[k] * rl;
      }
    }
    if (wave == 0) {
      // the first pivot that was not positive: its reciprocal root is the first that is not a positive number
      const unsigned long long notpos = __ballot(!(rl > 0.0 && rl < __builtin_huge_val())) & 0xffffull;
      if (notpos != 0) {
        const int bad = __builtin_ctzll(notpos);
        if (b0 + bad < s && lane == 0 && info[0] == PTQ_OK) {
          info[0] = PTQ_ERR_NOT_SPD;
          info[1] = n - 1 - (o + b0 + bad);
        }
      }
    }
  };

  // ---- 16 x 16 x 16 sub-block products  C = (C or 0) +- A B,  one wave each, two at a time so that
  // the MFMA chain of one fills the latency of the other.  All operands have the pitch of the block, so
  // every fragment is one LDS read at an immediate offset from a per-item base, and the work loops
  // contain no branch but their own.  (An odd item out is given twice: both copies have read before
  // either writes, and they write the same.)
  struct Item {
    const double* a;   // A(i, k) = a[i * 129 + k]
    const double* b;   // B(k, j) = b[k * 129 + j], or with BT  b[j * 129 + k]
    double* c;         // C(i, j) = c[i * 129 + j]
    bool fresh;        // C starts from zero
  };
  auto product2 = [&](auto bt, auto neg, const Item& x, const Item& y) {
    constexpr bool BT = decltype(bt)::value, NEG = decltype(neg)::value;
    const int oa = l16 * kLeafP + lq, ob = BT ? oa : lq * kLeafP + l16, oc = lq * kLeafP + l16;
    const double *xa = x.a + oa, *xb = x.b + ob, *ya = y.a + oa, *yb = y.b + ob;
    double *xc = x.c + oc, *yc = y.c + oc;
    double ax[4], bx[4], ay[4], by[4];
    f64x4 cx, cy;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      ax[kk] = xa[4 * kk];
      bx[kk] = xb[BT ? 4 * kk : 4 * kk * kLeafP];
      cx[kk] = xc[4 * kk * kLeafP];
      ay[kk] = ya[4 * kk];
      by[kk] = yb[BT ? 4 * kk : 4 * kk * kLeafP];
      cy[kk] = yc[4 * kk * kLeafP];
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      cx[kk] = x.fresh ? 0.0 : cx[kk];
      cy[kk] = y.fresh ? 0.0 : cy[kk];
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      cx = __builtin_amdgcn_mfma_f64_16x16x4f64(NEG ? -ax[kk] : ax[kk], bx[kk], cx, 0, 0, 0);
      cy = __builtin_amdgcn_mfma_f64_16x16x4f64(NEG ? -ay[kk] : ay[kk], by[kk], cy, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) xc[4 * r * kLeafP] = cx[r];
#pragma unroll
    for (int r = 0; r < 4; ++r) yc[4 * r * kLeafP] = cy[r];
  };
  // (one product alone: two accumulators, k steps 0,2 and 1,3, halve the dependent chain)
  auto product1 = [&](auto bt, auto neg, const Item& x) {
    constexpr bool BT = decltype(bt)::value, NEG = decltype(neg)::value;
    const int oa = l16 * kLeafP + lq, ob = BT ? oa : lq * kLeafP + l16, oc = lq * kLeafP + l16;
    const double *xa = x.a + oa, *xb = x.b + ob;
    double* xc = x.c + oc;
    double ax[4], bx[4];
    f64x4 c0, c1 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      ax[kk] = xa[4 * kk];
      bx[kk] = xb[BT ? 4 * kk : 4 * kk * kLeafP];
      c0[kk] = xc[4 * kk * kLeafP];
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) c0[kk] = x.fresh ? 0.0 : c0[kk];
#pragma unroll
    for (int kk = 0; kk < 4; kk += 2) {
      c0 = __builtin_amdgcn_mfma_f64_16x16x4f64(NEG ? -ax[kk] : ax[kk], bx[kk], c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f64_16x16x4f64(NEG ? -ax[kk + 1] : ax[kk + 1], bx[kk + 1], c1, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) xc[4 * r * kLeafP] = c0[r] + c1[r];
  };
  using std::false_type;
  using std::true_type;
  auto uniform = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
  // G_ij -= L_ik L_jk^T
  auto update_item = [&](int k, int i, int j) {
    return Item{S + (16 * i) * kLeafP + 16 * k, S + (16 * j) * kLeafP + 16 * k, S + (16 * i) * kLeafP + 16 * j, false};
  };
  // X_kj = -X_kk T_kj, in place in the parked sub-block (j, k)
  auto finish_item = [&](int k, int j) {
    double* blk = S + (16 * j) * kLeafP + 16 * k;
    return Item{XD + 16 * k, blk, blk, true};
  };
  // R(k): the trailing update with block column k of everything right of block column k+1 (that
  // one is on the critical path and has a phase of its own): G_ij -= L_ik L_jk^T, i >= j >= k+2;
  // dealt to `count` waves, this one is number `slot`
  auto rest_of_update = [&](int k, int slot, int count) {
    const int T = nb - 2 - k, items = T * (T + 1) / 2;
    auto item = [&](int q) {
      // item q is (ii, jj), ii >= jj, of the triangle in row order: q = ii (ii + 1) / 2 + jj
      const int ii = uniform((int)((sqrtf((float)(8 * q + 1)) - 1.0f) * 0.5f));
      return update_item(k, k + 2 + ii, k + 2 + q - ii * (ii + 1) / 2);
    };
    for (int q = slot; q < items; q += 2 * count)
      product2(true_type{}, true_type{}, item(q), item(q + count < items ? q + count : q));
  };
  // C(k): T_ij (+)= L_ik X_kj for every i > k, j <= k (the first contribution, j == k, is X_kk's and
  // starts the sum)
  auto contributions = [&](int k, int slot, int count) {
    const int cols = k + 1, items = (nb - 1 - k) * cols;
    const float rcols = 1.0f / (float)cols;
    auto item = [&](int q) {
      const int qi = uniform((int)(((float)q + 0.5f) * rcols));   // q / cols (small integers: exact)
      const int i = k + 1 + qi, j = q - qi * cols;
      const bool first = (j == k);
      return Item{S + (16 * i) * kLeafP + 16 * k, first ? XD + 16 * k : S + (16 * j) * kLeafP + 16 * k,
                  S + (16 * j) * kLeafP + 16 * i, first};
    };
    for (int q = slot; q < items; q += 2 * count)
      product2(false_type{}, false_type{}, item(q), item(q + count < items ? q + count : q));
  };

  // X(i, j), i >= j, goes to U[n-1-(o+i)][n-1-(o+j)].  Rows [r0, r1) of X by `threads` threads, this one
  // being number t: thread = (column, row phase), a column's consecutive threads write consecutive addresses.
  auto store_rows = [&](int r0, int r1, int t, int threads) {
    const int j = t & 127, jb = j >> 4, step = threads >> 7;
    double* ucol = U + (int64_t)(n - 1 - o) * ldu + (n - 1 - (o + j));
    for (int i = r0 + (t >> 7); i < r1; i += step) {
      if (i < s && j <= i) {
        const int ib = i >> 4;
        const double x = (ib == jb) ? XD[(i & 15) * kLeafP + 16 * ib + (j & 15)]
                                    : S[(16 * jb + (i & 15)) * kLeafP + 16 * ib + (j & 15)];
        ucol[-(int64_t)i * ldu] = x;
      }
    }
  };

  for (int d = 0; d <= nb; ++d) {
    // ---- A(d)
    if (d < nb) {
      // (a workgroup's waves go to the four SIMDs in turn: waves 0 and 1 factor the panel, and the
      //  waves that share their SIMDs, 4 and 5, stay out of their way)
      if (wave < kPanelWaves) {
        panel(d);
      } else if ((wave & 3) >= kPanelWaves) {
        const int slot = (wave & 3) - kPanelWaves + (4 - kPanelWaves) * (wave >> 2);   // 0 .. 2 (4 - kPanelWaves) - 1
        constexpr int helpers = 2 * (4 - kPanelWaves);
        if (d >= 1) rest_of_update(d - 1, slot, helpers);
        if (d >= 2) contributions(d - 2, helpers - 1 - slot, helpers);   // (the wave with the fewest items above goes first)
      } else if (d >= 2) {
        // the waves that share the panel's SIMDs have little to do meanwhile: block row d-2 of X is
        // final (its last step was F(d-2) in the phase before) and goes out to memory
        store_rows(16 * (d - 2), 16 * (d - 1), tid - 256, 128);
      }
    } else if (nb >= 2) {
      contributions(nb - 2, wave, 8);
    }
    __syncthreads();
    // ---- B(d): one product per wave.  Block column d+1 gets its update with block column d (nb-1-d
    // products), and F(d-1) its d-1: never more than eight together.
    {
      const int T = d < nb ? nb - 1 - d : 0, fin = d >= 2 ? d - 1 : 0;
      if (wave < T)
        product1(true_type{}, true_type{}, update_item(d, d + 1 + wave, d + 1));
      else if (wave < T + fin)
        product1(false_type{}, true_type{}, finish_item(d - 1, wave - T));
    }
    __syncthreads();
  }

  // the last two block rows of X (the others went out along the way)
  store_rows(nb >= 2 ? 16 * (nb - 2) : 0, sp, tid, kLeafThreads);
}

// ---- the four GEMM steps of one recursion node -------------------------------
// Each step describes its operands as strided views for the tile at (i0, j0):
// A(i, k) and B(k, j) with i, j tile-local and k counted from the block start.
struct Node {
  double* G;      // work matrix, n x n, ld = n
  double* U;      // output, X reversed: X(i, j) = U[n-1-i][n-1-j]
  int ldu;
  int n, o, s1, s2;
  int r;          // first row of the second block: o + s1, except for the early part of a panel or an update
                  // (see recurse), whose k range [o, o + s1) ends before the second block begins
  __device__ __forceinline__ const double* g(int i, int j) const { return G + (int64_t)i * n + j; }
  __device__ __forceinline__ const double* x(int i, int j) const {
    return U + (int64_t)(n - 1 - i) * ldu + (n - 1 - j);
  }
};

// L21 = G21 X11^T, stored transposed in the mirror block of G; columns [c0, s1) of it.
struct OpPanel {
  static constexpr bool A_KFAST = true, B_KFAST = true;
  static constexpr int K_ORDER = +2;  // k range grows with the column tile: last column tile first
  static constexpr bool LOWER_ONLY = false;
  Node nd;
  int c0;
  __device__ int M() const { return nd.s2; }
  __device__ int N() const { return nd.s1 - c0; }
  __device__ bool active(int, int, int, int) const { return true; }
  __device__ void krange(int, int, int, int j1, int& kb, int& ke) const { kb = 0; ke = min(nd.s1, c0 + j1); }
  __device__ DView a(int i0) const { return DView{nd.g(nd.r + i0, nd.o), nd.n, 1}; }
  __device__ DView b(int j0) const { return DView{nd.x(nd.o + c0 + j0, nd.o), -nd.ldu, -1}; }  // X11(j, k)
  __device__ void store(int i, int j, double v) const {
    if (i < nd.s2 && j < nd.s1 - c0) nd.G[(int64_t)(nd.o + c0 + j) * nd.n + nd.r + i] = v;
  }
};

// G22 -= L21 L21^T on the lower triangle (k over the node's columns [o, o + s1)).
struct OpSyrk {
  static constexpr bool A_KFAST = false, B_KFAST = false;
  static constexpr int K_ORDER = 0;   // every active tile has the full k range
  static constexpr bool LOWER_ONLY = true;  // only tiles that touch the lower triangle are launched
  Node nd;
  __device__ int M() const { return nd.s2; }
  __device__ int N() const { return nd.s2; }
  __device__ bool active(int, int i1, int j0, int) const { return i1 > j0; }
  __device__ void krange(int, int, int, int, int& kb, int& ke) const { kb = 0; ke = nd.s1; }
  __device__ DView a(int i0) const { return DView{nd.g(nd.o, nd.r + i0), 1, nd.n}; }  // L21(i, k)
  __device__ DView b(int j0) const { return DView{nd.g(nd.o, nd.r + j0), 1, nd.n}; }  // L21(j, k)
  __device__ void store(int i, int j, double v) const {
    if (i < nd.s2 && j <= i) nd.G[(int64_t)(nd.r + i) * nd.n + nd.r + j] -= v;
  }
};

// T = L21 X11, stored in the dead G21 block.
struct OpT {
  static constexpr bool A_KFAST = false, B_KFAST = false;
  static constexpr int K_ORDER = -2;  // k range shrinks with the column tile: first column tile first
  static constexpr bool LOWER_ONLY = false;
  Node nd;
  __device__ int M() const { return nd.s2; }
  __device__ int N() const { return nd.s1; }
  __device__ bool active(int, int, int, int) const { return true; }
  __device__ void krange(int, int, int j0, int, int& kb, int& ke) const { kb = j0; ke = nd.s1; }
  __device__ DView a(int i0) const { return DView{nd.g(nd.o, nd.o + nd.s1 + i0), 1, nd.n}; }
  __device__ DView b(int j0) const { return DView{nd.x(nd.o, nd.o + j0), -1, -nd.ldu}; }  // X11(k, j)
  __device__ void store(int i, int j, double v) const {
    if (i < nd.s2 && j < nd.s1) nd.G[(int64_t)(nd.o + nd.s1 + i) * nd.n + nd.o + j] = v;
  }
};

// X21 = -X22 T.
struct OpX21 {
  static constexpr bool A_KFAST = true, B_KFAST = false;
  static constexpr int K_ORDER = +1;  // k range grows with the row tile: last row tile first
  static constexpr bool LOWER_ONLY = false;
  Node nd;
  __device__ int M() const { return nd.s2; }
  __device__ int N() const { return nd.s1; }
  __device__ bool active(int, int, int, int) const { return true; }
  __device__ void krange(int, int i1, int, int, int& kb, int& ke) const { kb = 0; ke = min(nd.s2, i1); }
  __device__ DView a(int i0) const {  // X22(i, k)
    return DView{nd.x(nd.o + nd.s1 + i0, nd.o + nd.s1), -nd.ldu, -1};
  }
  __device__ DView b(int j0) const { return DView{nd.g(nd.o + nd.s1, nd.o + j0), 1, nd.n}; }  // T(k, j)
  __device__ void store(int i, int j, double v) const {
    if (i < nd.s2 && j < nd.s1)
      nd.U[(int64_t)(nd.n - 1 - (nd.o + nd.s1 + i)) * nd.ldu + (nd.n - 1 - (nd.o + j))] = -v;
  }
};

// Column tiles of row tile bi that reach the lower triangle (square matrix, tile BM x BN).
template <int TM, int TN>
__host__ __device__ inline int lower_tiles_in_row(int bi, int gx) {
  const int c = ((bi + 1) * 32 * TM - 1) / (32 * TN) + 1;
  return c < gx ? c : gx;
}
template <int TM, int TN>
inline int lower_tiles(int gx, int gy) {
  int s = 0;
  for (int bi = 0; bi < gy; ++bi) s += lower_tiles_in_row<TM, TN>(bi, gx);
  return s;
}

// Tile `lin` of the gx x gy tile grid of a step.  Triangular operands make the k ranges uneven, so
// the tiles are handed out longest first, over the whole grid: the index the k range depends on
// (K_ORDER: +-1 row tile, +-2 column tile; sign = which end is longest) is the slow one.
template <int TM, int TN, class Op>
__device__ __forceinline__ void node_gemm_tile(const Op& op, int lin, int gx, int gy, double* smem) {
  using T = DgemmTile<TM, TN>;
  int bi, bj;
  if (Op::LOWER_ONLY) {
    // row tile bi has lower_tiles_in_row(bi) tiles (bj = 0 ..); rows from the last one up
    bi = gy - 1;
    int c = lower_tiles_in_row<TM, TN>(bi, gx);
    while (lin >= c) {
      lin -= c;
      --bi;
      c = lower_tiles_in_row<TM, TN>(bi, gx);
    }
    bj = lin;
  } else if (Op::K_ORDER == 2 || Op::K_ORDER == -2) {
    const int q = lin / gy;
    bi = lin - q * gy;
    bj = Op::K_ORDER > 0 ? gx - 1 - q : q;
  } else {
    const int q = lin / gx;
    bj = lin - q * gx;
    bi = Op::K_ORDER > 0 ? gy - 1 - q : q;
  }
  // the tile is the same for every lane; said explicitly, because a buffer descriptor that the compiler takes for
  // lane-dependent is loaded through a loop over its distinct values around every request of the k loop
  // (the lower-triangle search above ended up so in the 128 x 128-tile update)
  bi = __builtin_amdgcn_readfirstlane(bi);
  bj = __builtin_amdgcn_readfirstlane(bj);
  const int i0 = bi * T::BM, j0 = bj * T::BN;
  const int i1 = min(i0 + T::BM, op.M()), j1 = min(j0 + T::BN, op.N());
  if (!op.active(i0, i1, j0, j1)) return;
  int kb, ke;
  op.krange(i0, i1, j0, j1, kb, ke);
  f64x4 acc[TM][TN];
  dgemm_zero(acc);
  // a tile with no ragged edge takes the software-pipelined loop (same sums in the same order)
  // (its buffer loads address a tile's footprint with 32-bit byte offsets)
  const DView va = op.a(i0), vb = op.b(j0);
  const int64_t spana = ((int64_t)T::BM * abs(va.so) + (int64_t)(ke - kb) * abs(va.sk)) * 8;
  const int64_t spanb = ((int64_t)T::BN * abs(vb.so) + (int64_t)(ke - kb) * abs(vb.sk)) * 8;
  const bool full = (i1 - i0 == T::BM) && (j1 - j0 == T::BN) && ke > kb && ((ke - kb) % kGemmBK == 0) &&
                    spana < ((int64_t)1 << 31) && spanb < ((int64_t)1 << 31);
  bool done = false;
  if constexpr (TM * TN >= 4) {
    if (full) {
      dgemm_mainloop_pipelined<TM, TN, Op::A_KFAST, Op::B_KFAST>(acc, va, vb, kb, ke, smem);
      done = true;
    }
  }
  if (!done)
    dgemm_mainloop<TM, TN, Op::A_KFAST, Op::B_KFAST>(acc, va, DgemmIdentity{}, vb, DgemmIdentity{}, i1 - i0, j1 - j0,
                                                     kb, ke, smem);
  dgemm_foreach(acc, [&](int i, int j, double v) { op.store(i0 + i, j0 + j, v); });
}

// (64 x 64 tiles: three workgroups per CU, so the registers are capped for three; the 128 x 128 tile
// keeps 128 accumulator registers and two sets of staging registers and runs one or two per CU)
template <int TM, int TN, bool STRIDED, class Op>
__global__ __launch_bounds__(256, (TM * TN == 4) ? 3 : 1) void node_gemm_kernel(Op op, int gx, int gy, int total) {
  extern __shared__ double smem[];
  if constexpr (STRIDED) {
    // fewer workgroups than tiles: a stride over the tile list (both tile loops end with a barrier,
    // so the LDS stages are free when the next tile starts)
    for (int lin = blockIdx.x; lin < total; lin += gridDim.x) node_gemm_tile<TM, TN>(op, lin, gx, gy, smem);
  } else {
    node_gemm_tile<TM, TN>(op, blockIdx.x, gx, gy, smem);
  }
}

// Two independent steps in one launch: workgroups [0, n1) take the tiles of the first.
template <int TM, int TN, class Op1, class Op2>
__global__ __launch_bounds__(256, (TM * TN == 4) ? 3 : 1) void node_gemm2_kernel(Op1 op1, Op2 op2, int n1, int gx1, int gy1, int gx2, int gy2) {
  extern __shared__ double smem[];
  const int b = blockIdx.x;
  if (b < n1)
    node_gemm_tile<TM, TN>(op1, b, gx1, gy1, smem);
  else
    node_gemm_tile<TM, TN>(op2, b - n1, gx2, gy2, smem);
}

// max_wgs > 0 caps the number of workgroups (the tiles are then taken in a stride): used for work that
// runs beside the critical chain on a second stream and must leave compute units free for it
template <int TM, int TN, class Op>
bool launch_tiles(const Op& op, int M, int N, hipStream_t st, int max_wgs = 0) {
  using T = DgemmTile<TM, TN>;
  constexpr int lds = T::kSmemDoubles * (int)sizeof(double);
  const int gx = (int)ceil_div(N, T::BN), gy = (int)ceil_div(M, T::BM);
  const int total = Op::LOWER_ONLY ? lower_tiles<TM, TN>(gx, gy) : gx * gy;
  if (max_wgs > 0 && max_wgs < total) {
    if (!lds_opt_in<node_gemm_kernel<TM, TN, true, Op>>(lds)) return false;
    node_gemm_kernel<TM, TN, true, Op><<<(unsigned)max_wgs, 256, lds, st>>>(op, gx, gy, total);
  } else {
    if (!lds_opt_in<node_gemm_kernel<TM, TN, false, Op>>(lds)) return false;
    node_gemm_kernel<TM, TN, false, Op><<<(unsigned)total, 256, lds, st>>>(op, gx, gy, total);
  }
  return true;
}

template <int TM, int TN, class Op1, class Op2>
bool launch_tiles2(const Op1& op1, int M1, int N1, const Op2& op2, int M2, int N2, hipStream_t st) {
  using T = DgemmTile<TM, TN>;
  constexpr int lds = T::kSmemDoubles * (int)sizeof(double);
  if (!lds_opt_in<node_gemm2_kernel<TM, TN, Op1, Op2>>(lds)) return false;
  const int gx1 = (int)ceil_div(N1, T::BN), gy1 = (int)ceil_div(M1, T::BM);
  const int gx2 = (int)ceil_div(N2, T::BN), gy2 = (int)ceil_div(M2, T::BM);
  const int n1 = Op1::LOWER_ONLY ? lower_tiles<TM, TN>(gx1, gy1) : gx1 * gy1;
  const int n2 = Op2::LOWER_ONLY ? lower_tiles<TM, TN>(gx2, gy2) : gx2 * gy2;
  node_gemm2_kernel<TM, TN, Op1, Op2><<<(unsigned)(n1 + n2), 256, lds, st>>>(op1, op2, n1, gx1, gy1, gx2, gy2);
  return true;
}

// Tile shape by problem size, as measured: 128 x 128 once there are enough tiles to fill the
// chip twice over; up to about a 1500-wide node 32 x 32 tiles (there the k loops are short and
// bound by the latency of their loads, whatever the tile: many small workgroups hide it best);
// 64 x 64 between.
inline int tile_class(int M, int N) {
  if (ceil_div(M, 128) * ceil_div(N, 128) >= 512) return 2;
  if (ceil_div(M, 64) * ceil_div(N, 64) <= 512) return 0;
  return 1;
}

template <class Op>
bool launch_node(const Op& op, int M, int N, hipStream_t st, int max_cus = 0) {
  switch (tile_class(M, N)) {
    case 2: return launch_tiles<4, 4, Op>(op, M, N, st, max_cus);          // one workgroup per compute unit
    case 1: return launch_tiles<2, 2, Op>(op, M, N, st, 3 * max_cus);      // three
    default: return launch_tiles<1, 1, Op>(op, M, N, st, 4 * max_cus);
  }
}

template <class Op1, class Op2>
bool launch_node2(const Op1& op1, int M1, int N1, const Op2& op2, int M2, int N2, hipStream_t st) {
  const int c1 = tile_class(M1, N1), c2 = tile_class(M2, N2);
  switch (c1 < c2 ? c1 : c2) {
    case 2: return launch_tiles2<4, 4, Op1, Op2>(op1, M1, N1, op2, M2, N2, st);
    case 1: return launch_tiles2<2, 2, Op1, Op2>(op1, M1, N1, op2, M2, N2, st);
    default: return launch_tiles2<1, 1, Op1, Op2>(op1, M1, N1, op2, M2, N2, st);
  }
}

// ---- helper streams for work that is off the critical chain -----------------------------------
// The chain  leaf -> panel -> update -> leaf ...  of a half of a node is a sequence of small,
// latency-bound launches that leaves most of the chip idle.  For the largest nodes (128 x 128 tiles)
// two pieces of the node's own work run beside those chains, each on a stream of its own with a cap
// on its workgroups, so that the chain's launches always find free compute units:
//  * beside the chain of the SECOND half:  T = L21 X11  (a quarter of the node's flops), which is
//    needed only by the node's last step -- forked after the trailing update, joined before
//    X21 = -X22 T  (cap kSideCus; measured at n = 11008: 128 gives the shortest total, 256 gains
//    nothing, 64 makes T the longer path);
//  * beside the second half of the FIRST half's recursion:  the early part of the node's panel and
//    update.  Once the first half A = [o, o + sA) of the first child is inverted, the columns
//    [0, sA) of L21 = G21 X11^T are computable (X11 is lower triangular: they need X_A only), and so
//    is their share  G22 -= L21[:, :sA] L21[:, :sA]^T  of the update.  The child signals that point
//    (`on_first_half`), the early part runs on its stream, and after the child the node finishes
//    the panel (columns [sA, s1)) and the update (k in [sA, s1)) on the caller's stream (cap
//    kEarlyCus; n = 11008: 18.0 ms without, 17.9 / 17.4 / 17.5 / 17.6 ms with 128 / 160 / 192 / 224;
//    n = 8192: 9.49 without, 9.04 / 8.95 with 128 / 192).
// Smaller nodes gain nothing (measured) and keep one stream, with T in the update's launch.  The
// streams and a few events per device are created on first use and kept for the life of the
// process (default priority).
constexpr int kSideCus = 128;
constexpr int kEarlyCus = 192;
constexpr int kMaxDepth = 12;
struct Side {
  std::mutex lock;   // the events are reused call after call: one caller at a time enqueues a factor
  hipStream_t stream = nullptr, early_stream = nullptr;
  hipEvent_t fork[kMaxDepth], join[kMaxDepth], early_fork[kMaxDepth], early_join[kMaxDepth];
  bool ok = false;
};

Side* side_for_device() {
  constexpr int kMaxDevices = 64;
  static Side sides[kMaxDevices];
  static std::atomic<int> state[kMaxDevices];   // 0 = untried, 1 = being set up, 2 = ready, 3 = unavailable
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  int expected = 0;
  if (state[dev].compare_exchange_strong(expected, 1)) {
    Side& sd = sides[dev];
    bool ok = hipStreamCreateWithFlags(&sd.stream, hipStreamNonBlocking) == hipSuccess &&
              hipStreamCreateWithFlags(&sd.early_stream, hipStreamNonBlocking) == hipSuccess;
    for (int d = 0; ok && d < kMaxDepth; ++d)
      ok = hipEventCreateWithFlags(&sd.fork[d], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&sd.join[d], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&sd.early_fork[d], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&sd.early_join[d], hipEventDisableTiming) == hipSuccess;
    sd.ok = ok;
    state[dev].store(ok ? 2 : 3, std::memory_order_release);
  }
  while (state[dev].load(std::memory_order_acquire) == 1) {
  }
  return state[dev].load(std::memory_order_acquire) == 2 ? &sides[dev] : nullptr;
}

inline int first_part(int s) { return ((int)ceil_div(s, kLeaf) / 2) * kLeaf; }

// `on_first_half`, if given, is called (on the host) right after the launches that invert the first half of
// this block have been enqueued on st.
bool recurse(double* G, double* U, int ldu, int n, int o, int s, int32_t* info, hipStream_t st, Side* side, int depth,
             const std::function<bool()>* on_first_half = nullptr) {
  if (s <= kLeaf) {
    leaf_kernel<<<1, kLeafThreads, kLeafLdsBytes, st>>>(G, n, o, s, U, ldu, info);
    return true;
  }
  const int s1 = first_part(s);
  const int s2 = s - s1;
  const Node nd{G, U, ldu, n, o, s1, s2, o + s1};
  if (side && depth < kMaxDepth && tile_class(s2, s1) == 2) {
    // a large node.  Early part: beside the second half of the first child's recursion
    const int sA = s1 > kLeaf ? first_part(s1) : 0;
    const bool early = sA > 0 && tile_class(s2, sA) == 2;
    const std::function<bool()> start_early = [&]() -> bool {
      const Node part{G, U, ldu, n, o, sA, s2, o + s1};
      return hipEventRecord(side->early_fork[depth], st) == hipSuccess &&
             hipStreamWaitEvent(side->early_stream, side->early_fork[depth], 0) == hipSuccess &&
             launch_node(OpPanel{part, 0}, s2, sA, side->early_stream, kEarlyCus) &&
             launch_node(OpSyrk{part}, s2, s2, side->early_stream, kEarlyCus) &&
             hipEventRecord(side->early_join[depth], side->early_stream) == hipSuccess;
    };
    if (!recurse(G, U, ldu, n, o, s1, info, st, side, depth + 1, early ? &start_early : nullptr)) return false;
    if (on_first_half && !(*on_first_half)()) return false;
    if (early) {
      const Node rest{G, U, ldu, n, o + sA, s1 - sA, s2, o + s1};
      if (hipStreamWaitEvent(st, side->early_join[depth], 0) != hipSuccess ||
          !launch_node(OpPanel{nd, sA}, s2, s1 - sA, st) || !launch_node(OpSyrk{rest}, s2, s2, st))
        return false;
    } else if (!launch_node(OpPanel{nd, 0}, s2, s1, st) || !launch_node(OpSyrk{nd}, s2, s2, st)) {
      return false;
    }
    // T beside the chain of the second half (fork after the update, join before X21)
    if (hipEventRecord(side->fork[depth], st) != hipSuccess ||
        hipStreamWaitEvent(side->stream, side->fork[depth], 0) != hipSuccess)
      return false;
    if (!launch_node(OpT{nd}, s2, s1, side->stream, kSideCus)) return false;
    if (hipEventRecord(side->join[depth], side->stream) != hipSuccess) return false;
    if (!recurse(G, U, ldu, n, o + s1, s2, info, st, side, depth + 1)) return false;
    if (hipStreamWaitEvent(st, side->join[depth], 0) != hipSuccess) return false;
    return launch_node(OpX21{nd}, s2, s1, st);
  }
  if (!recurse(G, U, ldu, n, o, s1, info, st, side, depth + 1)) return false;
  if (on_first_half && !(*on_first_half)()) return false;
  // the trailing update and T = L21 X11 both need only L21 and touch different blocks
  return launch_node(OpPanel{nd, 0}, s2, s1, st) && launch_node2(OpSyrk{nd}, s2, s2, OpT{nd}, s2, s1, st) &&
         recurse(G, U, ldu, n, o + s1, s2, info, st, side, depth + 1) && launch_node(OpX21{nd}, s2, s1, st);
}

}  // namespace

size_t cholesky_workspace_bytes(int64_t n) {
  return align_up((size_t)n * (size_t)n * sizeof(double), 256) + 256;
}

ptq_status cholesky_launch(const double* H, int64_t ldh, int64_t n, double damp, double* U, int64_t ldu,
                           uint8_t* dead_mask, int32_t* info, void* ws, size_t ws_bytes,
                           hipStream_t st) {
  if (n == 0) return PTQ_OK;
  if (ws_bytes < cholesky_workspace_bytes(n)) return PTQ_ERR_WORKSPACE;
  double* G = static_cast<double*>(ws);
  double* scal = reinterpret_cast<double*>(static_cast<char*>(ws) +
                                           align_up((size_t)n * (size_t)n * sizeof(double), 256));
  if (!lds_opt_in<leaf_kernel>((int)kLeafLdsBytes)) return PTQ_ERR_HIP;
  diag_stats_kernel<<<1, 1024, 0, st>>>(H, ldh, (int)n, damp, dead_mask, scal, info);
  PTQ_HIP_CHECK_LAUNCH();
  dim3 g((unsigned)ceil_div(n, 256), (unsigned)n);
  build_work_kernel<<<g, 256, 0, st>>>(H, ldh, (int)n, scal, G, U, ldu);
  PTQ_HIP_CHECK_LAUNCH();
  // the helper stream only where a node is large enough to use it (the top node is the largest)
  const int top1 = first_part((int)n);
  Side* side = (n > kLeaf && tile_class((int)n - top1, top1) == 2) ? side_for_device() : nullptr;
  bool ok;
  if (side) {
    std::lock_guard<std::mutex> hold(side->lock);
    ok = recurse(G, U, (int)ldu, (int)n, 0, (int)n, info, st, side, 0);
  } else {
    ok = recurse(G, U, (int)ldu, (int)n, 0, (int)n, info, st, nullptr, 0);
  }
  if (!ok) return PTQ_ERR_HIP;
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
