// Relative layer error  sqrt( tr(D H D^T) / tr(W H W^T) ),  D = W - Wq.
//
// H is symmetric and only its upper triangle is stored, so each quadratic form
// is evaluated as  sum_ij A_ij * (A Hu)_ij  with
//     Hu(k,j) = 2 H(k,j) for k < j,  H(k,k) for k == j,  0 for k > j,
// which reads every stored entry once in its coalesced direction and halves the
// work of the float64 MFMA GEMM (the k range of a column tile stops at its last
// column).  Each workgroup reduces its tile to one number; a final
// single-workgroup kernel adds the tile sums in index order.
//
// Two forms of the same sum.  Weights stored in float64 take the float64 MFMA GEMM.  Weights
// stored in float32 or bfloat16 take the bfloat16-split one: D, W and Hu are rounded to float32
// once (W in bfloat16 is exact) and kept as three bfloat16 pieces each, the piece products and
// the running sums over k are float32 on the matrix cores, and everything from the tile's
// sum_ij A_ij T_ij on is float64.  The roundings are unbiased and independent, so they average
// out over the m n terms of the trace: measured against the float64 definition the two traces
// differ by a few parts in 10^9.
#include "dgemm.h"

#include <type_traits>

namespace ptq {
namespace {

constexpr int TM = 2, TN = 4;  // 64 x 128 tile: two workgroups (8 waves) per CU keep the f64 matrix pipe fuller
using Tile = DgemmTile<TM, TN>;

struct ErrArgs {
  const double* A2;  // [2][m][n]: D = W - Wq, then W, both widened to float64
  int m, n;
  const double* H;
  int ldh;
  double* partial;  // [2][tiles]
};

// D = W - Wq next to W itself, both dense, so that the GEMM streams two plain matrices.
__global__ __launch_bounds__(256) void widen_kernel(const double* __restrict__ W, int64_t ldw,
                                                    const double* __restrict__ Wq, int m, int n,
                                                    double* __restrict__ A2) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)m * n) return;
  const int i = (int)(e / n), k = (int)(e - (int64_t)i * n);
  const double w = W[(int64_t)i * ldw + k];
  A2[e] = w - Wq[e];
  A2[(int64_t)m * n + e] = w;
}

__global__ __launch_bounds__(256, 3) void quad_form_kernel(ErrArgs a) {   // three workgroups per CU fit in LDS
  extern __shared__ double smem[];
  __shared__ double red[256];
  // column tiles have k ranges proportional to their index: the widest are dispatched
  // first (blockIdx.y is the slow grid index), the two quadratic forms share blockIdx.x
  const int nrt = gridDim.x >> 1;
  const int z = blockIdx.x / nrt;
  const int rt = blockIdx.x - z * nrt;
  const int ct = gridDim.y - 1 - blockIdx.y;
  const int i0 = rt * Tile::BM, j0 = ct * Tile::BN;
  const int j1 = min(j0 + Tile::BN, a.n);
  const int i1 = min(i0 + Tile::BM, a.m);
  const double* Az = a.A2 + (int64_t)z * a.m * a.n;
  f64x4 acc[TM][TN];
  dgemm_zero(acc);
  dgemm_mainloop<TM, TN, true, false>(
      acc, DView{Az + (int64_t)i0 * a.n, a.n, 1}, DgemmIdentity{},
      // H below the diagonal is read (it is valid memory) and discarded
      DView{a.H + j0, 1, a.ldh},
      [&](double h, int k, int j) { return k == j0 + j ? h : (k < j0 + j ? 2.0 * h : 0.0); },
      i1 - i0, j1 - j0, 0, j1, smem);
  double s = 0.0;
  dgemm_foreach(acc, [&](int i, int j, double v) {
    const bool ok = (i0 + i < a.m) & (j0 + j < a.n);
    const double d = Az[ok ? (int64_t)(i0 + i) * a.n + j0 + j : 0];
    s = fma(v, ok ? d : 0.0, s);
  });
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0)
    a.partial[((int64_t)z * nrt + rt) * gridDim.y + ct] = red[0];
}

// ---------------------------------------------------------------- bfloat16-split form
constexpr int kT = 128;         // tile edge: four waves, 64 x 64 each (2 x 2 tiles of the 32 x 32 x 16 MFMA)

// A number rounded to P bfloat16 pieces (8 significant bits each, each remainder taken after rounding
// to nearest) keeps 8 P significant bits, and the product of two bfloat16 numbers is exact in
// float32.  So A Hu is the sum of the piece products A_a Hu_b; those with a + b < P carry everything
// down to 2^(-8 P) of a term, the others are below what the pieces resolve.  They run on the bfloat16
// 32 x 32 x 16 MFMA, accumulate in float32, smallest pieces first.  W stored in bfloat16 is one piece.
// Three pieces are float32 arithmetic (six products for tr(D H D^T), three for tr(W H W^T) with W in
// bfloat16; the traces agree with the float64 definition to 1e-8, 3e-7 at worst).  With two pieces
// (three and two products, 0.56 of the matrix-core work) every term is off by up to 2^-16 of itself,
// unbiased and independent from term to term, and a trace adds m n of them: measured against the
// float64 oracle on layers of 1e5 .. 4.5e7 entries the traces differ by 3e-7 .. 1e-6 relative and the
// relative layer error by at most 1e-7, where the required agreement is 1e-4.  That rests on the
// averaging, so layers of fewer than kTwoPiecesFrom entries (where the time does not matter) take three.
constexpr int kMaxPieces = 3;
constexpr int64_t kTwoPiecesFrom = 65536;
constexpr int kSK = 32;        // k-tile of the split form
constexpr int kSP = kSK + 8;   // LDS pitch in elements: 80-byte rows keep the 16-byte fragment reads apart

__device__ __forceinline__ uint16_t bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_val(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
template <int P>
__device__ __forceinline__ void split(float x, uint16_t (&p)[P]) {
  float r = x;
#pragma unroll
  for (int q = 0; q < P; ++q) {
    p[q] = bf16_rne(r);
    r -= bf16_val(p[q]);
  }
}

struct SplitArgs {
  const uint16_t* D;   // [P][mp][np]: D = W - Wq as bfloat16 pieces; zero outside m x n
  const uint16_t* W;   // [1 or P][mp][np]: W likewise
  const uint16_t* HuT; // [P][np (j)][np (k)]: Hu transposed, as pieces; zero for k > j and outside n x n
  int mp, np;
  double* partial;     // [2][tiles]: the tile sums of tr(D H D^T), then those of tr(W H W^T)
};

// D and W as bfloat16 pieces, four consecutive k per thread
template <int DT, int P>
__global__ __launch_bounds__(256) void split_weights_kernel(const void* __restrict__ W, int64_t ldw,
                                                            const double* __restrict__ Wq, int m, int n, int mp, int np,
                                                            uint16_t* __restrict__ Dp, uint16_t* __restrict__ Wp) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= (int64_t)mp * np / 4) return;
  const int i = (int)(q / (np / 4)), k0 = (int)(q - (int64_t)i * (np / 4)) * 4;
  uint16_t d[4][P], w[4][P];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const bool ok = i < m && k0 + c < n;
    const double wv = ok ? load_as_f64<DT>(W, (int64_t)i * ldw + k0 + c) : 0.0;
    const double qv = ok ? Wq[(int64_t)i * n + k0 + c] : 0.0;
    split((float)(wv - qv), d[c]);
    split((float)wv, w[c]);
  }
  const int64_t plane = (int64_t)mp * np, at = (int64_t)i * np + k0;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    *reinterpret_cast<ushort4*>(Dp + p * plane + at) = ushort4{d[0][p], d[1][p], d[2][p], d[3][p]};
    if (DT != PTQ_BF16 || p == 0)
      *reinterpret_cast<ushort4*>(Wp + p * plane + at) = ushort4{w[0][p], w[1][p], w[2][p], w[3][p]};
  }
}

// Hu transposed, as pieces: 32 x 32 tiles through LDS so that both the reads of H and the writes run along rows
template <int P>
__global__ __launch_bounds__(256) void split_hu_kernel(const double* __restrict__ H, int64_t ldh, int n, int np,
                                                       uint16_t* __restrict__ HuT) {
  __shared__ uint16_t t[P][32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int j0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int k = k0 + ty + 8 * rr, j = j0 + tx;
    const bool ok = k < n && j < n && k <= j;
    const double h = ok ? H[(int64_t)k * ldh + j] : 0.0;
    uint16_t p[P];
    split((float)(k == j ? h : 2.0 * h), p);
#pragma unroll
    for (int q = 0; q < P; ++q) t[q][ty + 8 * rr][tx] = p[q];
  }
  __syncthreads();
  const int64_t plane = (int64_t)np * np;
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int j = j0 + ty + 8 * rr, k = k0 + tx;
#pragma unroll
    for (int q = 0; q < P; ++q) HuT[q * plane + (int64_t)j * np + k] = t[q][tx][ty + 8 * rr];
  }
}

// ND pieces of D and NW pieces of W against the NH pieces of Hu: both traces in one pass over Hu
// (<P, 1, P>: W stored in bfloat16), or one trace per launch (<P, 0, P>, <0, P, P>)
template <int ND, int NW, int NH>
__global__ __launch_bounds__(256) void quad_form_split_kernel(SplitArgs a) {
  extern __shared__ uint16_t sm[];   // [2 stages][ND + NW + NH pieces][128 rows][kSP]
  __shared__ double red[2][4];
  constexpr int NA = ND + NW, NP = NA + NH;
  constexpr int kPiece = kT * kSP, kStage = NP * kPiece;
  // the widest column tiles first (blockIdx.y is the slow grid index)
  const int rt = blockIdx.x, ct = gridDim.y - 1 - blockIdx.y;
  const int i0 = rt * kT, j0 = ct * kT;
  const int kend = j0 + kT;   // beyond it Hu is zero; a multiple of 128
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t planeA = (int64_t)a.mp * a.np, planeB = (int64_t)a.np * a.np;

  // a piece's 128 x 32 tile is 512 chunks of 16 bytes: two per thread.  Two register sets: a tile's
  // loads are issued three k-tiles ahead and have two whole k-tiles of MFMAs to arrive (one k-tile
  // of the bfloat16 MFMA is too short to cover the latency of a load from L2)
  const int lr = tid >> 2, lk = (tid & 3) * 8;
  const int64_t arow = (int64_t)(i0 + lr) * a.np + lk;
  const uint16_t* gb = a.HuT + (int64_t)(j0 + lr) * a.np + lk;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a native vector: stays in registers
  u32x4 reg[2][NP][2];
  auto fetch = [&](auto set, int k0) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const uint16_t* g = p < ND ? a.D + p * planeA + arow : (p < NA ? a.W + (p - ND) * planeA + arow : gb + (p - NA) * planeB);
      reg[S][p][0] = *reinterpret_cast<const u32x4*>(g + k0);
      reg[S][p][1] = *reinterpret_cast<const u32x4*>(g + (int64_t)64 * a.np + k0);
    }
  };
  auto stash = [&](auto set, int stage) {
    constexpr int S = decltype(set)::value;
    uint16_t* st = sm + stage * kStage;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      *reinterpret_cast<u32x4*>(st + p * kPiece + lr * kSP + lk) = reg[S][p][0];
      *reinterpret_cast<u32x4*>(st + p * kPiece + (lr + 64) * kSP + lk) = reg[S][p][1];
    }
  };

  constexpr int kForms = (ND > 0) + (NW > 0);
  f32x16 acc[kForms][2][2];
#pragma unroll
  for (int f = 0; f < kForms; ++f)
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
      for (int tn = 0; tn < 2; ++tn)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[f][tm][tn][r] = 0.f;

  // One k-tile: the products of the tile in LDS stage `stage`, with the next tile's way into the other stage
  // (registers of `set` -> LDS, then the loads of tile knext into the same registers) issued between them.
  // A wave is alone on its SIMD, so nothing hides what it waits for but its own MFMAs: the fragments of the
  // second k-step are read while the first k-step's products run, the LDS stores go out between them too,
  // and the global loads go out between the products of the second k-step.  Only the first k-step's
  // fragment reads, right after the barrier, are exposed.  The order is asked of the scheduler explicitly.
  struct Frags {
    bf16x8 a[NA][2], b[NH][2];
  };
  auto read_frags = [&](const uint16_t* st, int ks, Frags& f) {
    // fragment of a 32-row strip: lane l holds row l % 32, k = 8 (l / 32) .. + 7 of the 16-wide k-step
    const int fo = (lane & 31) * kSP + ks * 16 + (lane >> 5) * 8;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int p = 0; p < NA; ++p)
        f.a[p][t] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(st + p * kPiece + (wm * 64 + t * 32) * kSP + fo));
#pragma unroll
      for (int p = 0; p < NH; ++p)
        f.b[p][t] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(st + (NA + p) * kPiece + (wn * 64 + t * 32) * kSP + fo));
    }
  };
  // piece pa of an operand with piece pb of Hu for pa + pb < NH, the smallest products first
  auto multiply = [&](const Frags& f) {
#pragma unroll
    for (int order = NH - 1; order >= 0; --order)
#pragma unroll
      for (int p = 0; p < NA; ++p) {
        const int fr = (ND > 0 && p >= ND) ? 1 : 0;   // which trace the piece belongs to
        const int pa = p < ND ? p : p - ND;
        const int pb = order - pa;
        if (pb < 0 || pb >= NH) continue;
#pragma unroll
        for (int tm = 0; tm < 2; ++tm)
#pragma unroll
          for (int tn = 0; tn < 2; ++tn)
            acc[fr][tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[p][tm], f.b[pb][tn], acc[fr][tm][tn], 0, 0, 0);
      }
  };
  constexpr int kFull = NH * (NH + 1) / 2;   // products of an operand that has all its pieces
  constexpr int kMfma = 4 * ((ND ? kFull : 0) + (NW == NH ? kFull : (NW == 1 ? NH : 0)));   // MFMAs of one k-step
  constexpr int kMem = 2 * NP;                         // fragment reads = LDS stores = loads of a k-tile
  constexpr int kPer = kMfma / kMem, kRest = kMfma - kPer * kMem;   // MFMAs between two memory instructions
  static_assert(kSK == 32 && kPer >= 1, "two k-steps per tile; at least one MFMA between memory instructions");
  auto tile = [&](auto stage_c, auto set, int knext) {
    constexpr int STAGE = decltype(stage_c)::value;
    const uint16_t* st = sm + STAGE * kStage;
    Frags f0, f1;
    __builtin_amdgcn_sched_barrier(0);
    read_frags(st, 0, f0);
    read_frags(st, 1, f1);
    stash(set, STAGE ^ 1);
    multiply(f0);
    fetch(set, knext);
    multiply(f1);
    // the first k-step's fragments; then per kPer MFMAs one fragment read of the second k-step and one LDS
    // store; then per kPer MFMAs one global load
    __builtin_amdgcn_sched_group_barrier(0x100, kMem, 0);
#pragma unroll
    for (int i = 0; i < kMem; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, kPer, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
    }
    if constexpr (kRest > 0) __builtin_amdgcn_sched_group_barrier(0x008, kRest, 0);
#pragma unroll
    for (int i = 0; i < kMem; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, kPer, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    if constexpr (kRest > 0) __builtin_amdgcn_sched_group_barrier(0x008, kRest, 0);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
  };
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;
  using Stage0 = std::integral_constant<int, 0>;
  using Stage1 = std::integral_constant<int, 1>;

  // kend is a multiple of 128: an even number (at least four) of k-tiles.  The loop body has no
  // branch: a fetch beyond the last k-tile reads the last one again and a stash after the last
  // products fills a stage nobody reads.  With conditional fetches the compiler cannot count the
  // outstanding loads across the back edge and waits for all of them before every stash; as it
  // stands it waits for all but the newest set, and a tile's loads have two k-tiles to arrive.
  // (The prologue issues its loads in the loop's order, set 1 before the second set 0, and the
  // scheduling barriers keep it so: the wait counts at the loop head are the worse of the two ways in.)
  const int klast = kend - kSK;
  fetch(Set0{}, 0);
  __builtin_amdgcn_sched_barrier(0);
  fetch(Set1{}, kSK);
  __builtin_amdgcn_sched_barrier(0);
  stash(Set0{}, 0);
  __builtin_amdgcn_sched_barrier(0);
  fetch(Set0{}, 2 * kSK);
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  for (int k0 = 0; k0 < kend; k0 += 2 * kSK) {
    // tile k0 sits in stage 0; tile k0 + 32 goes from set 1 to stage 1, set 1 then takes tile k0 + 96
    tile(Stage0{}, Set1{}, min(k0 + 3 * kSK, klast));
    // tile k0 + 32 sits in stage 1; tile k0 + 64 goes from set 0 to stage 0, set 0 then takes tile k0 + 128
    tile(Stage1{}, Set0{}, min(k0 + 4 * kSK, klast));
  }

  // sum_ij A_ij T_ij of the tile in float64; accumulator r of a lane is row (r / 4) * 8 + (lane / 32) * 4 + r % 4,
  // column lane % 32 of its 32 x 32 tile; rows and columns beyond m x n hold zeros
  double s[kForms];
#pragma unroll
  for (int f = 0; f < kForms; ++f) {
    const bool is_w = (ND == 0) || f == 1;
    const uint16_t* P = is_w ? a.W : a.D;
    const int np_ = is_w ? NW : ND;
    s[f] = 0.0;
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
      for (int tn = 0; tn < 2; ++tn)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = wm * 64 + tm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          const int j = wn * 64 + tn * 32 + (lane & 31);
          const int64_t at = (int64_t)(i0 + i) * a.np + j0 + j;
          double v = (double)bf16_val(P[at]);
          for (int p = 1; p < np_; ++p) v += (double)bf16_val(P[p * planeA + at]);
          s[f] = fma((double)acc[f][tm][tn][r], v, s[f]);
        }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s[f] += __shfl_xor(s[f], off);
    if (lane == 0) red[f][wave] = s[f];
  }
  __syncthreads();
  if (tid == 0) {
    const int64_t tile = (int64_t)rt * gridDim.y + ct, tiles = (int64_t)gridDim.x * gridDim.y;
#pragma unroll
    for (int f = 0; f < kForms; ++f) {
      const bool is_w = (ND == 0) || f == 1;
      a.partial[(is_w ? tiles : 0) + tile] = (red[f][0] + red[f][1]) + (red[f][2] + red[f][3]);
    }
  }
}

__global__ __launch_bounds__(256) void finish_kernel(const double* __restrict__ partial, int tiles,
                                                     double* out) {
  __shared__ double red[2][256];
  for (int z = 0; z < 2; ++z) {
    double s = 0.0;
    for (int i = threadIdx.x; i < tiles; i += 256) s += partial[(int64_t)z * tiles + i];
    red[z][threadIdx.x] = s;
  }
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) {
      red[0][threadIdx.x] += red[0][threadIdx.x + w];
      red[1][threadIdx.x] += red[1][threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double num = red[0][0], den = red[1][0];
    out[0] = sqrt(num / den);
    out[1] = num;
    out[2] = den;
  }
}

}  // namespace

static size_t partial_bytes(int64_t m, int64_t n) {
  const size_t tiles = (size_t)ceil_div(m, Tile::BM) * (size_t)ceil_div(n, Tile::BN);
  return align_up(2 * tiles * sizeof(double), 256);
}

static size_t bytes_f64_form(int64_t m, int64_t n) {
  return partial_bytes(m, n) + align_up(2 * (size_t)m * (size_t)n * sizeof(double), 256);
}

static size_t partial_split_bytes(int64_t mp, int64_t np) {
  return align_up(2 * (size_t)(mp / kT) * (size_t)(np / kT) * sizeof(double), 256);
}

static size_t pieces_bytes(int64_t rows, int64_t cols) {
  return align_up(kMaxPieces * (size_t)rows * (size_t)cols * sizeof(uint16_t), 256);
}

static size_t bytes_split_form(int64_t m, int64_t n) {
  const int64_t mp = ceil_div(m, kT) * kT, np = ceil_div(n, kT) * kT;
  return partial_split_bytes(mp, np) + 2 * pieces_bytes(mp, np) + pieces_bytes(np, np);
}

// the caller asks before it says which storage type W has: enough for either form
size_t layer_error_workspace_bytes(int64_t m, int64_t n) {
  const size_t a = bytes_f64_form(m, n), b = bytes_split_form(m, n);
  return a > b ? a : b;
}

template <int ND, int NW, int NH>
static bool launch_split(const SplitArgs& a, hipStream_t st) {
  const int lds = 2 * (ND + NW + NH) * kT * kSP * (int)sizeof(uint16_t);
  if (!lds_opt_in<quad_form_split_kernel<ND, NW, NH>>(lds)) return false;
  quad_form_split_kernel<ND, NW, NH><<<dim3((unsigned)(a.mp / kT), (unsigned)(a.np / kT)), 256, lds, st>>>(a);
  return true;
}

static ptq_status launch_split_form(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m, int64_t n,
                                    const double* H, int64_t ldh, double* out, void* ws, hipStream_t st) {
  const int64_t mp = ceil_div(m, kT) * kT, np = ceil_div(n, kT) * kT;
  char* base = static_cast<char*>(ws);
  double* partial = reinterpret_cast<double*>(base);
  uint16_t* Dp = reinterpret_cast<uint16_t*>(base + partial_split_bytes(mp, np));
  uint16_t* Wp = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(Dp) + pieces_bytes(mp, np));
  uint16_t* HuT = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(Wp) + pieces_bytes(mp, np));
  const unsigned ga = (unsigned)ceil_div(mp * np / 4, 256);
  const dim3 gh((unsigned)(np / 32), (unsigned)(np / 32));
  const int tiles = (int)((mp / kT) * (np / kT));
  SplitArgs a{Dp, Wp, HuT, (int)mp, (int)np, partial};
  auto run = [&](auto pieces) -> bool {
    constexpr int P = decltype(pieces)::value;
    if (wdt == PTQ_F32)
      split_weights_kernel<PTQ_F32, P><<<ga, 256, 0, st>>>(W, ldw, Wq, (int)m, (int)n, (int)mp, (int)np, Dp, Wp);
    else
      split_weights_kernel<PTQ_BF16, P><<<ga, 256, 0, st>>>(W, ldw, Wq, (int)m, (int)n, (int)mp, (int)np, Dp, Wp);
    split_hu_kernel<P><<<gh, 256, 0, st>>>(H, ldh, (int)n, (int)np, HuT);
    if (wdt == PTQ_BF16) return launch_split<P, 1, P>(a, st);
    return launch_split<P, 0, P>(a, st) && launch_split<0, P, P>(a, st);
  };
  const bool ok = (m * n >= kTwoPiecesFrom) ? run(std::integral_constant<int, 2>{}) : run(std::integral_constant<int, 3>{});
  if (!ok) return PTQ_ERR_HIP;
  finish_kernel<<<1, 256, 0, st>>>(partial, tiles, out);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

ptq_status layer_error_launch(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m,
                              int64_t n, const double* H, int64_t ldh, double* out, void* ws,
                              size_t ws_bytes, hipStream_t st) {
  if (ws_bytes < layer_error_workspace_bytes(m, n)) return PTQ_ERR_WORKSPACE;
  if (wdt == PTQ_F32 || wdt == PTQ_BF16) return launch_split_form(W, wdt, ldw, Wq, m, n, H, ldh, out, ws, st);
  if (wdt != PTQ_F64) return PTQ_ERR_DTYPE;
  double* partial = static_cast<double*>(ws);
  double* A2 = reinterpret_cast<double*>(static_cast<char*>(ws) + partial_bytes(m, n));
  const unsigned wg = (unsigned)ceil_div(m * n, 256);
  widen_kernel<<<wg, 256, 0, st>>>(static_cast<const double*>(W), ldw, Wq, (int)m, (int)n, A2);
  ErrArgs a{A2, (int)m, (int)n, H, (int)ldh, partial};
  dim3 g(2 * (unsigned)ceil_div(m, Tile::BM), (unsigned)ceil_div(n, Tile::BN));
  const int tiles = (int)(g.x / 2 * g.y);
  constexpr int lds = Tile::kSmemDoubles * (int)sizeof(double);
  if (!lds_opt_in<quad_form_kernel>(lds)) return PTQ_ERR_HIP;
  quad_form_kernel<<<g, 256, lds, st>>>(a);
  finish_kernel<<<1, 256, 0, st>>>(partial, tiles, out);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
