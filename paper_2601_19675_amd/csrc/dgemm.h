// Workgroup-level float64 tile GEMM on the gfx950 matrix cores.
//
// One workgroup of 256 threads (4 wavefronts arranged 2 x 2) produces a
// (32*TM) x (32*TN) tile of  sum_k A(i,k) * B(k,j)  with v_mfma_f64_16x16x4.
// Operands are strided views of float64 matrices, staged in LDS in a
// [k][i] / [k][j] layout, and consumed as 16x4 / 4x16 fragments:
//   A fragment: lane l holds A(i = l % 16, k = l / 16)
//   B fragment: lane l holds B(k = l / 16, j = l % 16)
//   D fragment: lane l, register r holds D(i = 4*r + l / 16, j = l % 16)
// (the D layout of the f64 instruction differs from the f32 ones; it was
// confirmed on hardware).  At 64 cycles per instruction the matrix pipe needs
// two doubles per lane per instruction, so plain 8-byte LDS reads keep it busy;
// what has to be kept small is everything else a wave issues, because a wave
// issues in order and with one wave per SIMD nothing else fills the gaps.
// Hence: per-thread element offsets are computed once and advanced by one add
// per k-tile, loads for tile t+2 are issued before the MFMAs of tile t, and
// LDS is double-buffered so that there is one barrier per k-tile.
#pragma once
#include <type_traits>

#include "common.h"

namespace ptq {

constexpr int kGemmBK = 16;

template <int TM, int TN>
struct DgemmTile {
  static constexpr int BM = 32 * TM;
  static constexpr int BN = 32 * TN;
  // LDS pitches (doubles): +2 spreads both the k-strided stores of a k-contiguous
  // operand and the four k-rows of a fragment read over all banks
  static constexpr int PA = BM + 2;
  static constexpr int PB = BN + 2;
  static constexpr int kStageDoubles = kGemmBK * (PA + PB);
  static constexpr int kSmemDoubles = 2 * kStageDoubles;
  static constexpr int EA = BM * kGemmBK / 256;  // elements per thread per k-tile
  static constexpr int EB = BN * kGemmBK / 256;
};

// element(o, k) = p[o * so + k * sk], o = row of A / column of B inside the tile.
// All offsets of one tile fit in 31 bits.
struct DView {
  const double* p;
  int so, sk;
};

struct DgemmIdentity {
  __device__ __forceinline__ double operator()(double v, int, int) const { return v; }
};

// fa(v, i, k) / fb(v, k, j) may transform a loaded value (tile-local i / j,
// absolute k); they run one k-tile after the load, just before the LDS store.
// `rows` x `cols` is the valid part of the tile, k runs over [kbeg, kend).
// KFAST says whether k is the contiguous index of the view (coalescing).
template <int TM, int TN, bool A_KFAST, bool B_KFAST, class FA, class FB>
__device__ __forceinline__ void dgemm_mainloop(f64x4 (&acc)[TM][TN], DView A, FA fa, DView B, FB fb, int rows,
                                               int cols, int kbeg, int kend, double* smem) {
  using T = DgemmTile<TM, TN>;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  if (kbeg >= kend) return;

  // fixed per-thread element coordinates and running offsets (at k-tile 0)
  int offa[T::EA], offb[T::EB];
  unsigned oka = 0, okb = 0;
#pragma unroll
  for (int p = 0; p < T::EA; ++p) {
    const int e = tid + 256 * p;
    const int i = A_KFAST ? e / kGemmBK : e % T::BM;
    const int k = A_KFAST ? e % kGemmBK : e / T::BM;
    oka |= (i < rows ? 1u : 0u) << p;
    offa[p] = (i < rows ? i : rows - 1) * A.so + (kbeg + k) * A.sk;
  }
#pragma unroll
  for (int p = 0; p < T::EB; ++p) {
    const int e = tid + 256 * p;
    const int j = B_KFAST ? e / kGemmBK : e % T::BN;
    const int k = B_KFAST ? e % kGemmBK : e / T::BN;
    okb |= (j < cols ? 1u : 0u) << p;
    offb[p] = (j < cols ? j : cols - 1) * B.so + (kbeg + k) * B.sk;
  }
  const int stepa = kGemmBK * A.sk, stepb = kGemmBK * B.sk;

  // Register sets for the k-tiles in flight.  The smallest tile has two loads per operand and thread and
  // a k-tile of four MFMAs per wave: with one k-tile in flight every iteration waits out a whole memory
  // latency (measured: 0.6 - 1.3 us per iteration where the MFMAs need 0.1), so it keeps four in flight.
  constexpr int D = (TM * TN == 1) ? 4 : 1;
  double ra[D][T::EA], rb[D][T::EB];
  // loads of the next k-tile in line (tiles are fetched in rising order; its offsets are the current
  // ones) into register set SET; only the last tile can stick out of [kbeg, kend): there the k index is clamped
  auto fetch = [&](auto set, int k0) {
    constexpr int SET = decltype(set)::value;
    if (k0 + kGemmBK <= kend) {
#pragma unroll
      for (int p = 0; p < T::EA; ++p) ra[SET][p] = A.p[offa[p]];
#pragma unroll
      for (int p = 0; p < T::EB; ++p) rb[SET][p] = B.p[offb[p]];
    } else {
#pragma unroll
      for (int p = 0; p < T::EA; ++p) {
        const int k = A_KFAST ? (tid + 256 * p) % kGemmBK : (tid + 256 * p) / T::BM;
        const int over = k0 + k - (kend - 1);
        ra[SET][p] = A.p[offa[p] - (over > 0 ? over : 0) * A.sk];
      }
#pragma unroll
      for (int p = 0; p < T::EB; ++p) {
        const int k = B_KFAST ? (tid + 256 * p) % kGemmBK : (tid + 256 * p) / T::BN;
        const int over = k0 + k - (kend - 1);
        rb[SET][p] = B.p[offb[p] - (over > 0 ? over : 0) * B.sk];
      }
    }
#pragma unroll
    for (int p = 0; p < T::EA; ++p) offa[p] += stepa;
#pragma unroll
    for (int p = 0; p < T::EB; ++p) offb[p] += stepb;
  };
  // the same for a tile known to lie inside [kbeg, kend): no branch
  auto fetch_inner = [&](auto set) {
    constexpr int SET = decltype(set)::value;
#pragma unroll
    for (int p = 0; p < T::EA; ++p) ra[SET][p] = A.p[offa[p]];
#pragma unroll
    for (int p = 0; p < T::EB; ++p) rb[SET][p] = B.p[offb[p]];
#pragma unroll
    for (int p = 0; p < T::EA; ++p) offa[p] += stepa;
#pragma unroll
    for (int p = 0; p < T::EB; ++p) offb[p] += stepb;
  };
  auto stash = [&](auto set, int k0, double* st) {
    constexpr int SET = decltype(set)::value;
    double* sa = st;
    double* sb = st + kGemmBK * T::PA;
#pragma unroll
    for (int p = 0; p < T::EA; ++p) {
      const int e = tid + 256 * p;
      const int i = A_KFAST ? e / kGemmBK : e % T::BM;
      const int k = A_KFAST ? e % kGemmBK : e / T::BM;
      const bool ok = ((oka >> p) & 1u) && (k0 + k < kend);
      const double v = fa(ra[SET][p], i, k0 + k);
      sa[k * T::PA + i] = ok ? v : 0.0;
    }
#pragma unroll
    for (int p = 0; p < T::EB; ++p) {
      const int e = tid + 256 * p;
      const int j = B_KFAST ? e / kGemmBK : e % T::BN;
      const int k = B_KFAST ? e % kGemmBK : e / T::BN;
      const bool ok = ((okb >> p) & 1u) && (k0 + k < kend);
      const double v = fb(rb[SET][p], k0 + k, j);
      sb[k * T::PB + j] = ok ? v : 0.0;
    }
  };

  // A tile with fewer than four MFMAs per k-step would run them as one dependent chain (an MFMA's
  // result is ready only three instruction times later): the k-steps of a k-tile then go to NS
  // separate accumulator sets, added up at the end.
  constexpr int NS = (TM * TN >= 4) ? 1 : 4 / (TM * TN);
  f64x4 part[NS][TM][TN];
  if constexpr (NS > 1) {
#pragma unroll
    for (int q = 0; q < NS; ++q)
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) part[q][tm][tn] = f64x4{0.0, 0.0, 0.0, 0.0};
  }
  // the MFMAs of the k-tile in LDS stage `stage`
  auto compute = [&](int stage) {
    const double* sa = smem + stage * T::kStageDoubles;
    const double* sb = sa + kGemmBK * T::PA;
    // fragments of k-step kk+1 are read while the MFMAs of k-step kk run (two register sets):
    // with few waves per SIMD nothing else would cover the LDS latency
    double a[2][TM], b[2][TN];
    auto frags = [&](int kk, int slot) {
      const int kr = kk + (lane >> 4);
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) a[slot][tm] = sa[kr * T::PA + wm * 16 * TM + tm * 16 + (lane & 15)];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) b[slot][tn] = sb[kr * T::PB + wn * 16 * TN + tn * 16 + (lane & 15)];
    };
    frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < kGemmBK; kk += 4) {
      const int slot = (kk >> 2) & 1;
      if (kk + 4 < kGemmBK) frags(kk + 4, slot ^ 1);
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
          if constexpr (NS == 1)
            acc[tm][tn] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[slot][tm], b[slot][tn], acc[tm][tn], 0, 0, 0);
          else
            part[(kk >> 2) % NS][tm][tn] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[slot][tm], b[slot][tn],
                                                                                part[(kk >> 2) % NS][tm][tn], 0, 0, 0);
        }
      __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);   // the reads of the next k-step first
      __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);   // then this k-step's MFMAs
    }
  };

  // Tile t is computed from LDS stage t % 2 while tile t + 1 goes from register set (t + 1) % D to the
  // other stage and tile t + 1 + D is requested into the set that has just been emptied.
  const int ntile = (kend - kbeg + kGemmBK - 1) / kGemmBK, nfull = (kend - kbeg) / kGemmBK;
  auto k_of = [&](int t) { return kbeg + t * kGemmBK; };
  using std::integral_constant;
  // prologue: tile 0 into stage 0, tiles 1 .. D requested
  fetch(integral_constant<int, 0>{}, k_of(0));
  stash(integral_constant<int, 0>{}, k_of(0), smem);
  {
    auto request = [&](auto dc) {
      constexpr int d = decltype(dc)::value;   // tile d + 1 into set (d + 1) % D
      if (d + 1 < ntile) fetch(integral_constant<int, (d + 1) % D>{}, k_of(d + 1));
    };
    request(integral_constant<int, 0>{});
    if constexpr (D > 1) request(integral_constant<int, 1>{});
    if constexpr (D > 2) request(integral_constant<int, 2>{});
    if constexpr (D > 3) request(integral_constant<int, 3>{});
    static_assert(D <= 4, "the prologue is written out for up to four sets");
  }
  __syncthreads();
  int t0 = 0;
  // steady state, D iterations per round, no branch inside: every tile stashed and requested is a full one
  // (the last request of a round is tile t0 + 2 D)
  auto round = [&](auto inner) {
    constexpr bool INNER = decltype(inner)::value;
    auto iter = [&](auto dc) {
      constexpr int d = decltype(dc)::value;
      const int t = t0 + d;
      using Set = integral_constant<int, (d + 1) % D>;
      if constexpr (INNER) {
        stash(Set{}, k_of(t + 1), smem + ((d + 1) & 1) * T::kStageDoubles);
        fetch_inner(Set{});
        compute(d & 1);
        __syncthreads();
      } else {
        if (t < ntile) {
          if (t + 1 < ntile) stash(Set{}, k_of(t + 1), smem + ((t + 1) & 1) * T::kStageDoubles);
          if (t + 1 + D < ntile) fetch(Set{}, k_of(t + 1 + D));
          compute(t & 1);
          __syncthreads();
        }
      }
    };
    iter(integral_constant<int, 0>{});
    if constexpr (D > 1) iter(integral_constant<int, 1>{});
    if constexpr (D > 2) iter(integral_constant<int, 2>{});
    if constexpr (D > 3) iter(integral_constant<int, 3>{});
  };
  if constexpr (D % 2 == 0) {   // (stage parity by d needs an even round)
    for (; t0 + 2 * D < nfull; t0 += D) round(integral_constant<bool, true>{});
  }
  for (; t0 < ntile; t0 += D) round(integral_constant<bool, false>{});
  if constexpr (NS > 1) {
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          double sum = part[0][tm][tn][r];
#pragma unroll
          for (int q = 1; q < NS; ++q) sum += part[q][tm][tn][r];
          acc[tm][tn][r] += sum;
        }
      }
  }
}

// ---- the same product for a tile that lies fully inside its operands, software-pipelined ----
// The loop above spends a quarter of its time outside the matrix pipe: per k-tile every wave first
// parks the next tile in LDS and requests the one after (address arithmetic, masks, sixteen loads and
// sixteen LDS stores in a row) and only then starts its MFMAs, and with one to three waves per SIMD
// nothing else fills that gap.  Here a tile with no ragged edge (all rows and columns valid, k range a
// multiple of the k-tile) takes a loop whose body is one scheduling region in which those
// instructions sit BETWEEN the MFMAs: operands come through buffer loads whose per-thread offsets
// never change (the k-tile advances in a scalar offset, so there is no address arithmetic), go to
// one of two register sets, and are written to the other LDS stage one k-tile later, a load or a
// store after every MFMA or two.  Summation order per output element is that of the loop above.
typedef __attribute__((__vector_size__(2 * sizeof(int)))) int dgemm_i32x2;

template <int I, int MM, int NV, int NW>
__device__ __forceinline__ void dgemm_sched_step() {
  // MM MFMAs; after MFMA I one buffer load while I < NV and one LDS store while I < NW
  if constexpr (I < MM) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr (I < NV) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    if constexpr (I < NW) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
    dgemm_sched_step<I + 1, MM, NV, NW>();
  }
}

template <int TM, int TN, bool A_KFAST, bool B_KFAST>
__device__ __forceinline__ void dgemm_mainloop_pipelined(f64x4 (&acc)[TM][TN], DView A, DView B, int kbeg, int kend,
                                                         double* smem) {
  using T = DgemmTile<TM, TN>;
  constexpr int EA = T::EA, EB = T::EB, E = EA + EB, MM = TM * TN;
  static_assert(E <= 2 * MM, "loads of a k-tile are spread over the MFMAs of its first two k-steps");
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int K = kend - kbeg;
  const int ntile = K / kGemmBK;
  if (ntile <= 0) return;

  // buffer resources based at the lowest address the tile touches (strides may be negative)
  const int64_t loa = (A.so < 0 ? (int64_t)(T::BM - 1) * A.so : 0) + (A.sk < 0 ? (int64_t)(K - 1) * A.sk : 0);
  const int64_t lob = (B.so < 0 ? (int64_t)(T::BN - 1) * B.so : 0) + (B.sk < 0 ? (int64_t)(K - 1) * B.sk : 0);
  const __amdgpu_buffer_rsrc_t ra_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<double*>(A.p + (int64_t)kbeg * A.sk + loa), 0, (int)0xFFFFFFFFu, 0x00020000);
  const __amdgpu_buffer_rsrc_t rb_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<double*>(B.p + (int64_t)kbeg * B.sk + lob), 0, (int)0xFFFFFFFFu, 0x00020000);
  int voa[EA], vob[EB], lda[EA], ldb[EB];
#pragma unroll
  for (int p = 0; p < EA; ++p) {
    const int e = tid + 256 * p;
    const int i = A_KFAST ? e / kGemmBK : e % T::BM;
    const int k = A_KFAST ? e % kGemmBK : e / T::BM;
    voa[p] = (i * A.so + k * A.sk - (A.so < 0 ? (T::BM - 1) * A.so : 0) - (A.sk < 0 ? (kGemmBK - 1) * A.sk : 0)) * 8;
    lda[p] = k * T::PA + i;
  }
#pragma unroll
  for (int p = 0; p < EB; ++p) {
    const int e = tid + 256 * p;
    const int j = B_KFAST ? e / kGemmBK : e % T::BN;
    const int k = B_KFAST ? e % kGemmBK : e / T::BN;
    vob[p] = (j * B.so + k * B.sk - (B.so < 0 ? (T::BN - 1) * B.so : 0) - (B.sk < 0 ? (kGemmBK - 1) * B.sk : 0)) * 8;
    ldb[p] = kGemmBK * T::PA + k * T::PB + j;
  }
  // scalar byte offset of the k-tile about to be requested
  int soa = (A.sk < 0 ? -(K - kGemmBK) * A.sk : 0) * 8, sob = (B.sk < 0 ? -(K - kGemmBK) * B.sk : 0) * 8;
  const int stepa = kGemmBK * A.sk * 8, stepb = kGemmBK * B.sk * 8;

  double ra[2][EA], rb[2][EB];
  auto request = [&](int set) {
#pragma unroll
    for (int p = 0; p < EA; ++p)
      ra[set][p] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(ra_rsrc, voa[p], soa, 0));
#pragma unroll
    for (int p = 0; p < EB; ++p)
      rb[set][p] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(rb_rsrc, vob[p], sob, 0));
    soa += stepa;
    sob += stepb;
  };
  auto park = [&](int set, int stage, int from, int to) {   // elements [from, to) of the E a thread holds
    double* st = smem + stage * T::kStageDoubles;
#pragma unroll
    for (int q = 0; q < E; ++q) {
      if (q >= from && q < to) {
        if (q < EA) st[lda[q]] = ra[set][q];
        else st[ldb[q - EA]] = rb[set][q - EA];
      }
    }
  };

  // P: LDS stage that holds the current k-tile (= register set the tile after next is requested into)
  auto body = [&](auto p_, auto load_, auto store_) {
    constexpr int P = decltype(p_)::value;
    constexpr bool LOAD = decltype(load_)::value, STORE = decltype(store_)::value;
    const double* sa = smem + P * T::kStageDoubles;
    const double* sb = sa + kGemmBK * T::PA;
    if constexpr (LOAD) request(P);
    double a[2][TM], b[2][TN];
    auto frags = [&](int kk, int slot) {
      const int kr = kk + (lane >> 4);
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) a[slot][tm] = sa[kr * T::PA + wm * 16 * TM + tm * 16 + (lane & 15)];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) b[slot][tn] = sb[kr * T::PB + wn * 16 * TN + tn * 16 + (lane & 15)];
    };
    frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < kGemmBK; kk += 4) {
      const int slot = (kk >> 2) & 1;
      if (kk + 4 < kGemmBK) frags(kk + 4, slot ^ 1);
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[slot][tm], b[slot][tn], acc[tm][tn], 0, 0, 0);
      if constexpr (STORE) {
        if (kk == 8) park(P ^ 1, P ^ 1, 0, E / 2);
        if (kk == 12) park(P ^ 1, P ^ 1, E / 2, E);
      }
    }
    // the order the scheduler is asked for: per k-step the fragment reads of the next one, then its MFMAs
    // with one request after each in the first two k-steps and one LDS store after each in the last two
    constexpr int NV0 = !LOAD ? 0 : (E < MM ? E : MM), NV1 = !LOAD ? 0 : E - NV0;
    constexpr int NW2 = !STORE ? 0 : E / 2, NW3 = !STORE ? 0 : E - E / 2;
    __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
    dgemm_sched_step<0, MM, NV0, 0>();
    __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
    dgemm_sched_step<0, MM, NV1, 0>();
    __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
    dgemm_sched_step<0, MM, 0, NW2>();
    dgemm_sched_step<0, MM, 0, NW3>();
    __syncthreads();
  };
  using std::integral_constant;
  using I0 = integral_constant<int, 0>;
  using I1 = integral_constant<int, 1>;
  using Yes = integral_constant<bool, true>;
  using No = integral_constant<bool, false>;

  // prologue: tile 0 into stage 0, tile 1 on its way into register set 1
  request(0);
  park(0, 0, 0, E);
  if (ntile > 1) request(1);
  __syncthreads();
  int t = 0;
  for (; t + 3 < ntile; t += 2) {
    body(I0{}, Yes{}, Yes{});
    body(I1{}, Yes{}, Yes{});
  }
  const int rest = ntile - t;
  if (rest == 3) {
    body(I0{}, Yes{}, Yes{});
    body(I1{}, No{}, Yes{});
    body(I0{}, No{}, No{});
  } else if (rest == 2) {
    body(I0{}, No{}, Yes{});
    body(I1{}, No{}, No{});
  } else {
    body(I0{}, No{}, No{});
  }
}

// Visit every accumulator element with its tile-local (i, j).
template <int TM, int TN, class FC>
__device__ __forceinline__ void dgemm_foreach(const f64x4 (&acc)[TM][TN], FC fc) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = wm * 16 * TM + tm * 16 + 4 * r + (lane >> 4);
        const int j = wn * 16 * TN + tn * 16 + (lane & 15);
        fc(i, j, acc[tm][tn][r]);
      }
}

template <int TM, int TN>
__device__ __forceinline__ void dgemm_zero(f64x4 (&acc)[TM][TN]) {
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = f64x4{0.0, 0.0, 0.0, 0.0};
}

}  // namespace ptq
