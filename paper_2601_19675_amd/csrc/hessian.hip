// Proxy-Hessian accumulation  H += X^T X  (upper triangle), X tokens x channels.
//
// bf16 path.  Tokens are the contraction index and the slow axis of X, while
// the matrix cores want, per lane, eight consecutive k for ONE channel.  The
// tile is therefore staged in LDS exactly as it lies in memory ([token][channel])
// and transposed on the way to registers: a lane reads the dword holding
// channels (2p, 2p+1) for eight tokens and two byte-permutes per pair of tokens
// split it into the fragment of channel 2p and the fragment of channel 2p+1.
// Even channels feed one 32x32x16 MFMA tile, odd channels the next one, so the
// output rows/columns of a wave are an interleaving of its two tiles.  Both
// operands are built the same way, hence any k order inside a fragment cancels.
//
// Products of two bf16 numbers are exact in float32.  A workgroup accumulates
// its 128 x 128 tile in float32 over at most 8192 tokens and stores that
// partial tile; a second kernel adds the partial tiles into H in float64 in a
// fixed order, so the result is bit-reproducible from run to run.
//
// f32 path (small layers): float64 FMAs on a 64 x 64 tile, same partial scheme.
#include "common.h"

namespace ptq {
namespace {

constexpr int kTile = 128;      // bf16 macro tile (channels x channels)
constexpr int kKT = 32;         // tokens per LDS stage
constexpr int kPitch = kTile + 8;  // bf16 elements; 272-byte rows
constexpr int kMaxChunk = 8192;      // tokens summed in float32 before the float64 reduction
constexpr int kMaxChunkBig = 20480;  // ... in the 256 x 256-tile kernel (fewer, larger partial tiles)

constexpr int kTile32 = 64;     // f32-path tile
constexpr int kKT32 = 16;

__device__ __forceinline__ void tile_from_linear(int lin, int ntb, int& I, int& J) {
  // upper-triangular tile list, row by row: row I holds ntb - I tiles
  int i = 0;
  while (lin >= ntb - i) {
    lin -= ntb - i;
    ++i;
  }
  I = i;
  J = i + lin;
}

__global__ __launch_bounds__(256) void hessian_bf16_kernel(const uint16_t* __restrict__ X, int64_t ldx,
                                                           int64_t t, int n, int64_t tok0, int chunk,
                                                           int ntb, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) uint16_t As[kKT * kPitch];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[kKT * kPitch];
  int I, J;
  tile_from_linear(blockIdx.x, ntb, I, J);
  const bool diag = (I == J);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int64_t kbeg = tok0 + (int64_t)blockIdx.y * chunk;
  const int64_t kend = (kbeg + chunk < t) ? kbeg + chunk : t;

  // global -> LDS map: 16 threads cover one token row (8 channels = 16 bytes each)
  const int lrow = tid >> 4, lcol = (tid & 15) * 8;
  const bool a_in = (I * kTile + lcol) < n, b_in = (J * kTile + lcol) < n;
  const uint16_t* ga = X + I * kTile + lcol;
  const uint16_t* gb = X + J * kTile + lcol;

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  uint4 ra[2], rb[2];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int64_t k = k0 + lrow + 16 * p;
      const bool kin = k < kend;
      ra[p] = (kin && a_in) ? *reinterpret_cast<const uint4*>(ga + k * ldx) : uint4{0, 0, 0, 0};
      if (!diag) rb[p] = (kin && b_in) ? *reinterpret_cast<const uint4*>(gb + k * ldx) : uint4{0, 0, 0, 0};
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      *reinterpret_cast<uint4*>(&As[(lrow + 16 * p) * kPitch + lcol]) = ra[p];
      if (!diag) *reinterpret_cast<uint4*>(&Bs[(lrow + 16 * p) * kPitch + lcol]) = rb[p];
    }
  };
  // fragments of the even and the odd channels of a 64-channel strip
  auto fragments = [&](const uint16_t* T, int strip, int ks, bf16x8 (&f)[2]) {
    const int p = lane & 31, kg = lane >> 5;
    uint32_t d[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      d[i] = *reinterpret_cast<const uint32_t*>(&T[(ks * 16 + kg * 8 + i) * kPitch + strip * 64 + 2 * p]);
    uint32_t ev[4], od[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ev[i] = __builtin_amdgcn_perm(d[2 * i + 1], d[2 * i], 0x05040100u);
      od[i] = __builtin_amdgcn_perm(d[2 * i + 1], d[2 * i], 0x07060302u);
    }
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
    f[0] = __builtin_bit_cast(bf16x8, u32x4{ev[0], ev[1], ev[2], ev[3]});
    f[1] = __builtin_bit_cast(bf16x8, u32x4{od[0], od[1], od[2], od[3]});
  };

  if (kbeg < kend) {
    fetch(kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += kKT) {
      __syncthreads();
      stash();
      __syncthreads();
      if (k0 + kKT < kend) fetch(k0 + kKT);
      const uint16_t* Bt = diag ? As : Bs;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 fa[2], fb[2];
        fragments(As, wi, ks, fa);
        fragments(Bt, wj, ks, fb);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int b = 0; b < 2; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
      }
    }
  }

  float* out = partial + ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * (kTile * kTile);
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int il = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int jl = lane & 31;
        out[(wi * 64 + 2 * il + a) * kTile + wj * 64 + 2 * jl + b] = acc[a][b][r];
      }
}

// ---- large layers: 256 x 256 tile, each wave 128 x 128 (4 x 4 MFMA tiles) ------
// Same transposition trick with 8-byte LDS reads: a lane gets channels 4p..4p+3
// for eight tokens, four byte-permutes per token pair give the fragments of the
// channel classes c % 4 = 0..3, one class per MFMA tile.  A wave then issues 16
// MFMAs (512 matrix-pipe cycles) per 16 LDS reads, so LDS sits at about half of
// its bandwidth; accumulators fill the 256 AGPRs.  LDS is double-buffered with
// one barrier per 64 tokens; the global loads of tile t+2, the LDS stores of
// tile t+1 and the fragments of the next 16 tokens are issued between the MFMAs
// of the current 16 tokens.
constexpr int kBT = 256;
constexpr int kBP = kBT + 8;                       // 528-byte rows
constexpr int kBKT = 64;                           // tokens per LDS stage
constexpr int kBStage = 2 * kBKT * kBP;            // A and B, bf16 elements
constexpr size_t kBigLdsBytes = 2 * kBStage * sizeof(uint16_t);

template <bool diag>
__device__ __forceinline__ void big_tile(const uint16_t* __restrict__ X, int64_t ldx, int64_t t, int n,
                                         int64_t tok0, int chunk, int I, int J, int split,
                                         float* __restrict__ out, uint16_t* hs) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int64_t kbeg = tok0 + (int64_t)split * chunk;
  const int64_t kend = (kbeg + chunk < t) ? kbeg + chunk : t;
  typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  if (kbeg < kend) {
    // global -> LDS map: 32 threads cover one token row (8 channels = 16 bytes each),
    // eight rows per pass.  Rows past the end of the chunk re-read its last token
    // (pointer clamp, no branch) and are zeroed on the way into LDS.
    constexpr int kPass = kBKT / 8;
    const int lrow = tid >> 5, lcol = (tid & 31) * 8;
    const bool a_in = (I * kBT + lcol) < n, b_in = (J * kBT + lcol) < n;
    const uint16_t* ga = X + (kbeg + lrow) * ldx + (a_in ? I * kBT + lcol : 0);
    const uint16_t* gb = X + (kbeg + lrow) * ldx + (b_in ? J * kBT + lcol : 0);
    const uint16_t* la = X + (kend - 1) * ldx + (a_in ? I * kBT + lcol : 0);
    const uint16_t* lb = X + (kend - 1) * ldx + (b_in ? J * kBT + lcol : 0);
    const int64_t rstep = 8 * ldx;
    u32x4 ra[kPass], rb[kPass];
    auto fetch = [&]() {
#pragma unroll
      for (int p = 0; p < kPass; ++p) {
        const uint16_t* pa = ga + p * rstep;
        ra[p] = *reinterpret_cast<const u32x4*>(pa < la ? pa : la);
        if (!diag) {
          const uint16_t* pb = gb + p * rstep;
          rb[p] = *reinterpret_cast<const u32x4*>(pb < lb ? pb : lb);
        }
      }
      ga += kBKT * ldx;
      gb += kBKT * ldx;
    };
    auto stash = [&](int64_t k0, uint16_t* st) {
#pragma unroll
      for (int p = 0; p < kPass; ++p) {
        const bool kin = k0 + lrow + 8 * p < kend;
        const uint32_t ma = (kin && a_in) ? 0xffffffffu : 0u, mb = (kin && b_in) ? 0xffffffffu : 0u;
        *reinterpret_cast<u32x4*>(&st[(lrow + 8 * p) * kBP + lcol]) = ra[p] & ma;
        if (!diag) *reinterpret_cast<u32x4*>(&st[kBKT * kBP + (lrow + 8 * p) * kBP + lcol]) = rb[p] & mb;
      }
    };
    // fragments of the channel classes c % 4 of a 128-channel strip, tokens ks*16 + kg*8 .. +7
    auto fragments = [&](const uint16_t* T, int strip, int ks, bf16x8 (&f)[4]) {
      const int p = lane & 31, kg = lane >> 5;
      const uint16_t* src = T + (ks * 16 + kg * 8) * kBP + strip * 128 + 4 * p;
      uint2 d[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) d[i] = *reinterpret_cast<const uint2*>(src + i * kBP);
      u32x4 v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[0][i] = __builtin_amdgcn_perm(d[2 * i + 1].x, d[2 * i].x, 0x05040100u);
        v[1][i] = __builtin_amdgcn_perm(d[2 * i + 1].x, d[2 * i].x, 0x07060302u);
        v[2][i] = __builtin_amdgcn_perm(d[2 * i + 1].y, d[2 * i].y, 0x05040100u);
        v[3][i] = __builtin_amdgcn_perm(d[2 * i + 1].y, d[2 * i].y, 0x07060302u);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) f[q] = __builtin_bit_cast(bf16x8, v[q]);
    };
    auto mfma16 = [&](const bf16x8 (&fa)[4], const bf16x8 (&fb)[4]) {
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    };

    // stage s holds tile s; registers hold tile s+1 until it is stored
    fetch();
    stash(kbeg, hs);
    fetch();
    __syncthreads();
    int cur = 0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += kBKT) {
      const uint16_t* As = hs + cur * kBStage;
      const uint16_t* Bs = diag ? As : As + kBKT * kBP;
      bf16x8 fa[2][4], fb[2][4];
      fragments(As, wi, 0, fa[0]);
      fragments(Bs, wj, 0, fb[0]);
      // the next tile goes to the other stage, the one after that is requested;
      // past the end of the chunk both are harmless (clamped loads, zeroed rows)
      stash(k0 + kBKT, hs + (cur ^ 1) * kBStage);
      fetch();
#pragma unroll
      for (int ks = 0; ks < kBKT / 16; ++ks) {
        if (ks + 1 < kBKT / 16) {
          fragments(As, wi, ks + 1, fa[(ks + 1) & 1]);
          fragments(Bs, wj, ks + 1, fb[(ks + 1) & 1]);
        }
        mfma16(fa[ks & 1], fb[ks & 1]);
        // interleave: LDS reads of the next fragments first, then their permutes,
        // each group behind one MFMA so that the matrix pipe never waits for them
#pragma unroll
        for (int g = 0; g < 8; ++g) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
          __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);  // DS write (tile t+1)
          __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);  // VMEM read (tile t+2)
        }
#pragma unroll
        for (int g = 0; g < 8; ++g) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);  // VALU (permutes)
        }
      }
      __syncthreads();
      cur ^= 1;
    }
  }

#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int il = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int jl = lane & 31;
        out[(wi * 128 + 4 * il + a) * kBT + wj * 128 + 4 * jl + b] = acc[a][b][r];
      }
}

// Work order.  Workgroups are handed to the eight XCDs (each with its own L2)
// round-robin by workgroup id, so workgroup id = 8 * k + x is the k-th one of
// XCD x.  All (split, tile) items are laid out in one locality order -- split by
// split, and inside a split by super-tiles of 8 x 8 tiles -- and every XCD takes
// a contiguous eighth of that sequence: the 32 workgroups an XCD runs at a time
// then work on the same tokens of at most 16 channel strips, which its L2 serves.
constexpr int kSuper = 8;

__device__ __forceinline__ void tile_in_locality_order(int r, int ntb, int& I, int& J) {
  const int ns = (ntb + kSuper - 1) / kSuper;
  for (int a = 0; a < ns; ++a) {
    const int ha = min(kSuper, ntb - a * kSuper);
    for (int b = a; b < ns; ++b) {
      const int hb = min(kSuper, ntb - b * kSuper);
      const int cnt = (a == b) ? ha * (ha + 1) / 2 : ha * hb;
      if (r < cnt) {
        int i, j;
        if (a == b) {
          i = 0;
          while (r >= ha - i) {
            r -= ha - i;
            ++i;
          }
          j = i + r;
        } else {
          i = r / hb;
          j = r - i * hb;
        }
        I = a * kSuper + i;
        J = b * kSuper + j;
        return;
      }
      r -= cnt;
    }
  }
  I = J = 0;  // not reached
}

__global__ __launch_bounds__(256) void hessian_bf16_big_kernel(const uint16_t* __restrict__ X, int64_t ldx,
                                                               int64_t t, int n, int64_t tok0, int chunk,
                                                               int ntb, int ntiles, int nsplits,
                                                               float* __restrict__ partial) {
  extern __shared__ __attribute__((aligned(16))) uint16_t hs[];
  const int total = ntiles * nsplits;
  const int per_xcd = (total + 7) / 8;
  const int q = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (q >= total || (blockIdx.x >> 3) >= per_xcd) return;
  const int split = q / ntiles;
  int I, J;
  tile_in_locality_order(q - split * ntiles, ntb, I, J);
  const int lin = I * ntb - I * (I - 1) / 2 + (J - I);  // index in the row-major upper-triangular tile list
  float* out = partial + ((int64_t)split * ntiles + lin) * (kBT * kBT);
  if (I == J)
    big_tile<true>(X, ldx, t, n, tok0, chunk, I, J, split, out, hs);
  else
    big_tile<false>(X, ldx, t, n, tok0, chunk, I, J, split, out, hs);
}

// float32 activations: float64 FMAs, 64 x 64 tile, 4 x 4 outputs per thread.
__global__ __launch_bounds__(256) void hessian_f32_kernel(const float* __restrict__ X, int64_t ldx,
                                                          int64_t t, int n, int64_t tok0, int chunk,
                                                          int ntb, double* __restrict__ partial) {
  __shared__ double As[kKT32][kTile32 + 4];
  __shared__ double Bs[kKT32][kTile32 + 4];
  int I, J;
  tile_from_linear(blockIdx.x, ntb, I, J);
  const int tid = threadIdx.x;
  const int ty = tid >> 4, tx = tid & 15;
  const int64_t kbeg = tok0 + (int64_t)blockIdx.y * chunk;
  const int64_t kend = (kbeg + chunk < t) ? kbeg + chunk : t;
  double acc[4][4] = {};
  for (int64_t k0 = kbeg; k0 < kend; k0 += kKT32) {
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int e = tid + 256 * p;
      const int kk = e >> 6, c = e & 63;
      const int64_t k = k0 + kk;
      const int ca = I * kTile32 + c, cb = J * kTile32 + c;
      As[kk][c] = (k < kend && ca < n) ? (double)X[k * ldx + ca] : 0.0;
      Bs[kk][c] = (k < kend && cb < n) ? (double)X[k * ldx + cb] : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kKT32; ++kk) {
      double av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fma(av[i], bv[j], acc[i][j]);
    }
  }
  double* out = partial + ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * (kTile32 * kTile32);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) out[(ty * 4 + i) * kTile32 + tx * 4 + j] = acc[i][j];
}

// H[upper] += sum over splits of the partial tiles, in float64, fixed order.
template <class PT, int TILE>
__global__ __launch_bounds__(256) void hessian_reduce_kernel(const PT* __restrict__ partial, int splits,
                                                             int ntiles, int ntb, int n,
                                                             double* __restrict__ H, int64_t ldh) {
  int I, J;
  tile_from_linear(blockIdx.x, ntb, I, J);
  const int e = blockIdx.y * 256 + threadIdx.x;
  const int r = e / TILE, c = e % TILE;
  const int gi = I * TILE + r, gj = J * TILE + c;
  if (gi >= n || gj >= n || gi > gj) return;
  double s = 0.0;
  for (int sp = 0; sp < splits; ++sp)
    s += (double)partial[((int64_t)sp * ntiles + blockIdx.x) * (TILE * TILE) + e];
  H[(int64_t)gi * ldh + gj] += s;
}

struct Plan {
  int tile, ntb, ntiles, chunk, splits_total, splits_launch;
  size_t tile_bytes;
};

constexpr int64_t kBigFrom = 2048;                   // layers at least this wide use the 256-tile kernel
constexpr size_t kMaxPartialBytes = (size_t)1 << 30;  // partial tiles in flight per launch

Plan make_plan(int64_t n, int64_t t, ptq_dtype dt) {
  Plan p;
  const bool big = (dt == PTQ_BF16) && n >= kBigFrom;
  p.tile = (dt == PTQ_BF16) ? (big ? kBT : kTile) : kTile32;
  const int kt = (dt == PTQ_BF16) ? kKT : kKT32;
  p.ntb = (int)ceil_div(n, p.tile);
  p.ntiles = p.ntb * (p.ntb + 1) / 2;
  // Split the tokens so that the workgroups fill 256 CUs in whole rounds, with at most
  // max_chunk tokens summed in float32 by one workgroup: pick the split count with the
  // least (rounds x work per split).
  const int64_t max_chunk = big ? kMaxChunkBig : kMaxChunk;
  const int64_t s_min = ceil_div(t > 0 ? t : 1, max_chunk);
  int64_t best_s = s_min, best_cost = -1;
  for (int64_t sp = s_min; sp < s_min + 64; ++sp) {
    int64_t ch = ceil_div(ceil_div(t > 0 ? t : 1, sp), kt) * kt;
    if (ch < 256 && sp > s_min) break;
    // + 1024: writing and re-reading a partial tile costs about as much as 1024 tokens
    const int64_t cost = ceil_div(p.ntiles * sp, 256) * (ch + 1024);
    if (best_cost < 0 || cost < best_cost) {
      best_cost = cost;
      best_s = sp;
    }
  }
  int64_t chunk = ceil_div(ceil_div(t > 0 ? t : 1, best_s), kt) * kt;
  if (chunk < kt) chunk = kt;
  p.chunk = (int)chunk;
  p.splits_total = (int)ceil_div(t > 0 ? t : 1, chunk);
  p.tile_bytes = (size_t)p.tile * p.tile * ((dt == PTQ_BF16) ? sizeof(float) : sizeof(double));
  int64_t sl = big ? (int64_t)(kMaxPartialBytes / (p.tile_bytes * p.ntiles)) : ceil_div(2048, p.ntiles);
  if (sl > p.splits_total) sl = p.splits_total;
  if (sl < 1) sl = 1;
  p.splits_launch = (int)sl;
  return p;
}

}  // namespace

size_t hessian_workspace_bytes(int64_t n, int64_t t) {
  // sized for either input type
  const Plan a = make_plan(n, t, PTQ_BF16), b = make_plan(n, t, PTQ_F32);
  const size_t sa = a.tile_bytes * a.ntiles * a.splits_launch;
  const size_t sb = b.tile_bytes * b.ntiles * b.splits_launch;
  return align_up(sa > sb ? sa : sb, 256);
}

ptq_status hessian_launch(double* H, int64_t ldh, const void* X, ptq_dtype xdt, int64_t t, int64_t n,
                          int64_t ldx, void* ws, size_t ws_bytes, hipStream_t st) {
  if (t == 0 || n == 0) return PTQ_OK;
  const Plan p = make_plan(n, t, xdt);
  if (ws_bytes < p.tile_bytes * p.ntiles * p.splits_launch) return PTQ_ERR_WORKSPACE;
  for (int s0 = 0; s0 < p.splits_total; s0 += p.splits_launch) {
    const int ns = (p.splits_total - s0 < p.splits_launch) ? p.splits_total - s0 : p.splits_launch;
    const int64_t tok0 = (int64_t)s0 * p.chunk;
    dim3 g((unsigned)p.ntiles, (unsigned)ns);
    dim3 gr((unsigned)p.ntiles, (unsigned)(p.tile * p.tile / 256));
    if (xdt == PTQ_BF16 && p.tile == kBT) {
      static bool opted_in = false;
      if (!opted_in) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(hessian_bf16_big_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBigLdsBytes) != hipSuccess)
          return PTQ_ERR_HIP;
        opted_in = true;
      }
      const unsigned nwg = 8u * (unsigned)ceil_div((int64_t)p.ntiles * ns, 8);
      hessian_bf16_big_kernel<<<nwg, 256, kBigLdsBytes, st>>>(static_cast<const uint16_t*>(X), ldx, t, (int)n,
                                                              tok0, p.chunk, p.ntb, p.ntiles, ns,
                                                              static_cast<float*>(ws));
      hessian_reduce_kernel<float, kBT><<<gr, 256, 0, st>>>(static_cast<const float*>(ws), ns, p.ntiles,
                                                            p.ntb, (int)n, H, ldh);
    } else if (xdt == PTQ_BF16) {
      hessian_bf16_kernel<<<g, 256, 0, st>>>(static_cast<const uint16_t*>(X), ldx, t, (int)n, tok0, p.chunk,
                                             p.ntb, static_cast<float*>(ws));
      hessian_reduce_kernel<float, kTile><<<gr, 256, 0, st>>>(static_cast<const float*>(ws), ns, p.ntiles,
                                                              p.ntb, (int)n, H, ldh);
    } else {
      hessian_f32_kernel<<<g, 256, 0, st>>>(static_cast<const float*>(X), ldx, t, (int)n, tok0, p.chunk,
                                            p.ntb, static_cast<double*>(ws));
      hessian_reduce_kernel<double, kTile32><<<gr, 256, 0, st>>>(static_cast<const double*>(ws), ns,
                                                                 p.ntiles, p.ntb, (int)n, H, ldh);
    }
  }
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
