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
// float32 activations: hessian_f32.hip (float64 matrix cores, 64 x 64 or 128 x 128 tiles), same
// partial scheme with float64 partial tiles.
#include <type_traits>
#include <utility>

#include "common.h"

namespace ptq {
namespace {

constexpr int kTile = 128;      // bf16 macro tile (channels x channels)
constexpr int kKT = 32;         // tokens per LDS stage
constexpr int kPitch = kTile + 8;  // bf16 elements; 272-byte rows
constexpr int kMaxChunk = 8192;      // tokens summed in float32 before the float64 reduction
constexpr int kMaxChunkBig = 20480;  // ... in the 256 x 256-tile kernel (fewer, larger partial tiles)
constexpr int kMaxChunkHuge = 65536; // ... and once a split alone fills the chip several times over

constexpr int kTile32 = 64;          // float32 activations: tile of narrow layers
constexpr int kTile32Wide = 128;     // ... and from kWide32From channels on
constexpr int64_t kWide32From = 1024;
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
// The tile's operands go from global memory straight into LDS (buffer_load ... lds,
// 16 bytes per lane, no staging registers) as they lie in memory, [token][channel], into
// a ring of four 32-token stages.  The transposition to "eight consecutive tokens of one
// channel per lane" is done by the LDS itself: ds_read_b64_tr_b16 hands a lane four tokens
// of its channel, two such reads make one MFMA operand.  Per 16 tokens a wave issues 16
// of these reads and 16 MFMAs (32 cycles each), accumulators fill the 256 AGPRs.
//
// LDS layout of a stage: A part (32 token rows x 512 bytes) then B part.  A row holds 32
// chunks of 16 bytes (8 channels); chunk c of token row r sits at position c ^ swz(r & 3),
// which spreads the 16 chunks a half-wave reads (four token rows x 64 bytes) over all
// banks.  A DMA instruction writes 64 consecutive chunks (two token rows) in lane order, so
// the swizzle is applied on the global side: lane j of the instruction fetches the chunk
// that belongs at position j & 31.
//
// Tokens past the end of the chunk are never fetched: the buffer descriptor ends with the
// chunk and out-of-range lanes deliver zeros.  Channels past n (last tile row / column
// only) fetch some valid channel instead; the outputs they feed lie outside the matrix and
// are dropped by the reduction.
//
// The DMA requests are issued by inline assembly and tracked with explicit vmcnt waits:
// the compiler would otherwise wait for every outstanding request before each LDS read.
constexpr int kBT = 256;
constexpr int kBKS = 32;                          // tokens per stage
constexpr int kBRing = 4;                         // stages in LDS
constexpr int kBRow = kBT * 2;                    // bytes per token row of a part
constexpr int kBPart = kBKS * kBRow;              // 16 KB
constexpr int kBStage = 2 * kBPart;               // 32 KB
constexpr size_t kBigLdsBytes = (size_t)kBRing * kBStage;  // 128 KB

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short i16x4;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;

__device__ __forceinline__ int swz(int row) { return ((row & 1) * 10) | ((row & 2) * 2); }

// One request: 64 lanes x 16 bytes from (descriptor base + voff) to LDS address ldsaddr + 16 * lane.
// (m0 is not otherwise used in this kernel: no indirect register indexing, no other LDS DMA.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(i32x4 rsrc, uint32_t voff, uint32_t ldsaddr) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(ldsaddr), "v"(voff), "s"(rsrc)
               : "memory", "m0");
}

// The same with the LDS address as a scalar base plus a compile-time offset: one scalar instruction per request
// instead of an add into a temporary and a move.
template <uint32_t OFFSET>
__device__ __forceinline__ void dma16_at(i32x4 rsrc, uint32_t voff, uint32_t ldsbase) {
  asm volatile("s_add_u32 m0, %0, %3\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(ldsbase), "v"(voff), "s"(rsrc),
               "n"(OFFSET)
               : "memory", "m0", "scc");
}

#pragma clang diagnostic pop

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  // s_waitcnt vmcnt(N); the other counters at their maximum (no wait)
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>)
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <bool diag>
__device__ __forceinline__ void big_tile(const uint16_t* __restrict__ X, int64_t ldx, int64_t t, int n,
                                         int64_t tok0, int chunk, int I, int J, int split,
                                         float* __restrict__ out, uint16_t* hs) {
  typedef __attribute__((address_space(3))) char lds_char;
  typedef __attribute__((address_space(3))) i16x4 lds_i16x4;
  lds_char* lds = (lds_char*)hs;
  const uint32_t lbase = (uint32_t)(uintptr_t)lds;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave >> 1, wj = wave & 1;
  const int64_t kbeg = tok0 + (int64_t)split * chunk;
  const int64_t kend = (kbeg + chunk < t) ? kbeg + chunk : t;
  const int64_t len = kend - kbeg;

  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  if (len > 0) {
    const int nstage = (int)((len + kBKS - 1) / kBKS);
    constexpr int L = diag ? 4 : 8;  // DMA instructions per stage and wave

    // descriptor over the chunk's tokens (uniform, kept in scalar registers)
    const uint64_t gb0 = (uint64_t)(X + kbeg * ldx);
    i32x4 rs = {(int)__builtin_amdgcn_readfirstlane((uint32_t)gb0),
                (int)__builtin_amdgcn_readfirstlane((uint32_t)(gb0 >> 32)),
                (int)__builtin_amdgcn_readfirstlane((uint32_t)(len * ldx * 2)),  // bytes, < 2^32 (host)
                0x00020000};
    const uint32_t stage_step = __builtin_amdgcn_readfirstlane((uint32_t)(kBKS * ldx * 2));

    // per-lane byte offsets of the four DMA instructions of a part, inside a stage (the descriptor advances)
    uint32_t voA[4], voB[4];
    {
      const int pos = lane & 31;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 8 * i + 2 * wave + (lane >> 5);
        const int c = pos ^ swz(row);
        int colA = I * kBT + 8 * c, colB = J * kBT + 8 * c;
        if (colA >= n) colA = I * kBT;
        if (colB >= n) colB = J * kBT;
        voA[i] = (uint32_t)((row * ldx + colA) * 2);
        voB[i] = (uint32_t)((row * ldx + colB) * 2);
      }
    }
    // per-lane LDS read addresses inside a stage, one per MFMA tile of the wave's strips
    uint32_t adA[4], adB[4];
    {
      const int g = lane >> 4, h = g & 1, kg = g >> 1, j = lane & 15, r = j >> 2, q = j & 3;
      const int row = kg * 8 + r;
#pragma unroll
      for (int T = 0; T < 4; ++T) {
        const int cA = wi * 16 + T * 4 + 2 * h + (q >> 1);
        const int cB = wj * 16 + T * 4 + 2 * h + (q >> 1);
        adA[T] = row * kBRow + ((cA ^ swz(r)) * 16) + (q & 1) * 8;
        adB[T] = (diag ? 0 : kBPart) + row * kBRow + ((cB ^ swz(r)) * 16) + (q & 1) * 8;
      }
    }
    // fragment of eight tokens: rows +0..3 and +4..7 relative to the lane's row
    auto read_one = [&](uint32_t addr) -> bf16x8 {
      const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(lds + addr));
      const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(lds + addr + 4 * kBRow));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // DMA instruction q of a stage (A rows first, then B rows) into the slot at dst
    auto dma_q = [&](int q, uint32_t dst) {
      if (q < 4) dma16(rs, voA[q], dst + q * 4096);
      else dma16(rs, voB[q - 4], dst + kBPart + (q - 4) * 4096);
    };
    // One stage on: the descriptor moves (base up, extent down, never below zero -- past the end of the chunk every
    // lane is out of range and delivers zeros), the per-lane offsets stay.  Scalar work, where advancing the
    // eight per-lane offsets costs the wave eight vector instructions per stage.
    auto dma_advance = [&]() {
      const uint64_t base = (((uint64_t)(uint32_t)rs[1] << 32) | (uint32_t)rs[0]) + stage_step;
      const uint32_t extent = (uint32_t)rs[2];
      // (readfirstlane: the compiler forms the saturating difference in a vector register, and the descriptor
      // operand of the requests has to be scalar)
      rs[0] = (int)__builtin_amdgcn_readfirstlane((uint32_t)base);
      rs[1] = (int)__builtin_amdgcn_readfirstlane((uint32_t)(base >> 32));
      rs[2] = (int)__builtin_amdgcn_readfirstlane(extent > stage_step ? extent - stage_step : 0u);
    };
    // 16 MFMAs on (fa, fb) while the next fragments (na, nb) are read at `so`.  L/2 DMA
    // instructions, q0 onwards, go between the four groups of four MFMAs: issued in one
    // burst they fill the memory pipeline's queue and the wave (hence its MFMAs) stalls.
    // ROLE: 0 = the wave's whole 128 x 128 quadrant; on a diagonal tile 1 = only the MFMA
    // tiles on or above the diagonal (the quadrant is itself a diagonal block of H),
    // 2 = nothing (the quadrant lies below the diagonal; the wave only moves data).
    auto half = [&](auto role, const bf16x8 (&fa)[4], const bf16x8 (&fb)[4], bf16x8 (&na)[4], bf16x8 (&nb)[4],
                    uint32_t so, int q0, uint32_t dst) {
      constexpr int ROLE = decltype(role)::value;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if (ROLE != 2) {
          na[g] = read_one(so + adA[g]);
          nb[g] = read_one(so + adB[g]);
#pragma unroll
          for (int b = (ROLE == 1 ? g : 0); b < 4; ++b)
            acc[g][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[g], fb[b], acc[g][b], 0, 0, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // DS read
          if (ROLE == 0 || g < 3) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          if (ROLE == 0 || g < 2) __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (L == 8) dma_q(q0 + g, dst);
        else if (g & 1) dma_q(q0 + (g >> 1), dst);
        __builtin_amdgcn_sched_barrier(0);
      }
    };

    // prologue: stages 0, 1, 2 and the first half of stage 3 are requested; stage 0 must have
    // landed.  Stages past the end of the chunk are requested like the others and deliver zeros.
#pragma unroll
    for (int s = 0; s < kBRing - 1; ++s) {
#pragma unroll
      for (int q = 0; q < L; ++q) dma_q(q, lbase + s * kBStage + wave * 1024);
      dma_advance();
    }
#pragma unroll
    for (int q = 0; q < L / 2; ++q) dma_q(q, lbase + (kBRing - 1) * kBStage + wave * 1024);
    wait_vmcnt<2 * L + L / 2>();
    __builtin_amdgcn_s_barrier();

    // Iteration s: tokens 0..15 of stage s | barrier | tokens 16..31.  At the barrier every wave
    // has finished reading stage s, so its slot is refilled with stage s + 4: the first half of
    // those DMA instructions is spread over the second half of iteration s, the rest over the
    // first half of iteration s + 1.  In issue order the requests outstanding at the barrier are
    // those of stages s+1, s+2, s+3, and stage s+1 is the one that must have landed.
    // The same half with the ring slot known at compile time: SO (LDS offset of the tokens to read) folds into the
    // immediate offset of the LDS reads -- from a second set of per-lane addresses, 64 KB further on, for the upper
    // two slots, since the immediate has 16 bits -- and DST (slot being refilled) into the immediate of the request's
    // scalar add.  With a run-time slot every pair of reads and every request needs an add of its own, and this
    // loop is bound by what a wave issues besides its MFMAs.
    uint32_t hiA[4], hiB[4];
#pragma unroll
    for (int T = 0; T < 4; ++T) {
      hiA[T] = adA[T] + 65536u;
      hiB[T] = adB[T] + 65536u;
      // (opaque to the compiler, or it forms them again before every use instead of keeping eight registers)
      asm volatile("" : "+v"(hiA[T]), "+v"(hiB[T]));
    }
    const uint32_t wbase = lbase + wave * 1024;
    auto half_at = [&](auto role, auto so_, auto q0_, auto dst_, const bf16x8 (&fa)[4], const bf16x8 (&fb)[4],
                       bf16x8 (&na)[4], bf16x8 (&nb)[4]) {
      constexpr int ROLE = decltype(role)::value;
      constexpr uint32_t SO = decltype(so_)::value, DST = decltype(dst_)::value;
      constexpr int Q0 = decltype(q0_)::value;
      constexpr bool HI = SO >= 65536u;
      constexpr uint32_t so = HI ? SO - 65536u : SO;
      static_for<4>([&](auto g_) {
        constexpr int g = decltype(g_)::value;
        if constexpr (ROLE != 2) {
          na[g] = read_one(so + (HI ? hiA[g] : adA[g]));
          nb[g] = read_one(so + (HI ? hiB[g] : adB[g]));
#pragma unroll
          for (int b = (ROLE == 1 ? g : 0); b < 4; ++b)
            acc[g][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[g], fb[b], acc[g][b], 0, 0, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // DS read
          if (ROLE == 0 || g < 3) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          if (ROLE == 0 || g < 2) __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (L == 8 || (g & 1)) {
          constexpr int q = (L == 8) ? Q0 + g : Q0 + (g >> 1);
          if constexpr (q < 4) dma16_at<DST + q * 4096>(rs, voA[q], wbase);
          else dma16_at<DST + kBPart + (q - 4) * 4096>(rs, voB[q - 4], wbase);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    };

    // Iteration s: tokens 0..15 of stage s | barrier | tokens 16..31.  At the barrier every wave
    // has finished reading stage s, so its slot is refilled with stage s + 4: the first half of
    // those DMA instructions is spread over the second half of iteration s, the rest over the
    // first half of iteration s + 1.  In issue order the requests outstanding at the barrier are
    // those of stages s+1, s+2, s+3, and stage s+1 is the one that must have landed.
    // Four iterations per trip of the loop, one per ring slot; what is left over (the number of stages
    // is not a multiple of four) takes the form with a run-time slot.
    auto main_loop = [&](auto role) {
      constexpr int ROLE = decltype(role)::value;
      using std::integral_constant;
      bf16x8 fa0[4], fb0[4], fa1[4], fb1[4];
      if (ROLE != 2) {
#pragma unroll
        for (int T = 0; T < 4; ++T) {
          fa0[T] = read_one(adA[T]);
          fb0[T] = read_one(adB[T]);
        }
      }
      auto iteration_at = [&](auto slot_) {
        constexpr uint32_t SLOT = decltype(slot_)::value;
        constexpr uint32_t slot_off = SLOT * kBStage, pend_off = ((SLOT + kBRing - 1) & (kBRing - 1)) * kBStage,
                           next_off = ((SLOT + 1) & (kBRing - 1)) * kBStage;
        half_at(role, integral_constant<uint32_t, slot_off + 16 * kBRow>{}, integral_constant<int, L / 2>{},
                integral_constant<uint32_t, pend_off>{}, fa0, fb0, fa1, fb1);
        dma_advance();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wait_vmcnt<2 * L>();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        half_at(role, integral_constant<uint32_t, next_off>{}, integral_constant<int, 0>{},
                integral_constant<uint32_t, slot_off>{}, fa1, fb1, fa0, fb0);
      };
      int s = 0;
      for (; s + kBRing <= nstage; s += kBRing) {
        iteration_at(integral_constant<uint32_t, 0>{});
        iteration_at(integral_constant<uint32_t, 1>{});
        iteration_at(integral_constant<uint32_t, 2>{});
        iteration_at(integral_constant<uint32_t, 3>{});
      }
      for (; s < nstage; ++s) {
        const uint32_t slot_off = (s & (kBRing - 1)) * kBStage;
        const uint32_t pend_off = ((s + kBRing - 1) & (kBRing - 1)) * kBStage;
        const uint32_t next_off = ((s + 1) & (kBRing - 1)) * kBStage;
        half(role, fa0, fb0, fa1, fb1, slot_off + 16 * kBRow, L / 2, lbase + pend_off + wave * 1024);
        dma_advance();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wait_vmcnt<2 * L>();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        half(role, fa1, fb1, fa0, fb0, next_off, 0, lbase + slot_off + wave * 1024);
      }
    };
    if (!diag || wave == 1)
      main_loop(std::integral_constant<int, 0>{});
    else if (wave == 2)
      main_loop(std::integral_constant<int, 2>{});
    else
      main_loop(std::integral_constant<int, 1>{});
    wait_vmcnt<0>();  // nothing may still be landing in LDS when the workgroup ends
  }

#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int il = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int jl = lane & 31;
        out[(wi * 128 + 32 * a + il) * kBT + wj * 128 + 32 * b + jl] = acc[a][b][r];
      }
}

// Work order.  Workgroups are handed to the eight XCDs (each with its own L2) round-robin by
// workgroup id.  All (split, tile) items are laid out in one locality order -- split by split,
// and inside a split by super-tiles of 8 x 8 tiles.  The 256 workgroups in flight take 256
// consecutive items, and of those XCD x (ids = x mod 8) takes 32 consecutive ones: its L2 then
// serves a few channel strips over the same tokens, and the memory-side cache serves what the
// XCDs share (the same one or two splits, at most two slabs of tokens x n).
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
  const int q = 256 * (blockIdx.x >> 8) + 32 * (blockIdx.x & 7) + ((blockIdx.x & 255) >> 3);
  if (q >= total) return;
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

// H[upper] += sum over splits of the partial tiles, in float64, fixed order.  Four consecutive
// elements of a tile row per thread (TILE is a multiple of 4, so they share the row).
template <class PT, int TILE>
__global__ __launch_bounds__(256) void hessian_reduce_kernel(const PT* __restrict__ partial, int splits,
                                                             int ntiles, int ntb, int n,
                                                             double* __restrict__ H, int64_t ldh) {
  int I, J;
  tile_from_linear(blockIdx.x, ntb, I, J);
  const int e = (blockIdx.y * 256 + threadIdx.x) * 4;
  const int r = e / TILE, c = e % TILE;
  const int gi = I * TILE + r, gj = J * TILE + c;
  if (gi >= n || gj >= n || gi > gj + 3) return;
  double s[4] = {0.0, 0.0, 0.0, 0.0};
  for (int sp = 0; sp < splits; ++sp) {
    const PT* src = partial + ((int64_t)sp * ntiles + blockIdx.x) * (TILE * TILE) + e;
    PT v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = src[q];
#pragma unroll
    for (int q = 0; q < 4; ++q) s[q] += (double)v[q];
  }
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (gj + q < n && gi <= gj + q) H[(int64_t)gi * ldh + gj + q] += s[q];
}

struct Plan {
  int tile, ntb, ntiles, chunk, splits_total, splits_launch;
  size_t tile_bytes;
};

constexpr int64_t kBigFrom = 2048;                   // layers at least this wide use the 256-tile kernel
constexpr size_t kMaxPartialBytes = (size_t)1 << 30;  // partial tiles in flight per launch

// The 256-tile kernel addresses a chunk of tokens (and the ring's read-ahead past it) with
// 32-bit byte offsets, which bounds the row pitch.
bool big_kernel_fits(int64_t ldx) {
  return (kMaxChunkHuge + (kBRing + 1) * kBKS) * ldx * 2 < ((int64_t)1 << 32);
}

Plan make_plan(int64_t n, int64_t t, ptq_dtype dt, bool allow_big) {
  Plan p;
  const bool big = allow_big && (dt == PTQ_BF16) && n >= kBigFrom;
  p.tile = (dt == PTQ_BF16) ? (big ? kBT : kTile) : (n >= kWide32From ? kTile32Wide : kTile32);
  const int kt = (dt == PTQ_BF16) ? kKT : kKT32;
  p.ntb = (int)ceil_div(n, p.tile);
  p.ntiles = p.ntb * (p.ntb + 1) / 2;
  // Split the tokens so that the workgroups fill 256 CUs in whole rounds, with at most
  // max_chunk tokens summed in float32 by one workgroup: pick the split count with the
  // least (rounds x work per split).
  // (with >= 512 tiles the rounds are full for any split count, so longer float32 sums buy fewer partial tiles)
  const int64_t max_chunk = big ? (p.ntiles >= 512 ? kMaxChunkHuge : kMaxChunkBig) : kMaxChunk;
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
  // sized for either input type and either bf16 kernel
  size_t need = 0;
  for (int v = 0; v < 3; ++v) {
    const Plan p = make_plan(n, t, v == 2 ? PTQ_F32 : PTQ_BF16, v == 0);
    const size_t b = p.tile_bytes * p.ntiles * p.splits_launch;
    if (b > need) need = b;
  }
  return align_up(need, 256);
}

ptq_status hessian_launch(double* H, int64_t ldh, const void* X, ptq_dtype xdt, int64_t t, int64_t n,
                          int64_t ldx, void* ws, size_t ws_bytes, hipStream_t st) {
  if (t == 0 || n == 0) return PTQ_OK;
  const Plan p = make_plan(n, t, xdt, big_kernel_fits(ldx));
  if (ws_bytes < p.tile_bytes * p.ntiles * p.splits_launch) return PTQ_ERR_WORKSPACE;
  for (int s0 = 0; s0 < p.splits_total; s0 += p.splits_launch) {
    const int ns = (p.splits_total - s0 < p.splits_launch) ? p.splits_total - s0 : p.splits_launch;
    const int64_t tok0 = (int64_t)s0 * p.chunk;
    dim3 g((unsigned)p.ntiles, (unsigned)ns);
    dim3 gr((unsigned)p.ntiles, (unsigned)(p.tile * p.tile / 1024));
    if (xdt == PTQ_BF16 && p.tile == kBT) {
      if (!lds_opt_in<hessian_bf16_big_kernel>((int)kBigLdsBytes)) return PTQ_ERR_HIP;
      const unsigned nwg = 256u * (unsigned)ceil_div((int64_t)p.ntiles * ns, 256);
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
      if (!hessian_f32_partials_launch(static_cast<const float*>(X), ldx, t, (int)n, tok0, p.chunk, p.ntb, p.tile, g,
                                       static_cast<double*>(ws), st))
        return PTQ_ERR_HIP;
      if (p.tile == kTile32Wide)
        hessian_reduce_kernel<double, kTile32Wide><<<gr, 256, 0, st>>>(static_cast<const double*>(ws), ns,
                                                                       p.ntiles, p.ntb, (int)n, H, ldh);
      else
        hessian_reduce_kernel<double, kTile32><<<gr, 256, 0, st>>>(static_cast<const double*>(ws), ns,
                                                                   p.ntiles, p.ntb, (int)n, H, ldh);
    }
  }
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
