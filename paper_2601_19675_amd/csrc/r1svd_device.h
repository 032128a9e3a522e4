// Device helpers and constants shared by the translation units of the scaled rank-one sketching
// loop (r1svd.hip: activation scale, the float32 forms, the host entry; r1svd_bf16.hip: the forms
// that work on a bfloat16 weight as it is).
#pragma once
#include "common.h"

#include <climits>

namespace ptq {
namespace r1svd_detail {

constexpr int kComputeUnits = 256;
constexpr int kChainThreads = 512;
constexpr int kMaxColumns = 32768;
constexpr int kReduceCols = 16;                   // columns per workgroup of the partial-vector sum
constexpr int kReduceGroups = 64;                 // partial vectors in flight per column
constexpr int kMaxNormParts = kMaxColumns / kReduceCols;
static_assert(kReduceCols * 4 == kWave, "the last step of the sum pairs four lanes per column");

constexpr int kMaxStreamRank = 16;          // ranks the bfloat16 forms keep corrections for
constexpr int kMaxStreamColumns = 16384;    // columns they take
constexpr int kResidentRows = 512, kResidentCols = 1024;   // words per workgroup in the resident form's upart, zpart
constexpr size_t kShareWords = (size_t)kMaxStreamRank * kComputeUnits * 2;   // one buffer of its cpart or dpart
// resident form: two buffers each of tagged partial u, partial z and the two tables of dot products
constexpr size_t kResidentUpartBytes = (size_t)2 * kComputeUnits * kResidentRows * sizeof(unsigned long long);
constexpr size_t kResidentZpartBytes = (size_t)2 * kComputeUnits * kResidentCols * sizeof(unsigned long long);
constexpr size_t kResidentShareBytes = (size_t)2 * kShareWords * sizeof(unsigned long long);
constexpr size_t kResidentWorkspaceBytes = kResidentUpartBytes + kResidentZpartBytes + 2 * kResidentShareBytes;

// ---- small floating point formats --------------------------------------------------------
// Nearest value with MANT explicit mantissa bits and smallest normal exponent EMIN, ties to
// even, as the integer  (biased exponent << MANT) + mantissa  (subnormals: the bare mantissa);
// the caller adds the sign and handles overflow.  Exact: only scalings by powers of two and
// one rint.
template <int MANT, int EMIN>
__device__ __forceinline__ int small_float_code(double a) {
  if (a == 0.0) return 0;
  int e = ilogb(a);
  e = e < EMIN ? EMIN : e;
  const double r = rint(scalbn(a, MANT - e));     // in [0, 2^(MANT+1)]
  return ((e - EMIN) << MANT) + (int)r;
}

// e4m3: 4 exponent bits (bias 7), 3 mantissa bits, subnormals, largest finite value 448,
// no infinities; saturating.
__device__ __forceinline__ uint8_t e4m3_encode(double x) {
  const double a = fabs(x);
  int code;
  if (!(a == a)) code = 0x7f;
  else if (a >= 448.0) code = 0x7e;
  else { code = small_float_code<3, -6>(a); code = code > 0x7e ? 0x7e : code; }
  return (uint8_t)(code | (signbit(x) ? 0x80 : 0));
}
__device__ __forceinline__ double e4m3_decode(uint8_t c) {
  const int ef = (c >> 3) & 0xf, mt = c & 7;
  const double mag = ef == 0 ? scalbn((double)mt, -9) : scalbn((double)(8 + mt), ef - 10);
  return (c & 0x80) ? -mag : mag;
}
// IEEE binary16 bits of a non-negative double; saturates at the largest finite value, 65504.
__device__ __forceinline__ uint16_t fp16_encode_pos(double a) {
  if (!(a == a)) return 0x7e00;
  if (a >= 65504.0) return 0x7bff;
  return (uint16_t)small_float_code<10, -14>(a);
}
__device__ __forceinline__ double fp16_decode_pos(uint16_t h) {
  const int ef = h >> 10, mt = h & 0x3ff;
  if (ef == 31) return mt ? __builtin_nan("") : __builtin_inf();
  return ef == 0 ? scalbn((double)mt, -24) : scalbn((double)(1024 + mt), ef - 25);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Loads and stores that are coherent across the whole device without cache maintenance: the
// workgroups of one launch use them for everything they hand to each other (each compute die
// has an L2 of its own; an ordinary store may sit there, an ordinary load may find an old line).
__device__ __forceinline__ double load_dev(const double* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_dev(double* p, double v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_dev(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_dev(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// four adjacent floats, 16-byte aligned, as two 8-byte accesses
__device__ __forceinline__ void store_dev4(float* p, float x, float y, float z, float w) {
  unsigned long long* q = reinterpret_cast<unsigned long long*>(p);
  __hip_atomic_store(q, (unsigned long long)__float_as_uint(x) | ((unsigned long long)__float_as_uint(y) << 32),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(q + 1, (unsigned long long)__float_as_uint(z) | ((unsigned long long)__float_as_uint(w) << 32),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sums over the 64 lanes of a wave of R per-lane values, in float64, left in red[wave * R + row].
// Rows go in chunks of at most 8: C sums over the 64 lanes at once.  Each exchange halves the
// number of values a lane carries (the lane keeps the rows its bit selects and hands over the
// others), so C = 8 takes 4 + 2 + 1 exchanges and three plain ones instead of 8 x 6.
template <int R>
__device__ __forceinline__ void wave_row_sums(const float (&us)[R], double* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int C = R < 8 ? R : 8;
#pragma unroll
  for (int h = 0; h < R / C; ++h) {
    double ud[C];
#pragma unroll
    for (int i = 0; i < C; ++i) ud[i] = (double)us[h * C + i];
    int width = 32;
#pragma unroll
    for (int cnt = C; cnt > 1; cnt >>= 1, width >>= 1) {
      const bool upper = (lane & width) != 0;
#pragma unroll
      for (int j = 0; j < cnt / 2; ++j) {
        const double send = upper ? ud[j] : ud[j + cnt / 2];
        const double keep = upper ? ud[j + cnt / 2] : ud[j];
        ud[j] = keep + __shfl_xor(send, width);
      }
    }
#pragma unroll
    for (; width >= 1; width >>= 1) ud[0] += __shfl_xor(ud[0], width);
    constexpr int kLanesPerRow = kWave / C;
    if ((lane & (kLanesPerRow - 1)) == 0) red[wave * R + h * C + lane / kLanesPerRow] = ud[0];
  }
}

// Sums over 8 and over 32 adjacent lanes by the lane exchanges of common.h, added in a fixed order.
__device__ __forceinline__ double sum8(double t) {
  t += dpp_move<kDppSwapPairs>(t);
  t += dpp_move<kDppSwapHalfQuads>(t);
  t += dpp_move<kDppHalfMirror>(t);
  return t;
}
__device__ __forceinline__ double sum32(double t) {
  t = sum8(t);
  t += dpp_move<kDppMirror>(t);
  t += __shfl_xor(t, 16);
  return t;
}

// Sums over the 64 lanes of a wave of 8 per-lane values, in float64: the values go through
// `stage` (8 x 64 floats of this wave's own), 8 lanes add up a row (each 8 values, then among
// themselves).  Every lane returns the sum of row lane / 8.
__device__ __forceinline__ double wave_row_sums_staged(const float (&us)[8], float* stage) {
  const int lane = threadIdx.x & 63;
  __builtin_amdgcn_wave_barrier();   // the reads of the previous call precede these writes
#pragma unroll
  for (int x = 0; x < 8; ++x) stage[x * 64 + lane] = us[x];
  __builtin_amdgcn_wave_barrier();   // a wave's LDS accesses complete in order
  const float4 v0 = *reinterpret_cast<const float4*>(stage + (lane >> 3) * 64 + (lane & 7) * 8);
  const float4 v1 = *reinterpret_cast<const float4*>(stage + (lane >> 3) * 64 + (lane & 7) * 8 + 4);
  const double t = (((double)v0.x + (double)v0.y) + ((double)v0.z + (double)v0.w)) +
                   (((double)v1.x + (double)v1.y) + ((double)v1.z + (double)v1.w));
  return sum8(t);
}

// R per-lane values summed over the wave into red[wave * R + row]: through the staging area in
// chunks of 8 rows (4 rows are padded to 8), fewer rows by the exchange above.
template <int R>
__device__ __forceinline__ void wave_row_sums_into(const float (&us)[R], double* red, float* stage) {
  if constexpr (R % 8 == 0 || R == 4) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int h = 0; h < (R + 7) / 8; ++h) {
      float part[8];
#pragma unroll
      for (int x = 0; x < 8; ++x) part[x] = h * 8 + x < R ? us[h * 8 + x] : 0.f;
      const double t = wave_row_sums_staged(part, stage);
      if ((lane & 7) == 0 && h * 8 + (lane >> 3) < R) red[wave * R + h * 8 + (lane >> 3)] = t;
    }
  } else {
    wave_row_sums<R>(us, red);
  }
}

// ---- the grid barrier of the single-launch forms ------------------------------------------------
// Barrier state: one arrival counter per group of 16 workgroups, one for the groups, and one
// release word per group, each in a 128-byte line of its own.
constexpr int kBarrierGroup = 16;
constexpr int kBarrierLine = 32;   // words
constexpr int kBarrierWords = (2 * (kComputeUnits / kBarrierGroup) + 1) * kBarrierLine;

static __global__ void chain_init_kernel(int* expo, int count, unsigned* bar, int* abort) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) expo[i] = INT_MIN;
  if (i < kBarrierWords) bar[i] = 0u;
  if (i == 0) *abort = 0;
}

// What the workgroups exchange goes through load_dev / store_dev, so the barrier needs no cache
// write-back or invalidation (a device-wide fence walks the whole L2 and, issued by every
// workgroup at every barrier, costs more than the loop's arithmetic): every wave waits for its
// own stores to be acknowledged, the workgroup meets, and one thread counts it as arrived.
// Arrivals are counted in two levels, because read-modify-writes of ONE word are served one
// after the other and 256 of them take longer than everything else in an application: the last
// of a group of 16 reports for the group, the last group releases all groups.  All words only
// grow; `phase` is the number of this barrier, counted from 1.
__device__ __forceinline__ void grid_barrier(unsigned* bar, unsigned phase, int* abort, unsigned spin_limit) {
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (threadIdx.x == 0) {
    const int G = gridDim.x, g = blockIdx.x / kBarrierGroup;
    const int groups = (G + kBarrierGroup - 1) / kBarrierGroup;
    const int members = G - g * kBarrierGroup < kBarrierGroup ? G - g * kBarrierGroup : kBarrierGroup;
    unsigned* top = bar + (kComputeUnits / kBarrierGroup) * kBarrierLine;
    unsigned* release = top + kBarrierLine;
    if (atomicAdd(bar + g * kBarrierLine, 1u) + 1u == (unsigned)members * phase)
      if (atomicAdd(top, 1u) + 1u == (unsigned)groups * phase)
        for (int j = 0; j < groups; ++j)
          __hip_atomic_store(release + j * kBarrierLine, phase, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0;
    while (__hip_atomic_load(release + g * kBarrierLine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < phase) {
      if ((spins & 255u) == 0 && __hip_atomic_load(abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
      if (++spins > spin_limit) {
        __hip_atomic_store(abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
  }
  __syncthreads();
}

// Sum of ptr[0..count) over the workgroup in a fixed order; the same value in every thread.
template <int T>
__device__ __forceinline__ double block_sum(const double* ptr, int count, double* scratch) {
  double t = 0.0;
  for (int j = threadIdx.x; j < count; j += T) t += load_dev(ptr + j);
  t = wave_sum(t);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = t;
  __syncthreads();
  double total = 0.0;
#pragma unroll
  for (int wv = 0; wv < T / kWave; ++wv) total += scratch[wv];
  return total;
}

// ---- words that carry their own arrival flag ---------------------------------------------------
// What workgroups of one launch hand to each other without a barrier in between is an 8-byte word:
// the value in the low half, the number of the application it belongs to in the high half,
// written with one device-coherent store.  A reader loads the words it needs and loads them again
// until their high halves show the application it is waiting for: store, signal and load cost
// one trip to memory instead of three.  A reader gives up after spin_limit rounds and raises
// `abort`, which ends every later wait at once.
__device__ __forceinline__ void store_tagged(unsigned long long* p, unsigned bits, unsigned tag) {
  __hip_atomic_store(p, (unsigned long long)bits | ((unsigned long long)tag << 32), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_tagged(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// One round of waiting for tagged words: false when the wait is to be abandoned.
__device__ __forceinline__ bool keep_waiting(unsigned& spins, int* abort, unsigned spin_limit) {
  if ((spins & 63u) == 63u && __hip_atomic_load(abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return false;
  if (++spins > spin_limit) {
    __hip_atomic_store(abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return false;
  }
  __builtin_amdgcn_s_sleep(1);
  return true;
}

// 2^-e as a double for the exponent that travels with the data (INT_MIN: nothing to scale).
__device__ __forceinline__ double unscale(int e) {
  if (e == INT_MIN) return 1.0;
  return scalbn(1.0, -(e > 126 ? 126 : (e < -126 ? -126 : e)));
}

static __global__ void tile_init_kernel(unsigned* words, int count, int* abort) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) words[i] = 0u;
  if (i == 0) *abort = 0;
}


}  // namespace r1svd_detail

// What r1svd_launch hands to the forms that use a bfloat16 weight as it is; workspace pointers are
// device memory laid out by the caller.
struct R1svdBf16Call {
  const uint16_t* W; int64_t ldw; int64_t m, n;
  const double* s; const float* S; int64_t lds; int r, it;
  uint8_t* U; uint8_t* V; uint16_t* sigma16; float* Rout; int64_t ldr;
  float* sf; double* shares; int* expo; unsigned* bar; int* abort_flag;
  float* zpart; double* z; double* u; double* unrm2; double* normpart;
  float* zapp; int64_t zstride; char* resident_ws;
  unsigned spin_limit; bool stream_only;
};
// Runs the loop and the residual in the resident form, else the stream form; false if the device can
// hold neither launch (nothing that matters has been written then).
bool r1svd_bf16_launch(const R1svdBf16Call& c, hipStream_t st);

}  // namespace ptq
