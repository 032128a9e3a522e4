// Blocked column-by-column quantization with error compensation.
//
// Rows of W are independent given the factor U, so a workgroup owns 16 rows
// (one MFMA M-tile) and nothing is exchanged between workgroups.  The lazy
// update is applied "left-looking": when the column loop arrives at block
// [i1, i2), the block's current values are
//
//     S = W[:, i1:i2] - E[:, 0:i1] * U[0:i1, i1:i2]            (float64 MFMA)
//
// with E the errors e_j of all earlier columns (kept transposed, [n][rows], in
// the workspace).  That is the same sum the right-looking rank-B updates would
// have accumulated, but it reads E once and writes nothing but the block.
// Inside the block the same scheme repeats with 16-column mini-blocks: one lane
// per row walks 16 columns in registers (the only truly serial part), then the
// 16 new errors are pushed onto the rest of the block with four MFMAs per
// 16-column tile.
#include "common.h"

namespace ptq {
namespace {

constexpr int kRowTile = 16;    // rows of one MFMA M-tile; a workgroup owns MT of them (MT = 1, 2 or 3)
constexpr int kRowAlign = 96;   // the error matrix is padded to a multiple of every workgroup height
constexpr int kThreads = 512;   // eight waves: one wave per SIMD cannot keep the float64 matrix pipe busy
constexpr int kWaves = kThreads / 64;

__global__ void inv_diag_kernel(const double* __restrict__ U, int64_t ldu, int n, double* invd) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) invd[j] = 1.0 / U[(int64_t)j * ldu + j];
}

// doubles of the LDS region that first holds the partial sums of the lazy update and then the state tile
__host__ __device__ constexpr int state_doubles(int mt, int bw) {
  return mt == 1 ? 4 * kRowTile * bw : kRowTile * mt * (bw + 1);
}

struct QuantArgs {
  const void* W;
  int64_t ldw;
  int m, n, mpad;
  const double* U;
  int64_t ldu;
  const uint8_t* dead;
  const double* invd;
  double* errT;  // [n][mpad]
  int bits, group;
  int i1, bw;    // block start, block width (multiple of 16)
  uint8_t* codes;
  float* scales;
  uint8_t* zeros;
  double* Wq;
  double* row_err2;
  int static_groups;   // scales / zeros hold the grids already (taken from the given weights): use, do not derive
};

// NT = number of 16-column tiles the kernel is instantiated for (>= bw / 16); MT = row tiles of 16
// rows per workgroup.  With 256 compute units a layer of up to 4096 rows gives every unit one row
// tile (MT = 1); taller layers take two or three tiles per workgroup, so that one pass over the
// panel of U serves up to 48 rows and the serial column walk (one lane per row, one wave whatever
// the height) is shared by them.
template <int DT, int NT, int MT>
__device__ __forceinline__ void quant_block(const QuantArgs& a, double* lds) {
  constexpr int kRows = kRowTile * MT;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int row0 = blockIdx.x * kRows;
  const int nt = a.bw >> 4;
  const int sp = a.bw + 1;  // pitch of the state tile
  const double* __restrict__ U = a.U;
  const double* __restrict__ invd = a.invd;

  // LDS carve-up: partial sums of four waves at a time (reused as the state tile),
  // the mini-block errors, the mini-block's 16 x 16 diagonal block of U and its
  // reciprocal pivots (double-buffered), group min / max, and the code tile.
  double* P = lds;                                  // MT = 1: [4][16][bw]; else [rows][bw]
  double* S = lds;                                  // [rows][bw + 1]   (aliases P)
  double* Em = lds + state_doubles(MT, a.bw);       // [16 k][rows]
  double* Qm = Em + 16 * kRows;                     // [16 k][rows + 1]: the mini-block's dequantized values
  double* Ud = Qm + 16 * (kRows + 1);               // [2][16][16]
  double* Id = Ud + 512;                            // [2][16]
  double* gmin = Id + 32;                           // [rows]
  double* gmax = gmin + kRows;                      // [rows]
  uint8_t* Ct = reinterpret_cast<uint8_t*>(gmax + kRows);  // [rows][bw]

  if constexpr (MT == 1) {
  // ---- phase 1: acc = E[rows, 0:i1] * U[0:i1, block], k split over the waves,
    //      operands of the next kDepth steps in flight while the MFMAs run
    f64x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f64x4{0.0, 0.0, 0.0, 0.0};
    // (pairs of tiles share 16-byte loads when the block is a whole number of pairs, an even ldu keeps
    // them aligned, and the offsets fit the buffer form; see below)
    const bool paired = (nt % 2 == 0) && (a.ldu % 2 == 0) &&
                        (int64_t)a.n * a.ldu * 8 < ((int64_t)1 << 31) && (int64_t)a.n * a.mpad * 8 < ((int64_t)1 << 31);
    auto column_of = [&](int t, int cl) { return paired ? 32 * (t >> 1) + 2 * cl + (t & 1) : 16 * t + cl; };
    {
      constexpr int kDepth = (NT >= 16) ? 2 : 4;
      const int kl = lane >> 4, cl = lane & 15;
      const int wv = __builtin_amdgcn_readfirstlane(wave);   // uniform: scalar loop control
      int coff[NT];  // tiles beyond the block re-read its last tile (result unused)
#pragma unroll
      for (int t = 0; t < NT; ++t) coff[t] = 16 * (t < nt ? t : nt - 1);
      const int niter = (a.i1 - 4 * wv + 4 * kWaves - 1) / (4 * kWaves);  // k = 32 it + 4 wave + kl < i1 (a multiple of 16)
      double av[kDepth], bv[kDepth][NT];
      auto mfmas = [&](int d) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[d], bv[d][t], acc[t], 0, 0, 0);
      };
      // The loop: slot d's MFMAs, then the request for the step kDepth later into the same slot.  In the
      // steady state there is no branch between the first request and the last iteration, every slot is
      // valid and has a successor, and the requests are buffer loads whose per-lane offsets never change
      // (the step advances in a scalar offset: no address arithmetic between the MFMAs).
      auto run = [&](auto issue) {
        int it = 0;
        if (niter >= 2 * kDepth) {
#pragma unroll
          for (int d = 0; d < kDepth; ++d) issue(d, d);
          for (; it + 2 * kDepth <= niter; it += kDepth) {
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
              mfmas(d);
              issue(d, it + d + kDepth);
            }
          }
        } else {
#pragma unroll
          for (int d = 0; d < kDepth; ++d)
            if (d < niter) issue(d, d);
        }
        for (; it < niter; it += kDepth) {
#pragma unroll
          for (int d = 0; d < kDepth; ++d) {
            if (it + d < niter) {
              mfmas(d);
              if (it + d + kDepth < niter) issue(d, it + d + kDepth);
            }
          }
        }
      };
      const bool offsets32 = (int64_t)a.n * a.ldu * 8 < ((int64_t)1 << 31) && (int64_t)a.n * a.mpad * 8 < ((int64_t)1 << 31);
      if (offsets32) {
        const __amdgpu_buffer_rsrc_t re = __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(a.errT + row0), 0,
                                                                            (int)0xFFFFFFFFu, 0x00020000);
        const __amdgpu_buffer_rsrc_t ru = __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(U + a.i1), 0,
                                                                            (int)0xFFFFFFFFu, 0x00020000);
        const int ve = ((4 * wv + kl) * a.mpad + cl) * 8;
        const int se = 4 * kWaves * a.mpad * 8, su = 4 * kWaves * (int)a.ldu * 8;
        if (paired) {
          // The address unit takes a wave's load in 16 steps of four lanes whatever the width, so 8-byte
          // loads top out at 32 bytes per clock and compute unit -- less than the eight MFMAs of a k-step
          // need.  A lane therefore fetches two neighbouring columns at once (16 bytes) and gives one to each
          // of a pair of tiles: tile 2p + q works on columns 32 p + 2 cl + q.  The MFMA does not care which
          // columns make up a tile; the partial sums go back to their columns through the same map.
          int vu[NT / 2];
#pragma unroll
          for (int p = 0; p < NT / 2; ++p) vu[p] = ((4 * wv + kl) * (int)a.ldu + 2 * cl + (coff[2 * p] & ~31)) * 8;
          typedef double f64x2 __attribute__((ext_vector_type(2)));
          run([&](int slot, int it) {
            av[slot] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(re, ve, it * se, 0));
#pragma unroll
            for (int p = 0; p < NT / 2; ++p) {
              const f64x2 two = __builtin_bit_cast(f64x2, __builtin_amdgcn_raw_buffer_load_b128(ru, vu[p], it * su, 0));
              bv[slot][2 * p] = two[0];
              bv[slot][2 * p + 1] = two[1];
            }
          });
        } else {
          int vu[NT];
#pragma unroll
          for (int t = 0; t < NT; ++t) vu[t] = ((4 * wv + kl) * (int)a.ldu + cl + coff[t]) * 8;
          run([&](int slot, int it) {
            av[slot] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(re, ve, it * se, 0));
#pragma unroll
            for (int t = 0; t < NT; ++t)
              bv[slot][t] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(ru, vu[t], it * su, 0));
          });
        }
      } else {
        const double* ep = a.errT + (int64_t)(4 * wv + kl) * a.mpad + row0 + cl;
        const double* up = U + (int64_t)(4 * wv + kl) * a.ldu + a.i1 + cl;
        run([&](int slot, int it) {
          av[slot] = ep[(int64_t)it * (4 * kWaves) * a.mpad];
          const double* u = up + (int64_t)it * (4 * kWaves) * a.ldu;
#pragma unroll
          for (int t = 0; t < NT; ++t) bv[slot][t] = u[coff[t]];
        });
      }
    }
    // the eight partial sums are folded in two rounds through four LDS slots
    if (wave >= 4) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
        if (t < nt) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            P[((wave - 4) * kRows + 4 * r + (lane >> 4)) * a.bw + column_of(t, lane & 15)] = acc[t][r];
        }
    }
    __syncthreads();
    if (wave < 4) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
        if (t < nt) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            P[(wave * kRows + 4 * r + (lane >> 4)) * a.bw + column_of(t, lane & 15)] += acc[t][r];
        }
    }
    __syncthreads();

  } else {
    const int wv = __builtin_amdgcn_readfirstlane(wave);   // uniform: scalar loop control
    const bool paired = (nt % 2 == 0) && (a.ldu % 2 == 0) && (a.mpad % 2 == 0) &&
                        (int64_t)a.n * a.ldu * 8 < ((int64_t)1 << 31) && (int64_t)a.n * a.mpad * 8 < ((int64_t)1 << 31);
    if (paired) {
      // ---- phase 1, several row tiles, 16-byte loads (see the one-tile form for why): the waves are two
      //      groups that take alternate k-steps; inside a group a wave owns pairs of column tiles (a lane
      //      fetches two neighbouring columns of U at once, tile 2p + q works on columns 32 p + 2 cl + q) for
      //      all row tiles, and the first two row tiles are a pair as well (a lane fetches the errors of rows
      //      2 cl and 2 cl + 1 at once: row tile 0 works on the even rows of the first 32, tile 1 on the odd
      //      ones).  Three load instructions feed six MFMAs.  The two groups' sums meet in the state tile.
      constexpr int PPW = (NT / 2 + 3) / 4;   // pairs of column tiles per wave
      constexpr int kDepth = 4;
      typedef double f64x2 __attribute__((ext_vector_type(2)));
      const int grp = wv >> 2, w4 = wv & 3;
      f64x4 acc[MT][2 * PPW];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int q = 0; q < 2 * PPW; ++q) acc[mt][q] = f64x4{0.0, 0.0, 0.0, 0.0};
      const bool active = 2 * w4 < nt;
      if (active) {
        const int kl = lane >> 4, cl = lane & 15;
        const int steps = a.i1 >> 2;                    // i1 is a multiple of 16
        const int niter = (steps - grp + 1) >> 1;       // this group's k-steps: grp, grp + 2, ...
        double av[kDepth][MT], bv[kDepth][2 * PPW];
        auto mfmas = [&](int d) {
#pragma unroll
          for (int q = 0; q < 2 * PPW; ++q)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              acc[mt][q] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[d][mt], bv[d][q], acc[mt][q], 0, 0, 0);
        };
        const __amdgpu_buffer_rsrc_t re = __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(a.errT + row0), 0,
                                                                            (int)0xFFFFFFFFu, 0x00020000);
        const __amdgpu_buffer_rsrc_t ru = __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(U + a.i1), 0,
                                                                            (int)0xFFFFFFFFu, 0x00020000);
        const int ve01 = ((4 * grp + kl) * a.mpad + 2 * cl) * 8;          // rows 2 cl, 2 cl + 1
        const int ve2 = ((4 * grp + kl) * a.mpad + 32 + cl) * 8;          // row 32 + cl (three row tiles)
        int vu[PPW];
#pragma unroll
        for (int q = 0; q < PPW; ++q) {
          const int pr = (2 * (w4 + 4 * q) < nt) ? w4 + 4 * q : w4;       // a pair beyond the block re-reads a valid one
          vu[q] = ((4 * grp + kl) * (int)a.ldu + 32 * pr + 2 * cl) * 8;
        }
        const int se = 8 * a.mpad * 8, su = 8 * (int)a.ldu * 8;
        auto issue = [&](int slot, int it) {
          const f64x2 e01 = __builtin_bit_cast(f64x2, __builtin_amdgcn_raw_buffer_load_b128(re, ve01, it * se, 0));
          av[slot][0] = e01[0];
          av[slot][1] = e01[1];
          if constexpr (MT == 3) av[slot][2] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(re, ve2, it * se, 0));
#pragma unroll
          for (int q = 0; q < PPW; ++q) {
            const f64x2 two = __builtin_bit_cast(f64x2, __builtin_amdgcn_raw_buffer_load_b128(ru, vu[q], it * su, 0));
            bv[slot][2 * q] = two[0];
            bv[slot][2 * q + 1] = two[1];
          }
        };
        int it = 0;   // branch-free steady state, as in the one-tile form
        if (niter >= 2 * kDepth) {
#pragma unroll
          for (int d = 0; d < kDepth; ++d) issue(d, d);
          for (; it + 2 * kDepth <= niter; it += kDepth) {
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
              mfmas(d);
              issue(d, it + d + kDepth);
            }
          }
        } else {
#pragma unroll
          for (int d = 0; d < kDepth; ++d)
            if (d < niter) issue(d, d);
        }
        for (; it < niter; it += kDepth) {
#pragma unroll
          for (int d = 0; d < kDepth; ++d) {
            if (it + d < niter) {
              mfmas(d);
              if (it + d + kDepth < niter) issue(d, it + d + kDepth);
            }
          }
        }
      }
      // row of accumulator element r of row tile mt, column of tile 2 pr + q2
      auto put = [&](bool add) {
        if (!active) return;
#pragma unroll
        for (int q = 0; q < 2 * PPW; ++q) {
          const int pr = w4 + 4 * (q >> 1);
          if (2 * pr < nt) {
            const int col = 32 * pr + 2 * (lane & 15) + (q & 1);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int i = 4 * r + (lane >> 4);
                const int row = mt < 2 ? 2 * i + mt : 32 + i;
                double* at = P + row * a.bw + col;
                *at = add ? *at + acc[mt][q][r] : acc[mt][q][r];
              }
          }
        }
      };
      if (grp == 1) put(false);
      __syncthreads();
      if (grp == 0) put(true);
      __syncthreads();
    } else {
      // ---- phase 1, several row tiles: a wave owns column tiles (wave, wave + 8, ...) and runs over all k
      //      itself -- no partial sums to fold; the operand of U is fetched once for all MT row tiles, the
      //      rows of E (the same for every wave) come out of the cache after the first wave's fetch
      constexpr int TPW = (NT + kWaves - 1) / kWaves;
      constexpr int kDepth = 4;
      f64x4 acc[MT][TPW];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int q = 0; q < TPW; ++q) acc[mt][q] = f64x4{0.0, 0.0, 0.0, 0.0};
      if (wv < nt) {
        const int kl = lane >> 4, cl = lane & 15;
        int coff[TPW];  // tiles beyond the block re-read a valid tile (result unused)
#pragma unroll
        for (int q = 0; q < TPW; ++q) coff[q] = 16 * ((wv + kWaves * q) < nt ? wv + kWaves * q : wv);
        const int niter = a.i1 >> 2;   // i1 is a multiple of 16
        double av[kDepth][MT], bv[kDepth][TPW];
        auto mfmas = [&](int d) {
#pragma unroll
          for (int q = 0; q < TPW; ++q)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              acc[mt][q] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[d][mt], bv[d][q], acc[mt][q], 0, 0, 0);
        };
        auto run = [&](auto issue) {   // branch-free steady state, as in the one-tile form
          int it = 0;
          if (niter >= 2 * kDepth) {
#pragma unroll
            for (int d = 0; d < kDepth; ++d) issue(d, d);
            for (; it + 2 * kDepth <= niter; it += kDepth) {
#pragma unroll
              for (int d = 0; d < kDepth; ++d) {
                mfmas(d);
                issue(d, it + d + kDepth);
              }
            }
          } else {
#pragma unroll
            for (int d = 0; d < kDepth; ++d)
              if (d < niter) issue(d, d);
          }
          for (; it < niter; it += kDepth) {
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
              if (it + d < niter) {
                mfmas(d);
                if (it + d + kDepth < niter) issue(d, it + d + kDepth);
              }
            }
          }
        };
        const bool offsets32 = (int64_t)a.n * a.ldu * 8 < ((int64_t)1 << 31) && (int64_t)a.n * a.mpad * 8 < ((int64_t)1 << 31);
        if (offsets32) {
          const __amdgpu_buffer_rsrc_t re = __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(a.errT + row0), 0,
                                                                              (int)0xFFFFFFFFu, 0x00020000);
          const __amdgpu_buffer_rsrc_t ru = __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(U + a.i1), 0,
                                                                              (int)0xFFFFFFFFu, 0x00020000);
          int ve[MT], vu[TPW];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) ve[mt] = (kl * a.mpad + cl + kRowTile * mt) * 8;
#pragma unroll
          for (int q = 0; q < TPW; ++q) vu[q] = (kl * (int)a.ldu + cl + coff[q]) * 8;
          const int se = 4 * a.mpad * 8, su = 4 * (int)a.ldu * 8;
          run([&](int slot, int it) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              av[slot][mt] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(re, ve[mt], it * se, 0));
#pragma unroll
            for (int q = 0; q < TPW; ++q)
              bv[slot][q] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(ru, vu[q], it * su, 0));
          });
        } else {
          const double* ep = a.errT + (int64_t)kl * a.mpad + row0 + cl;
          const double* up = U + (int64_t)kl * a.ldu + a.i1 + cl;
          run([&](int slot, int it) {
            const double* e = ep + (int64_t)it * 4 * a.mpad;
            const double* u = up + (int64_t)it * 4 * a.ldu;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) av[slot][mt] = e[kRowTile * mt];
#pragma unroll
            for (int q = 0; q < TPW; ++q) bv[slot][q] = u[coff[q]];
          });
        }
#pragma unroll
        for (int q = 0; q < TPW; ++q) {
          const int t = wave + kWaves * q;
          if (t < nt) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
              for (int r = 0; r < 4; ++r)
                P[(kRowTile * mt + 4 * r + (lane >> 4)) * a.bw + 16 * t + (lane & 15)] = acc[mt][q][r];
          }
        }
      }
      __syncthreads();

    }
  }

  // ---- state tile S = W - (sum of the partial sums), dead channels read as zero
  {
    constexpr int NP = (kRows * 16 * NT + kThreads - 1) / kThreads;
    double sv[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int e = tid + kThreads * p;
      sv[p] = 0.0;
      if (e < kRows * a.bw) {
        const int r = e / a.bw, c = e - r * a.bw;
        double w = 0.0;
        if (row0 + r < a.m && !(a.dead && a.dead[a.i1 + c]))
          w = load_as_f64<DT>(a.W, (int64_t)(row0 + r) * a.ldw + a.i1 + c);
        if constexpr (MT == 1) {
          const double s01 = P[(0 * kRows + r) * a.bw + c] + P[(1 * kRows + r) * a.bw + c];
          const double s23 = P[(2 * kRows + r) * a.bw + c] + P[(3 * kRows + r) * a.bw + c];
          sv[p] = w - (s01 + s23);
        } else {
          sv[p] = w - P[r * a.bw + c];
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int e = tid + kThreads * p;
      if (e < kRows * a.bw) {
        const int r = e / a.bw, c = e - r * a.bw;
        S[r * sp + c] = sv[p];
      }
    }
    // diagonal block of the first mini-block
    if (tid < 256) Ud[tid] = U[(int64_t)(a.i1 + (tid >> 4)) * a.ldu + a.i1 + (tid & 15)];
    if (tid < 16) Id[tid] = invd[a.i1 + tid];
  }
  __syncthreads();

  // ---- phase 2: 16-column mini-blocks
  const double maxq = (double)((1 << a.bits) - 1);
  const int ng = a.n / a.group;
  double scale = 1.0, rscale = 1.0, zero = 0.0, klo = 0.0, khi = 0.0, err2 = 0.0;  // lanes 0..15 of wave 0
  constexpr int kUpd = (NT + kWaves - 1) / kWaves;  // tiles one wave may have to update per mini-block
  for (int mb = 0; mb < nt; ++mb) {
    const int c0 = 16 * mb;           // first column of the mini-block inside the block
    const int gcol = a.i1 + c0;       // ... and in the layer
    const int buf = mb & 1;
    const bool gstart = (gcol % a.group) == 0;
    // operands that do not depend on this mini-block's results: the next diagonal
    // block and the rows of U that push this mini-block's errors onto later tiles
    double ud_next = 0.0, id_next = 0.0;
    if (mb + 1 < nt) {
      if (tid < 256) ud_next = U[(int64_t)(gcol + 16 + (tid >> 4)) * a.ldu + gcol + 16 + (tid & 15)];
      if (tid < 16) id_next = invd[gcol + 16 + tid];
    }
    double ub[kUpd][4];
#pragma unroll
    for (int q = 0; q < kUpd; ++q) {
      const int t = mb + 1 + wave + kWaves * q;
      const int tc = t < nt ? t : nt - 1;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        ub[q][kk] = U[(int64_t)(gcol + 4 * kk + (lane >> 4)) * a.ldu + a.i1 + 16 * tc + (lane & 15)];
    }
    if (gstart && !a.static_groups) {
      // min / max of the group's current values: 16 lanes per row, 16 rows per pass of the first four waves
      if (tid < 256) {
#pragma unroll
        for (int pass = 0; pass < MT; ++pass) {
          const int r = kRowTile * pass + (tid >> 4), sub = tid & 15;
          double lo = 0.0, hi = 0.0;
          for (int c = sub; c < a.group; c += 16) {
            const double v = S[r * sp + c0 + c];
            lo = fmin(lo, v);
            hi = fmax(hi, v);
          }
          // over the row's 16 lanes (min and max do not depend on the order)
          lo = fmin(lo, dpp_move<kDppSwapPairs>(lo));         hi = fmax(hi, dpp_move<kDppSwapPairs>(hi));
          lo = fmin(lo, dpp_move<kDppSwapHalfQuads>(lo));     hi = fmax(hi, dpp_move<kDppSwapHalfQuads>(hi));
          lo = fmin(lo, dpp_move<kDppHalfMirror>(lo));        hi = fmax(hi, dpp_move<kDppHalfMirror>(hi));
          lo = fmin(lo, dpp_move<kDppMirror>(lo));            hi = fmax(hi, dpp_move<kDppMirror>(hi));
          if (sub == 0) {
            gmin[r] = lo;
            gmax[r] = hi;
          }
        }
      }
      __syncthreads();
    }
    if (tid < kRows) {
      const int r = tid;
      const bool rlive = row0 + r < a.m;
      if (gstart && a.static_groups) {
        const int64_t at = (int64_t)(rlive ? row0 + r : 0) * ng + gcol / a.group;
        scale = (double)a.scales[at];
        rscale = 1.0 / scale;
        zero = (double)a.zeros[at];
        klo = -zero;
        khi = maxq - zero;
      } else if (gstart) {
        double lo = gmin[r], hi = gmax[r];
        if (lo == hi) {
          lo = -1.0;
          hi = 1.0;
        }
        const float sf = (float)((hi - lo) / maxq);
        scale = (double)sf;
        rscale = 1.0 / scale;
        zero = rint(-lo / scale);
        klo = -zero;
        khi = maxq - zero;
        if (rlive) {
          a.scales[(int64_t)(row0 + r) * ng + gcol / a.group] = sf;
          a.zeros[(int64_t)(row0 + r) * ng + gcol / a.group] = (uint8_t)zero;
        }
      }
      // The walk is one dependent chain of float64 operations per column; everything that does not
      // depend on it is taken out of its way: the reciprocal pivots and the entries of U that carry
      // a column's error to the very next column sit in registers before it starts; the error's
      // effect on the columns further on is applied one step later, next to the following column's
      // chain, as independent operations that fill its latency (left to itself the compiler gathers
      // them in front of each column as one more chain; the scheduling barrier keeps a step's
      // instructions in their step); and the results go to LDS only -- other waves write them out.
      double w[16], idr[16], sd[15], rp[16], rc[16];
      const double* ud = Ud + buf * 256;
#pragma unroll
      for (int j = 0; j < 16; ++j) w[j] = S[r * sp + c0 + j];
#pragma unroll
      for (int j = 0; j < 16; ++j) idr[j] = Id[buf * 16 + j];
#pragma unroll
      for (int j = 0; j < 15; ++j) sd[j] = ud[j * 16 + j + 1];
      double ep = 0.0;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        // the rest of row j of U, for the next step
#pragma unroll
        for (int c = j + 2; c < 16; ++c) rc[c] = ud[j * 16 + c];
        // column j - 1 onto the columns after this one: nothing below waits for these
        if (j > 0) {
#pragma unroll
          for (int c = j + 1; c < 16; ++c) w[c] = fma(-ep, rp[c], w[c]);
        }
        // x = w / scale, correctly rounded from the reciprocal (one Newton step
        // on the quotient), so that exact ties round as a true division would
        const double q0 = w[j] * rscale;
        const double rem = fma(-q0, scale, w[j]);
        const double x = fma(rem, rscale, q0);
        // k = code - zero, clamped; scale * k is exact (24-bit x 9-bit), so one
        // fma gives w - q with the same single rounding as the subtraction
        const double k = fmin(fmax(rint(x), klo), khi);
        const double e = fma(-scale, k, w[j]) * idr[j];
        if (j < 15) w[j + 1] = fma(-e, sd[j], w[j + 1]);
        err2 = fma(e, e, err2);
        Ct[r * a.bw + c0 + j] = (uint8_t)(k + zero);
        Em[j * kRows + r] = e;
        Qm[j * (kRows + 1) + r] = scale * k;
        ep = e;
#pragma unroll
        for (int c = j + 2; c < 16; ++c) rp[c] = rc[c];
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
    // push the 16 new errors onto the later tiles of the block
#pragma unroll
    for (int q = 0; q < kUpd; ++q) {
      const int t = mb + 1 + wave + kWaves * q;
      if (t < nt) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          f64x4 d = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            const double av = Em[(4 * kk + (lane >> 4)) * kRows + kRowTile * mt + (lane & 15)];
            d = __builtin_amdgcn_mfma_f64_16x16x4f64(av, ub[q][kk], d, 0, 0, 0);
          }
          double sv[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) sv[r] = S[(kRowTile * mt + 4 * r + (lane >> 4)) * sp + 16 * t + (lane & 15)];
#pragma unroll
          for (int r = 0; r < 4; ++r) S[(kRowTile * mt + 4 * r + (lane >> 4)) * sp + 16 * t + (lane & 15)] = sv[r] - d[r];
        }
      }
    }
    // the mini-block's errors (for the later blocks) and dequantized values leave through the
    // upper four waves, 128 contiguous bytes per 16 lanes
    if (tid >= 256) {
#pragma unroll
      for (int pass = 0; pass < MT; ++pass) {
        const int e = tid - 256 + 256 * pass;          // Em is [16 k][rows]: e = k * rows + row
        const int k = e / kRows, rr = e - k * kRows;
        a.errT[(int64_t)(gcol + k) * a.mpad + row0 + rr] = Em[e];
        const int r = e >> 4, j = e & 15;
        if (a.Wq && row0 + r < a.m) a.Wq[(int64_t)(row0 + r) * a.n + gcol + j] = Qm[j * (kRows + 1) + r];
      }
    }
    if (mb + 1 < nt) {
      if (tid < 256) Ud[(buf ^ 1) * 256 + tid] = ud_next;
      if (tid < 16) Id[(buf ^ 1) * 16 + tid] = id_next;
    }
    __syncthreads();
  }

  // ---- outputs of the block
  for (int e = tid; e < kRows * a.bw; e += kThreads) {
    const int r = e / a.bw, c = e - r * a.bw;
    if (row0 + r < a.m) a.codes[(int64_t)(row0 + r) * a.n + a.i1 + c] = Ct[r * a.bw + c];
  }
  if (a.row_err2 && tid < kRows && row0 + tid < a.m) {
    if (a.i1 == 0)
      a.row_err2[row0 + tid] = err2;
    else
      a.row_err2[row0 + tid] += err2;
  }
}

template <int DT, int NT, int MT>
__global__ __launch_bounds__(kThreads) void quant_block_kernel(QuantArgs a) {
  extern __shared__ double lds[];
  quant_block<DT, NT, MT>(a, lds);
}

// All blocks of a layer in one launch: a workgroup's rows depend on no other workgroup's, so it walks the blocks at
// its own pace (a launch per block makes every workgroup wait for the slowest one of every block).  What a block
// leaves in global memory for the next ones -- its errors, the running row sums -- is written and read by the same
// workgroup, hence the same compute unit and cache: a workgroup barrier between blocks orders it.
template <int DT, int NT, int MT>
__global__ __launch_bounds__(kThreads) void quant_layer_kernel(QuantArgs a, int block) {
  extern __shared__ double lds[];
  for (int i1 = 0; i1 < a.n; i1 += block) {
    QuantArgs b = a;
    b.i1 = i1;
    b.bw = (a.n - i1 < block) ? a.n - i1 : block;
    // With several row tiles the arguments are made opaque per block: what the compiler would otherwise compute
    // once for all blocks and keep -- per-lane offsets into U, the errors, the outputs -- costs more registers than
    // the kernel has (measured, 8192 x 4096: 3.09 ms opaque, 3.24 not, 3.38 with a launch per block).  With one row
    // tile keeping them pays (4096 x 11008: 9.93 ms against 10.52 opaque and 10.19 with a launch per block).
    if constexpr (MT > 1) {
      asm volatile("" : "+s"(b.U), "+s"(b.errT), "+s"(b.W), "+s"(b.Wq), "+s"(b.codes), "+s"(b.mpad), "+s"(b.n));
      asm volatile("" : "+s"(b.invd), "+s"(b.dead), "+s"(b.scales), "+s"(b.zeros), "+s"(b.ldu), "+s"(b.ldw), "+s"(b.m));
    }
    quant_block<DT, NT, MT>(b, lds);
    __syncthreads();
  }
}

size_t block_lds_bytes(int mt, int bw) {
  const int rows = kRowTile * mt;
  return (size_t)(state_doubles(mt, bw) + 16 * rows + 16 * (rows + 1) + 512 + 32 + 2 * rows) * sizeof(double) +
         (size_t)rows * bw;
}

template <int DT, int NT, int MT>
ptq_status launch_block(const QuantArgs& a, hipStream_t st) {
  if (!lds_opt_in<quant_block_kernel<DT, NT, MT>>((int)block_lds_bytes(MT, 16 * NT))) return PTQ_ERR_HIP;
  const unsigned wgs = (unsigned)ceil_div(a.m, kRowTile * MT);
  quant_block_kernel<DT, NT, MT><<<wgs, kThreads, block_lds_bytes(MT, a.bw), st>>>(a);
  return PTQ_OK;
}

template <int DT, int NT, int MT>
ptq_status launch_layer(const QuantArgs& a, int block, hipStream_t st) {
  const unsigned wgs = (unsigned)ceil_div(a.m, kRowTile * MT);
  if (!lds_opt_in<quant_layer_kernel<DT, NT, MT>>((int)block_lds_bytes(MT, 16 * NT))) return PTQ_ERR_HIP;
  quant_layer_kernel<DT, NT, MT><<<wgs, kThreads, block_lds_bytes(MT, block), st>>>(a, block);
  return PTQ_OK;
}

template <int DT, int MT>
ptq_status run_blocks(QuantArgs a, int block, hipStream_t st) {
  // one launch for the layer; blocks wider than 128 columns (the 16-tile instantiation is short of registers as it
  // is) keep a launch per block
  if (block <= 128) {
    const int nt = block / 16;
    if (nt <= 2) return launch_layer<DT, 2, MT>(a, block, st);
    if (nt <= 4) return launch_layer<DT, 4, MT>(a, block, st);
    return launch_layer<DT, 8, MT>(a, block, st);
  }
  for (int i1 = 0; i1 < a.n; i1 += block) {
    a.i1 = i1;
    a.bw = (a.n - i1 < block) ? a.n - i1 : block;
    const int nt = a.bw / 16;
    ptq_status rc;
    if (nt <= 2) rc = launch_block<DT, 2, MT>(a, st);
    else if (nt <= 4) rc = launch_block<DT, 4, MT>(a, st);
    else if (nt <= 8) rc = launch_block<DT, 8, MT>(a, st);
    else rc = launch_block<DT, 16, MT>(a, st);
    if (rc != PTQ_OK) return rc;
  }
  return PTQ_OK;
}

// Row tiles per workgroup: one while the layer's row tiles fit the chip's 256 compute units (with a
// little slack), else as many (up to 3) as bring the workgroup count back to about one per unit.
int row_tiles_per_workgroup(int64_t m) {
  const int64_t tiles = ceil_div(m, kRowTile);
  if (tiles <= 288) return 1;
  return tiles <= 576 ? 2 : 3;
}

template <int DT>
ptq_status run_blocks_any(const QuantArgs& a, int block, hipStream_t st) {
  switch (row_tiles_per_workgroup(a.m)) {
    case 1: return run_blocks<DT, 1>(a, block, st);
    case 2: return run_blocks<DT, 2>(a, block, st);
    default: return run_blocks<DT, 3>(a, block, st);
  }
}

}  // namespace

// Static groups: the grid of every (row, group) from the weights as given (dead columns count as
// zeros), by the same arithmetic as the column walk uses at a group start.  One thread each.
template <int DT>
__global__ __launch_bounds__(256) void static_grid_kernel(const void* __restrict__ W, int64_t ldw, int m, int n,
                                                          const uint8_t* __restrict__ dead, int bits, int group,
                                                          float* __restrict__ scales, uint8_t* __restrict__ zeros) {
  const int ng = n / group;
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)m * ng) return;
  const int r = (int)(e / ng), k = (int)(e - (int64_t)r * ng);
  const double maxq = (double)((1 << bits) - 1);
  double lo = 0.0, hi = 0.0;
  for (int c = k * group; c < (k + 1) * group; ++c) {
    const double v = (dead && dead[c]) ? 0.0 : load_as_f64<DT>(W, (int64_t)r * ldw + c);
    lo = fmin(lo, v);
    hi = fmax(hi, v);
  }
  if (lo == hi) {
    lo = -1.0;
    hi = 1.0;
  }
  const float sf = (float)((hi - lo) / maxq);
  scales[e] = sf;
  zeros[e] = (uint8_t)rint(-lo / (double)sf);
}

size_t quantize_workspace_bytes(int64_t m, int64_t n) {
  const int64_t mpad = ceil_div(m, kRowAlign) * kRowAlign;
  return align_up((size_t)n * (size_t)mpad * sizeof(double), 256) + align_up((size_t)n * sizeof(double), 256);
}

ptq_status quantize_launch(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n,
                           const double* U, int64_t ldu, const uint8_t* dead_mask, int bits, int group,
                           int block, uint8_t* codes, float* scales, uint8_t* zeros, double* Wq,
                           double* row_err2, int static_groups, void* ws, size_t ws_bytes, hipStream_t st) {
  if (m == 0 || n == 0) return PTQ_OK;
  if (ws_bytes < quantize_workspace_bytes(m, n)) return PTQ_ERR_WORKSPACE;
  // a group wider than the block makes the grid depend on columns beyond the
  // block: run with the block widened to the group (the block size only
  // changes the order of summation)
  if (group > block) block = group;
  QuantArgs a;
  a.W = W;
  a.ldw = ldw;
  a.m = (int)m;
  a.n = (int)n;
  a.mpad = (int)(ceil_div(m, kRowAlign) * kRowAlign);
  a.U = U;
  a.ldu = ldu;
  a.dead = dead_mask;
  a.errT = static_cast<double*>(ws);
  a.invd = reinterpret_cast<double*>(static_cast<char*>(ws) +
                                     align_up((size_t)n * (size_t)a.mpad * sizeof(double), 256));
  a.bits = bits;
  a.group = group;
  a.i1 = 0;
  a.bw = 0;
  a.codes = codes;
  a.scales = scales;
  a.zeros = zeros;
  a.Wq = Wq;
  a.row_err2 = row_err2;
  a.static_groups = static_groups;
  if (static_groups) {
    const unsigned gg = (unsigned)ceil_div(m * (n / group), 256);
    switch (wdt) {
      case PTQ_F32: static_grid_kernel<PTQ_F32><<<gg, 256, 0, st>>>(W, ldw, (int)m, (int)n, dead_mask, bits, group, scales, zeros); break;
      case PTQ_BF16: static_grid_kernel<PTQ_BF16><<<gg, 256, 0, st>>>(W, ldw, (int)m, (int)n, dead_mask, bits, group, scales, zeros); break;
      case PTQ_F64: static_grid_kernel<PTQ_F64><<<gg, 256, 0, st>>>(W, ldw, (int)m, (int)n, dead_mask, bits, group, scales, zeros); break;
      default: return PTQ_ERR_DTYPE;
    }
  }
  inv_diag_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, st>>>(U, ldu, (int)n, const_cast<double*>(a.invd));
  PTQ_HIP_CHECK_LAUNCH();
  ptq_status rc;
  switch (wdt) {
    case PTQ_F32: rc = run_blocks_any<PTQ_F32>(a, block, st); break;
    case PTQ_BF16: rc = run_blocks_any<PTQ_BF16>(a, block, st); break;
    case PTQ_F64: rc = run_blocks_any<PTQ_F64>(a, block, st); break;
    default: return PTQ_ERR_DTYPE;
  }
  if (rc != PTQ_OK) return rc;
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
