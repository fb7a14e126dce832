// Y (+)= A X with dense row-major X, Y (Section 7.2.2 evaluates SpMM over a hybrid blocked
// ELL / COO layout).  One kernel per storage layout; lanes of a wavefront run across the
// columns of X so every gathered X row is one contiguous read.
#include "common.h"
#include "device.h"

namespace us {

typedef float float4v __attribute__((ext_vector_type(4)));

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Map launch index i
// to a tile so that every XCD works on one contiguous range of tiles and neighbouring tiles
// (which gather overlapping X rows for banded matrices) share an L2.
__device__ __forceinline__ int64_t xcd_tile(int64_t i, int64_t per_xcd) { return (i & 7) * per_xcd + (i >> 3); }

// ------------------------------------------------------------------ BCSR 4x4 on the matrix cores
// One wavefront owns one block row and 64 columns of X.  v_mfma_f32_4x4x1 computes 16
// independent 4x4 += (4x1)(1x4) products; feeding the same A column to all 16 and 64
// different X columns gives Y[4 x 64] += A[:,k] X[k, 64 cols] per instruction, i.e. lane l
// ends up holding column l of the 4 output rows.
//
// HBM is not what binds this kernel (its fetches are the compulsory ones; the 3.2 GB of gathered X rows
// come out of L2), instruction issue and L1 traffic are: a wave64 VALU instruction occupies its SIMD for
// 4 cycles and a 64-lane load of 16 bytes per lane costs the L1 a kilobyte whatever it returns.  So
//  * block columns are read with one coalesced load per 64 blocks and handed out by v_readlane (scalars),
//    the address of a gathered row is scalar arithmetic plus a per-lane offset that never changes;
//  * the values of four blocks (64 floats) are ONE coalesced load, lane (u, k, r) taking element [r][k] of
//    block u, i.e. the block transposed on the way in: lanes 4q .. 4q+3 then hold column k of block u with
//    q = 4u + k, exactly the four A values of a 4x4x1 product, and the MFMA's A-broadcast (cbsz = 4,
//    abid = q) feeds them to all 16 of its blocks -- no copies of A across lanes, no shuffles;
//  * full groups of four blocks run without any bounds logic (ncols % 4 == 0 means no block sticks out
//    of the matrix; otherwise the guarded path takes every block).
constexpr int BCSR_R = 2;   // groups of four blocks in flight: 16 * BCSR_R gathered rows per wavefront before the first MFMA

template <int Q>
__device__ __forceinline__ float4v mfma_bcast(float a, float x, float4v acc) {
  return __builtin_amdgcn_mfma_f32_4x4x1f32(a, x, acc, 4, Q, 0);
}

template <int R>
__global__ __launch_bounds__(256) void bcsr44_spmm_mfma_kernel(const int32_t *ptr, const int32_t *idx,
                                                              const float *val, int64_t nbr, int64_t per_xcd,
                                                              int64_t nrows, int64_t ncols, const float *X,
                                                              int64_t N, int64_t ldx, float *Y, int64_t ldy,
                                                              int accumulate) {
  const int lane = lane_id();
  const int64_t br = xcd_tile(blockIdx.x, per_xcd) * 4 + wave_id();
  if (br >= nbr) return;
  const int64_t c = (int64_t)blockIdx.y * 64 + lane;
  const bool col_ok = c < N;
  const uint32_t xoff = (uint32_t)(col_ok ? c : N - 1);           // clamped: loads stay in bounds, stores are guarded
  // lane = 16u + 4k + r reads element 16u + 4r + k of the group's 64 values
  const uint32_t toff = (uint32_t)((lane & 48) | ((lane & 3) << 2) | ((lane >> 2) & 3));
  const uint32_t aoff = (uint32_t)(lane & 3) * 4u;                  // guarded path: row of the block this lane feeds
  const bool cols_divide = (ncols & 3) == 0;
  float4v acc = {0.f, 0.f, 0.f, 0.f};
  const int b0 = __builtin_amdgcn_readfirstlane(ptr[br]), b1 = __builtin_amdgcn_readfirstlane(ptr[br + 1]);
  for (int bb = b0; bb < b1; bb += 64) {
    const int cnt = min(64, b1 - bb);
    const int32_t my_bc = lane < cnt ? idx[bb + lane] : 0;   // block columns of the next 64 blocks, one per lane
    const int full = cols_divide ? cnt / (4 * R) * (4 * R) : 0;
    for (int j0 = 0; j0 < full; j0 += 4 * R) {
      float a[R];
      float xv[R][4][4];
#pragma unroll
      for (int g = 0; g < R; ++g) {
        a[g] = (val + (int64_t)(bb + j0 + 4 * g) * 16)[toff];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int64_t xr = (int64_t)__builtin_amdgcn_readlane(my_bc, j0 + 4 * g + u) * 4;
#pragma unroll
          for (int k = 0; k < 4; ++k) xv[g][u][k] = (X + (xr + k) * ldx)[xoff];
        }
      }
#pragma unroll
      for (int g = 0; g < R; ++g) {
        acc = mfma_bcast<0>(a[g], xv[g][0][0], acc);  acc = mfma_bcast<1>(a[g], xv[g][0][1], acc);
        acc = mfma_bcast<2>(a[g], xv[g][0][2], acc);  acc = mfma_bcast<3>(a[g], xv[g][0][3], acc);
        acc = mfma_bcast<4>(a[g], xv[g][1][0], acc);  acc = mfma_bcast<5>(a[g], xv[g][1][1], acc);
        acc = mfma_bcast<6>(a[g], xv[g][1][2], acc);  acc = mfma_bcast<7>(a[g], xv[g][1][3], acc);
        acc = mfma_bcast<8>(a[g], xv[g][2][0], acc);  acc = mfma_bcast<9>(a[g], xv[g][2][1], acc);
        acc = mfma_bcast<10>(a[g], xv[g][2][2], acc); acc = mfma_bcast<11>(a[g], xv[g][2][3], acc);
        acc = mfma_bcast<12>(a[g], xv[g][3][0], acc); acc = mfma_bcast<13>(a[g], xv[g][3][1], acc);
        acc = mfma_bcast<14>(a[g], xv[g][3][2], acc); acc = mfma_bcast<15>(a[g], xv[g][3][3], acc);
      }
    }
    for (int j = full; j < cnt; ++j) {   // guarded: leftover blocks, or a last block column that sticks out of the matrix
      const int64_t xr = (int64_t)__builtin_amdgcn_readlane(my_bc, j) * 4;
      const float4v av = *reinterpret_cast<const float4v *>(val + (int64_t)(bb + j) * 16 + aoff);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float x = xr + k < ncols ? X[(xr + k) * ldx + xoff] : 0.f;
        acc = __builtin_amdgcn_mfma_f32_4x4x1f32(av[k], x, acc, 0, 0, 0);
      }
    }
  }
  if (col_ok) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int64_t row = br * 4 + r;
      if (row < nrows) {
        float *yp = Y + row * ldy + c;
        *yp = (accumulate ? *yp : 0.f) + acc[r];
      }
    }
  }
}

// Blocked ELL with 4x4 blocks on the matrix cores: a wavefront owns one block row and 64 columns of X, as above; the
// blocks of a block row sit in the slots 0, 1, ... (slot-major slab, nbr blocks apart), so the block column is one
// scalar load per slot and every lane reads the row of the block that it feeds to the 4x4x1 product (lanes with
// equal lane % 4 read the same 16 bytes).  Four slots are in flight together: sixteen gathered rows of X.
__global__ __launch_bounds__(256) void bell44_spmm_mfma_kernel(const int32_t *ecol, const float *val, int64_t K,
                                                              int64_t nbr, int64_t per_xcd, int64_t nrows, int64_t ncols,
                                                              const float *X, int64_t N, int64_t ldx, float *Y,
                                                              int64_t ldy, int accumulate) {
  const int lane = lane_id();
  const int64_t br = xcd_tile(blockIdx.x, per_xcd) * 4 + wave_id();
  if (br >= nbr) return;
  const int64_t c = (int64_t)blockIdx.y * 64 + lane;
  const bool col_ok = c < N;
  const uint32_t xoff = (uint32_t)(col_ok ? c : N - 1);   // clamped: loads stay in bounds, stores are guarded
  const uint32_t aoff = (uint32_t)(lane & 3) * 4u;
  float4v acc = {0.f, 0.f, 0.f, 0.f};
  constexpr int S = 4;   // slots in flight together: 16 gathered rows of X (2: 1.10 ms, 4: 0.38 ms, 8: 0.58 ms on the FEM-like matrix)
  for (int64_t k0 = 0; k0 < K; k0 += S) {
    int32_t bc[S];
    float4v av[S];
    float xv[S][4];
#pragma unroll
    for (int u = 0; u < S; ++u)   // the block columns first (scalar loads), then everything that hangs on them
      bc[u] = k0 + u < K ? __builtin_amdgcn_readfirstlane(ecol[(k0 + u) * nbr + br]) : -1;
#pragma unroll
    for (int u = 0; u < S; ++u) {
      av[u] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) xv[u][kk] = 0.f;
      if (bc[u] >= 0) {   // (scalar)
        av[u] = *reinterpret_cast<const float4v *>(val + ((k0 + u) * nbr + br) * 16 + aoff);
        const int64_t xr = (int64_t)bc[u] * 4;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          if (xr + kk < ncols) xv[u][kk] = X[(xr + kk) * ldx + xoff];
      }
    }
    if (bc[0] < 0) break;   // slots fill from the front
#pragma unroll
    for (int u = 0; u < S; ++u)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) acc = __builtin_amdgcn_mfma_f32_4x4x1f32(av[u][kk], xv[u][kk], acc, 0, 0, 0);
  }
  if (col_ok) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t row = br * 4 + r;
      if (row < nrows) {
        float *yp = Y + row * ldy + c;
        *yp = (accumulate ? *yp : 0.f) + acc[r];
      }
    }
  }
}

// blocked ELL of any block size: one wavefront per (row, 64 columns), plain FMAs
__global__ __launch_bounds__(256) void bell_spmm_kernel(const int32_t *ecol, const float *val, int64_t K, int64_t nbr,
                                                       int bh, int bw, int64_t nrows, int64_t ncols, const float *X,
                                                       int64_t N, int64_t ldx, float *Y, int64_t ldy, int accumulate) {
  const int64_t i = (int64_t)blockIdx.x * 4 + wave_id();
  if (i >= nrows) return;
  const int64_t c = (int64_t)blockIdx.y * 64 + lane_id();
  if (c >= N) return;
  const int64_t br = i / bh;
  const int ri = (int)(i - br * bh);
  float s = accumulate ? Y[i * ldy + c] : 0.f;
  for (int64_t k = 0; k < K; ++k) {
    const int64_t bc = ecol[k * nbr + br];
    if (bc < 0) break;
    const float *v = val + ((k * nbr + br) * bh + ri) * bw;
    for (int q = 0; q < bw; ++q) {
      const int64_t j = bc * bw + q;
      if (j < ncols) s += v[q] * X[j * ldx + c];
    }
  }
  Y[i * ldy + c] = s;
}

// any block size: one wavefront per (block row, 64 columns), plain FMAs
// 1, 2 or 4 columns of X / Y per lane
template <int VEC> struct VecT;
template <> struct VecT<1> { typedef float type; };
template <> struct VecT<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct VecT<4> { typedef float type __attribute__((ext_vector_type(4))); };

// BCSR with blocks other than 4 x 4 (up to 64 values a block): a wavefront owns a block row x 64 * VEC columns and
// keeps one accumulator per row of the block.  One coalesced load brings the values of as many blocks as fit 64 lanes
// (and one their block columns); they are handed out by v_readlane (the position is the same for every lane: a
// scalar).  The columns of those blocks are walked eight at a time: eight rows of X in flight, each used for all bh
// rows of its block.  BHP = block height rounded up to a power of two (size of the register array).
// (One wavefront per block row that walked the blocks once per ROW of the block, re-reading X and loading every value
// as a 64-lane broadcast, took 10.4 ms for 8 x 8 blocks and 3.1 ms for 2 x 2 on the FEM-like matrix at N = 64; this
// takes 2.2 and 1.2 ms.  8 x 8 blocks there are three quarters padding and 64 multiply-adds a block: instruction issue.)
template <int VEC, int BHP>
__global__ __launch_bounds__(256) void bcsr_spmm_rows_kernel(const int32_t *ptr, const int32_t *idx, const float *val,
                                                            int64_t nbr, int bh, int bw, int64_t per_xcd, int64_t nrows,
                                                            int64_t ncols, const float *X, int64_t N, int64_t ldx, float *Y,
                                                            int64_t ldy, int accumulate) {
  typedef typename VecT<VEC>::type V;
  constexpr int U = 8;   // rows of X in flight
  const int lane = lane_id();
  const int64_t br = xcd_tile(blockIdx.x, per_xcd) * 4 + wave_id();
  if (br >= nbr) return;
  const int64_t c = ((int64_t)blockIdx.y * 64 + lane) * VEC;
  const bool col_ok = c < N;
  const uint32_t xoff = (uint32_t)(col_ok ? c : 0);   // clamped: loads stay in bounds, stores are guarded
  const int64_t row0 = br * bh;
  const int bsz = bh * bw, group = 64 / bsz;          // blocks whose values one load brings
  V acc[BHP];
#pragma unroll
  for (int r = 0; r < BHP; ++r)
    acc[r] = (accumulate && col_ok && r < bh && row0 + r < nrows) ? *reinterpret_cast<const V *>(Y + (row0 + r) * ldy + c) : V(0.f);
  const int b1 = ptr[br + 1];
  for (int b0 = ptr[br]; b0 < b1; b0 += group) {
    const int nb = min(group, b1 - b0);
    const int vmine = __builtin_bit_cast(int, lane < nb * bsz ? val[(int64_t)b0 * bsz + lane] : 0.f);
    const int cmine = lane < nb ? idx[b0 + lane] : 0;
    // the nb * bw columns of these blocks, U at a time; (g, k) = block in the group, column in the block
    const int nslots = nb * bw;
    int g = 0, k = 0;
    for (int s0 = 0; s0 < nslots; s0 += U) {
      V xv[U];
      int at[U];   // lane of vmine that holds row 0 of the slot's column
#pragma unroll
      for (int u = 0; u < U; ++u) {   // (everything here is the same for every lane: scalar arithmetic and branches)
        const int64_t xr = (int64_t)__builtin_amdgcn_readlane(cmine, g) * bw + k;
        const bool live = s0 + u < nslots && xr < ncols;
        xv[u] = live ? *reinterpret_cast<const V *>(X + xr * ldx + xoff) : V(0.f);
        at[u] = live ? g * bsz + k : -1;
        if (++k == bw) { k = 0; g = g + 1 < nb ? g + 1 : g; }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (at[u] >= 0) {
#pragma unroll
          for (int r = 0; r < BHP; ++r)
            if (r < bh) acc[r] += __builtin_bit_cast(float, __builtin_amdgcn_readlane(vmine, at[u] + r * bw)) * xv[u];
        }
      }
    }
  }
  if (col_ok) {
#pragma unroll
    for (int r = 0; r < BHP; ++r)
      if (r < bh && row0 + r < nrows) *reinterpret_cast<V *>(Y + (row0 + r) * ldy + c) = acc[r];
  }
}

// BDIA: the same shape of work.  A node is a piece of a diagonal, bh consecutive rows long: its values are one load,
// its rows of X are consecutive, and a wavefront owns the block row x 64 * VEC columns with one accumulator per row.
template <int VEC, int BHP>
__global__ __launch_bounds__(256) void bdia_spmm_rows_kernel(const int32_t *ptr, const int32_t *off, const float *val,
                                                            int64_t nbr, int bh, int64_t per_xcd, int64_t nrows, int64_t ncols,
                                                            const float *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                                                            int accumulate) {
  typedef typename VecT<VEC>::type V;
  const int lane = lane_id();
  const int64_t br = xcd_tile(blockIdx.x, per_xcd) * 4 + wave_id();
  if (br >= nbr) return;
  const int64_t c = ((int64_t)blockIdx.y * 64 + lane) * VEC;
  const bool col_ok = c < N;
  const uint32_t xoff = (uint32_t)(col_ok ? c : 0);
  const int64_t row0 = br * bh;
  V acc[BHP];
#pragma unroll
  for (int r = 0; r < BHP; ++r)
    acc[r] = (accumulate && col_ok && r < bh && row0 + r < nrows) ? *reinterpret_cast<const V *>(Y + (row0 + r) * ldy + c) : V(0.f);
  constexpr int J = BHP >= 8 ? 1 : 8 / BHP;   // nodes taken together: eight rows of X in flight
  const int n1 = ptr[br + 1];
  for (int n0 = ptr[br]; n0 < n1; n0 += J) {
    int vmine[J];
    V xv[J][BHP];
#pragma unroll
    for (int q = 0; q < J; ++q) {
      const bool live = n0 + q < n1;           // the same for every lane
      const int64_t o = live ? off[n0 + q] : 0;
      vmine[q] = __builtin_bit_cast(int, (live && lane < bh) ? val[(int64_t)(n0 + q) * bh + lane] : 0.f);
#pragma unroll
      for (int r = 0; r < BHP; ++r) {
        const int64_t j = row0 + r + o;
        xv[q][r] = (live && r < bh && row0 + r < nrows && j >= 0 && j < ncols) ? *reinterpret_cast<const V *>(X + j * ldx + xoff) : V(0.f);
      }
    }
#pragma unroll
    for (int q = 0; q < J; ++q)
#pragma unroll
      for (int r = 0; r < BHP; ++r)
        if (r < bh) acc[r] += __builtin_bit_cast(float, __builtin_amdgcn_readlane(vmine[q], r)) * xv[q][r];
  }
  if (col_ok) {
#pragma unroll
    for (int r = 0; r < BHP; ++r)
      if (r < bh && row0 + r < nrows) *reinterpret_cast<V *>(Y + (row0 + r) * ldy + c) = acc[r];
  }
}

__global__ __launch_bounds__(256) void bcsr_spmm_kernel(const int32_t *ptr, const int32_t *idx, const float *val,
                                                       int64_t nbr, int bh, int bw, int64_t nrows, int64_t ncols,
                                                       const float *X, int64_t N, int64_t ldx, float *Y,
                                                       int64_t ldy, int accumulate) {
  const int lane = lane_id();
  const int64_t br = (int64_t)blockIdx.x * 4 + wave_id();
  if (br >= nbr) return;
  const int64_t c = (int64_t)blockIdx.y * 64 + lane;
  if (c >= N) return;
  const int bsz = bh * bw;
  for (int r = 0; r < bh; ++r) {
    int64_t row = br * bh + r;
    if (row >= nrows) break;
    float s = accumulate ? Y[row * ldy + c] : 0.f;
    for (int b = ptr[br]; b < ptr[br + 1]; ++b)
      for (int k = 0; k < bw; ++k) {
        int64_t xr = (int64_t)idx[b] * bw + k;
        if (xr < ncols) s += val[(int64_t)b * bsz + r * bw + k] * X[xr * ldx + c];
      }
    Y[row * ldy + c] = s;
  }
}

// ------------------------------------------------------------------ row-grouped layouts, one wavefront per (row, 64 columns)
// A lane owns VEC consecutive columns (VEC = 2 covers N = 128 with one wavefront per row).

// ELL: a wavefront owns 8 consecutive rows.  One coalesced load brings the column indices and values
// of 8 slots x 8 rows (lane = slot*8 + row); they are handed out by v_readlane, i.e. as scalars, so
// the address of a gathered row is scalar arithmetic plus a fixed per-lane offset, the gather of a pad
// slot is skipped by a scalar branch (two thirds of the slots of a percentile-wide slab are pads; its
// operand is a zero, written unconditionally: a vector-typed register array assigned only inside
// branches makes the compiler copy it per branch, 46 -> 300 VGPRs), and up to 8 independent
// 256/512-byte gathers per wavefront are in flight.
// Workgroups are dealt round-robin to the 8 XCDs; launch index -> row tile goes through xcd_tile so
// that each XCD sweeps one contiguous range of rows and the rows of X that neighbouring matrix rows
// share (local columns) are found again in that XCD's L2.
template <int VEC>
__global__ __launch_bounds__(256) void ell_spmm_kernel(const int32_t *ecol, const float *ev, int64_t K, int64_t nrows,
                                                      int64_t per_xcd, const float *X, int64_t N, int64_t ldx, float *Y,
                                                      int64_t ldy, int accumulate) {
  typedef typename VecT<VEC>::type V;
  const int lane = lane_id();
  const int64_t i0 = (xcd_tile(blockIdx.x, per_xcd) * 4 + wave_id()) * 8;
  if (i0 >= nrows) return;
  const int64_t c = ((int64_t)blockIdx.y * 64 + lane) * VEC;
  const bool col_ok = c < N;
  const uint32_t xoff = (uint32_t)(col_ok ? c : 0);   // clamped: loads stay in bounds (N >= VEC), stores are guarded
  V acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r)
    acc[r] = (accumulate && col_ok && i0 + r < nrows) ? *reinterpret_cast<const V *>(Y + (i0 + r) * ldy + c) : V(0.f);
  const int my_slot = lane >> 3, my_row = lane & 7;
  for (int64_t k0 = 0; k0 < K; k0 += 8) {
    const int64_t kk = k0 + my_slot, i = i0 + my_row;
    const bool ok = kk < K && i < nrows;
    const int32_t mycol = ok ? __builtin_nontemporal_load(ecol + kk * nrows + i) : -1;
    const float myval = ok ? __builtin_nontemporal_load(ev + kk * nrows + i) : 0.f;
    const uint64_t live = __ballot(mycol >= 0);   // bit slot*8 + row
    if (live == 0) break;  // slots fill from the front: all 8 rows have ended
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) {
      const uint32_t live8 = (uint32_t)(live >> (s8 * 8)) & 0xFFu;   // scalar: which of the 8 rows have this slot
      if (live8 == 0) break;
      V xv[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        xv[r] = V(0.f);
        if (live8 & (1u << r)) {
          const int64_t cs = __builtin_amdgcn_readlane(mycol, s8 * 8 + r);
          xv[r] = *reinterpret_cast<const V *>(X + cs * ldx + xoff);
        }
      }
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const float vs = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, myval), s8 * 8 + r));
        acc[r] += vs * xv[r];
      }
    }
  }
  if (col_ok) {
#pragma unroll
    for (int r = 0; r < 8; ++r)
      if (i0 + r < nrows) *reinterpret_cast<V *>(Y + (i0 + r) * ldy + c) = acc[r];
  }
}

// DIA (and the DIA variant, whose slab is indexed by column): a wavefront owns 8 consecutive rows x 64 * VEC columns.
// For diagonal k the 8 rows read 8 consecutive rows of X, so the loads of one diagonal are independent and in
// flight together, the 8 values of the diagonal are one load handed out by v_readlane (scalars), and a row of X
// that the other diagonals use again is found in the L2 of the XCD, which walks a contiguous range of row tiles
// (offsets up to a few thousand rows: a window of a megabyte or two).
// (Measured on the seven diagonals of the banded workload, N = 64: 1.09 ms with one wavefront per row and a
// broadcast load per value, 0.41 ms this way = 2.75 TB/s on the compulsory bytes, and the counters show no byte
// fetched twice.  Four diagonals' loads in flight together, or four 8-row steps per wavefront, changed nothing:
// what is left is the L2, which serves every row of X once per diagonal, 9 TB/s at this speed.)
constexpr int DIA_R = 8;
template <int VEC>
__global__ __launch_bounds__(256) void dia_spmm_rows_kernel(const int32_t *off, const float *val, int64_t ndiag,
                                                           int64_t nrows, int64_t ncols, int by_col, int64_t per_xcd,
                                                           const float *X, int64_t N, int64_t ldx, float *Y,
                                                           int64_t ldy, int accumulate) {
  typedef typename VecT<VEC>::type V;
  constexpr int R = DIA_R;
  const int lane = lane_id();
  const int64_t i0 = (xcd_tile(blockIdx.x, per_xcd) * 4 + wave_id()) * R;
  if (i0 >= nrows) return;
  const int64_t c = ((int64_t)blockIdx.y * 64 + lane) * VEC;
  const bool col_ok = c < N;
  const uint32_t xoff = (uint32_t)(col_ok ? c : 0);   // clamped: loads stay in bounds, stores are guarded
  V acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r)
    acc[r] = (accumulate && col_ok && i0 + r < nrows) ? *reinterpret_cast<const V *>(Y + (i0 + r) * ldy + c) : V(0.f);
  const int64_t slab = by_col ? ncols : nrows;
  for (int64_t k = 0; k < ndiag; ++k) {
    const int64_t o = off[k];
    // lane r < R: the value of row i0 + r on this diagonal (zero where the diagonal leaves the matrix)
    const int64_t i = i0 + lane, j = i + o;
    const bool in = lane < R && i < nrows && j >= 0 && j < ncols;
    const float mine = in ? val[k * slab + (by_col ? j : i)] : 0.f;
    V xv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t jr = i0 + r + o;   // the same for every lane: a scalar branch
      xv[r] = (i0 + r < nrows && jr >= 0 && jr < ncols) ? *reinterpret_cast<const V *>(X + jr * ldx + xoff) : V(0.f);
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
      acc[r] += __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine), r)) * xv[r];
  }
  if (col_ok) {
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (i0 + r < nrows) *reinterpret_cast<V *>(Y + (i0 + r) * ldy + c) = acc[r];
  }
}


// ------------------------------------------------------------------ entries grouped by row (COO sorted by row, CSR, DCSR): equal shares of non-zeros per wavefront
// The row of entry e is read from the COO row array, or found in ptr (plus the stored-row list
// for DCSR), so a 20,000-entry row costs the same as 20,000 one-entry rows.
struct RowSrc {
  const int32_t *row;   // COO: row of every entry, else null
  const int32_t *ptr;   // CSR / DCSR: children of parent p are [ptr[p], ptr[p+1])
  const int32_t *ids;   // DCSR: row index of parent p, else null
  int64_t nparents;
  __device__ __forceinline__ int32_t of(int64_t e) const {
    if (row) return __builtin_nontemporal_load(row + e);
    int64_t p = parent_of(ptr, nparents, e);
    return ids ? ids[p] : (int32_t)p;
  }
};

// A wavefront walks CS_CHUNK consecutive entries; for each it adds val * X[col, :] into a
// register accumulator and flushes when the row changes.  Row pieces cut by a chunk boundary
// go to a carry buffer and are summed in chunk order by the fix-up kernel (reproducible).
constexpr int CS_CHUNK = 512;
// ... or fewer when the list is short: a wavefront's entries are a serial chain of gather rounds (eight rows of X at a
// time), so 147 k entries cut into 287 chunks kept 287 wavefronts busy for 64 rounds each, 0.26 ms on a part with
// 1024 SIMDs; chunks of 64 entries make it 2,293 wavefronts of 8 rounds.
static int chunk_entries(int64_t nnz) {
  int len = CS_CHUNK;
  while (len > 64 && nnz / len < 8192) len >>= 1;
  return len;
}

// SEARCH (rows found in ptr): the rows of the whole chunk are looked up first and kept in LDS: the parents of the two
// entries around the chunk by bisection over all parents, then eight entries per lane with their bisections between
// those two in step.  One full bisection after the other (per batch of 64 entries, plus four for the chunk's ends) is
// ~250 dependent loads -- a remainder of 147 k entries in 2 M rows, a few hundred wavefronts that all run at once, took
// 0.32 ms of pure latency that way -- and twenty scattered loads per entry where the rows of a chunk are a handful.
template <int VEC, bool SEARCH>
__global__ __launch_bounds__(256) void coo_spmm_kernel(RowSrc row, const int32_t *col, const float *val,
                                                      int64_t nnz, int chunk_len, int64_t per_xcd, const float *X, int64_t N,
                                                      int64_t ldx, float *Y, int64_t ldy, int32_t *carry_row, float *carry) {
  typedef typename VecT<VEC>::type V;
  constexpr int PER_LANE = CS_CHUNK / 64;   // slots of the look-up: chunk_len <= CS_CHUNK
  __shared__ int32_t s_rows[SEARCH ? 4 : 1][SEARCH ? CS_CHUNK : 1];
  const int lane = lane_id();
  // launch index -> chunk through xcd_tile: an XCD walks one contiguous range of entries (rows), so the
  // rows of X that neighbouring matrix rows share are found again in its own L2
  const int64_t chunk = xcd_tile(blockIdx.x, per_xcd) * 4 + wave_id();
  const int64_t e0 = chunk * chunk_len;
  if (e0 >= nnz) return;
  const int64_t e1 = min(e0 + chunk_len, nnz);
  const int64_t c = ((int64_t)blockIdx.y * 64 + lane) * VEC;
  const bool col_ok = c < N;
  const uint32_t xoff = (uint32_t)(col_ok ? c : 0);   // clamped: loads stay in bounds, stores are guarded
  int32_t row_before, row_after, first_row, last_row;
  if constexpr (SEARCH) {
    // parents of the entries just before and just after the chunk: two bisections over all parents, in step, the same
    // for every lane (ptr[p] <= e < ptr[p + 1])
    const int64_t eb = e0 > 0 ? e0 - 1 : e0, ea = e1 < nnz ? e1 : e1 - 1;
    int32_t blo = 0, bhi = (int32_t)row.nparents, alo = 0, ahi = (int32_t)row.nparents;
    while (blo < bhi || alo < ahi) {
      if (blo < bhi) {
        const int32_t mid = blo + ((bhi - blo) >> 1);
        if ((int64_t)row.ptr[mid + 1] <= eb) blo = mid + 1; else bhi = mid;
      }
      if (alo < ahi) {
        const int32_t mid = alo + ((ahi - alo) >> 1);
        if ((int64_t)row.ptr[mid + 1] <= ea) alo = mid + 1; else ahi = mid;
      }
    }
    // every entry of the chunk has its parent between those two: PER_LANE entries per lane, their bisections over
    // that range in step (a chunk inside one long row needs none, 96-entry rows three steps instead of twenty)
    int32_t lo[PER_LANE], hi[PER_LANE];
#pragma unroll
    for (int q = 0; q < PER_LANE; ++q) {
      const bool live = e0 + q * 64 + lane < e1;
      lo[q] = blo; hi[q] = live ? alo : blo;
    }
    for (bool more = true; more;) {
      more = false;
#pragma unroll
      for (int q = 0; q < PER_LANE; ++q) {
        if (lo[q] < hi[q]) {
          const int32_t mid = lo[q] + ((hi[q] - lo[q]) >> 1);
          if ((int64_t)row.ptr[mid + 1] <= e0 + q * 64 + lane) lo[q] = mid + 1; else hi[q] = mid;
          more = true;
        }
      }
      more = __any(more);
    }
#pragma unroll
    for (int q = 0; q < PER_LANE; ++q)
      if (e0 + q * 64 + lane < e1) s_rows[wave_id()][q * 64 + lane] = row.ids ? row.ids[lo[q]] : lo[q];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    row_before = e0 > 0 ? (row.ids ? row.ids[blo] : blo) : -1;
    row_after = e1 < nnz ? (row.ids ? row.ids[alo] : alo) : -1;
    first_row = s_rows[wave_id()][0]; last_row = s_rows[wave_id()][e1 - 1 - e0];
  } else {
    row_before = e0 > 0 ? row.of(e0 - 1) : -1;
    row_after = e1 < nnz ? row.of(e1) : -1;
    first_row = row.of(e0); last_row = row.of(e1 - 1);
  }
  V *carry_head = reinterpret_cast<V *>(carry + ((chunk * 2 + 0) * gridDim.y + blockIdx.y) * (64 * VEC)) + lane;
  V *carry_tail = reinterpret_cast<V *>(carry + ((chunk * 2 + 1) * gridDim.y + blockIdx.y) * (64 * VEC)) + lane;
  const bool head_cut = first_row == row_before, tail_cut = last_row == row_after;
  V acc = V(0.f);
  int32_t cur = first_row;
  bool in_head = true;  // still inside the first row piece of the chunk
  constexpr int U = 8;
  for (int64_t base = e0; base < e1; base += 64) {
    const int64_t e = base + lane;
    int32_t r = -1;
    if (e < e1) {
      if constexpr (SEARCH) r = s_rows[wave_id()][e - e0]; else r = row.of(e);
    }
    const int32_t cc = e < e1 ? __builtin_nontemporal_load(col + e) : 0;
    const float v = e < e1 ? __builtin_nontemporal_load(val + e) : 0.f;
    const int cnt = (int)min((int64_t)64, e1 - base);
    for (int t0 = 0; t0 < cnt; t0 += U) {
      // row, column and value of entry t are scalars (v_readlane): the gather address is scalar
      // arithmetic plus a fixed per-lane offset and the row-change test is a scalar branch
      int32_t rt[U];
      float vt[U];
      V xv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {   // 8 gathers of X rows in flight
        const int t = t0 + u < cnt ? t0 + u : cnt - 1;
        rt[u] = __builtin_amdgcn_readlane(r, t);
        vt[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), t));
        const int64_t ct = __builtin_amdgcn_readlane(cc, t);
        xv[u] = *reinterpret_cast<const V *>(X + ct * ldx + xoff);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (t0 + u < cnt) {
          if (rt[u] != cur) {  // flush the finished piece of row `cur`
            if (col_ok) {
              if (in_head && head_cut) *carry_head = acc;
              else { V *yp = reinterpret_cast<V *>(Y + (int64_t)cur * ldy + c); *yp += acc; }
            }
            in_head = false;
            acc = V(0.f);
            cur = rt[u];
          }
          acc += vt[u] * xv[u];
        }
      }
    }
  }
  // last piece
  const bool single = in_head;  // the whole chunk lies inside one row
  if (col_ok) {
    V *yp = reinterpret_cast<V *>(Y + (int64_t)cur * ldy + c);
    if (single) {
      if (head_cut || tail_cut) { *carry_head = acc; *carry_tail = V(0.f); }
      else *yp += acc;
    } else {
      if (tail_cut) *carry_tail = acc;
      else *yp += acc;
    }
  }
  if (lane == 0 && blockIdx.y == 0) {
    bool head_used = single ? (head_cut || tail_cut) : head_cut;
    bool tail_used = single ? (head_cut || tail_cut) : tail_cut;
    carry_row[chunk * 2 + 0] = head_used ? first_row : -1;
    carry_row[chunk * 2 + 1] = tail_used ? last_row : -1;
  }
}

__global__ __launch_bounds__(256) void coo_spmm_fixup_kernel(const int32_t *carry_row, const float *carry,
                                                            int64_t nentries, int64_t ncb, int cbw, int64_t N,
                                                            float *Y, int64_t ldy) {
  const int lane = lane_id();
  const int64_t e = (int64_t)blockIdx.x * 4 + wave_id();
  if (e >= nentries) return;
  const int32_t r = carry_row[e];
  if (r < 0) return;
  // only the first entry of the run of row r works (a run never skips an entry, see above)
  if (e > 0 && carry_row[e - 1] == r) return;
  // length of the run, 64 entries per look (a 20,000-entry row leaves ~80 pieces: walking them one
  // dependent load at a time made this kernel the tail of the whole product)
  int64_t len = 0;
  for (;;) {
    const int64_t j = e + len + lane;
    const uint64_t same = __ballot(j < nentries && carry_row[j] == r);
    const int run = same == ~0ull ? 64 : __ffsll((unsigned long long)~same) - 1;
    len += run;
    if (run < 64) break;
  }
  for (int q = lane; q < cbw; q += 64) {
    const int64_t c = (int64_t)blockIdx.y * cbw + q;
    if (c >= N) continue;
    const float *p = carry + (e * ncb + blockIdx.y) * cbw + q;
    const int64_t stride = ncb * cbw;
    float s = 0.f;
    int64_t j = 0;
    for (; j + 8 <= len; j += 8) {   // 8 independent loads in flight, added in piece order
      float t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = p[(j + u) * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += t[u];
    }
    for (; j < len; ++j) s += p[j * stride];
    Y[(int64_t)r * ldy + c] += s;
  }
}

// scatter form for CSC / DCSC: one wavefront per (stored column, 64 columns of X)
__global__ __launch_bounds__(256) void csc_spmm_atomic_kernel(const int32_t *ptr, const int32_t *idx, const float *val,
                                                             const int32_t *col_ids, int64_t ncols_stored,
                                                             const float *X, int64_t N, int64_t ldx, float *Y,
                                                             int64_t ldy) {
  const int64_t j = (int64_t)blockIdx.x * 4 + wave_id();
  if (j >= ncols_stored) return;
  const int64_t cc = (int64_t)blockIdx.y * 64 + lane_id();
  if (cc >= N) return;
  const float xv = X[(int64_t)(col_ids ? col_ids[j] : j) * ldx + cc];
  for (int e = ptr[j]; e < ptr[j + 1]; ++e) atomicAdd(&Y[(int64_t)idx[e] * ldy + cc], val[e] * xv);
}

// CSB: the entries lie in (block row, block column, in-block row, in-block column) order, so a wavefront that walks
// a chunk of consecutive entries meets every row of a block as one run.  It looks up the block of each of its
// entries first (the blocks of the chunk's two ends by bisection over all blocks, the others between those two),
// keeps row and column in LDS, then works like the row-major kernel: row, column and value of an entry are scalars,
// eight rows of X in flight, one accumulator, flushed when the row changes.  Other blocks of the block row (in other
// chunks) add to the same rows of Y, so a flush is an fp32 atomic add (not bit-reproducible): one per run and column,
// where one wavefront per entry did one per entry and column and a bisection over all blocks each time (45.7 ms for
// 50 M entries in 512 x 512 blocks at N = 64).
template <int VEC>
__global__ __launch_bounds__(256) void csb_spmm_kernel(const int32_t *ptr, const int32_t *in_row, const int32_t *in_col,
                                                      const float *val, int64_t n, int chunk_len, int64_t per_xcd,
                                                      int64_t nblocks, int64_t nbc, int64_t bh, int64_t bw, const float *X,
                                                      int64_t N, int64_t ldx, float *Y, int64_t ldy) {
  typedef typename VecT<VEC>::type V;
  __shared__ int32_t s_row[4][CS_CHUNK], s_col[4][CS_CHUNK];
  const int lane = lane_id(), w = wave_id();
  const int64_t chunk = xcd_tile(blockIdx.x, per_xcd) * 4 + w;
  const int64_t e0 = chunk * chunk_len;
  if (e0 >= n) return;
  const int64_t e1 = min(e0 + chunk_len, n);
  const int64_t c = ((int64_t)blockIdx.y * 64 + lane) * VEC;
  const bool col_ok = c < N;
  const uint32_t xoff = (uint32_t)(col_ok ? c : 0);   // clamped: loads stay in bounds, stores are guarded
  const int64_t blk_first = parent_of(ptr, nblocks, e0), blk_last = parent_of(ptr, nblocks, e1 - 1);
  for (int64_t e = e0 + lane; e < e1; e += 64) {
    int64_t lo = blk_first, hi = blk_last;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)ptr[mid + 1] <= e) lo = mid + 1; else hi = mid;
    }
    s_row[w][e - e0] = (int32_t)((lo / nbc) * bh + in_row[e]);
    s_col[w][e - e0] = (int32_t)((lo % nbc) * bw + in_col[e]);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  auto flush = [&](int32_t row, const V &acc) {
    if (!col_ok) return;
    float *yp = Y + (int64_t)row * ldy + c;
    if constexpr (VEC == 1) atomicAdd(yp, acc);
    else {
#pragma unroll
      for (int i = 0; i < VEC; ++i) atomicAdd(yp + i, acc[i]);
    }
  };
  V acc = V(0.f);
  int32_t cur = s_row[w][0];
  constexpr int U = 8;
  for (int64_t base = e0; base < e1; base += 64) {
    const int64_t e = base + lane;
    const int32_t r = e < e1 ? s_row[w][e - e0] : -1, cc = e < e1 ? s_col[w][e - e0] : 0;
    const float v = e < e1 ? __builtin_nontemporal_load(val + e) : 0.f;
    const int cnt = (int)min((int64_t)64, e1 - base);
    for (int t0 = 0; t0 < cnt; t0 += U) {
      int32_t rt[U];
      float vt[U];
      V xv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int t = t0 + u < cnt ? t0 + u : cnt - 1;
        rt[u] = __builtin_amdgcn_readlane(r, t);
        vt[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), t));
        const int64_t ct = __builtin_amdgcn_readlane(cc, t);
        xv[u] = *reinterpret_cast<const V *>(X + ct * ldx + xoff);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (t0 + u < cnt) {
          if (rt[u] != cur) {
            flush(cur, acc);
            acc = V(0.f);
            cur = rt[u];
          }
          acc += vt[u] * xv[u];
        }
      }
    }
  }
  flush(cur, acc);
}

// scatter form for the column-major COO
__global__ __launch_bounds__(256) void coo_spmm_atomic_kernel(const int32_t *r, const int32_t *c, const float *val,
                                                             int64_t nnz, const float *X, int64_t N, int64_t ldx,
                                                             float *Y, int64_t ldy) {
  const int64_t e = (int64_t)blockIdx.x * 4 + wave_id();
  if (e >= nnz) return;
  const int64_t cc = (int64_t)blockIdx.y * 64 + lane_id();
  if (cc < N) atomicAdd(&Y[(int64_t)r[e] * ldy + cc], val[e] * X[(int64_t)c[e] * ldx + cc]);
}

// Y[i][0..N) = 0 for a Y whose rows are ldy > N apart (the columns past N are the caller's and stay untouched)
__global__ __launch_bounds__(256) void zero_rows_kernel(float *Y, int64_t nrows, int64_t N, int64_t ldy) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= nrows * N) return;
  const int64_t i = e / N;
  Y[i * ldy + (e - i * N)] = 0.f;
}

static void zero_rows(Env &env, float *Y, int64_t nrows, int64_t N, int64_t ldy) {
  if (ldy == N) { fill_u32(env, (uint32_t *)Y, (uint64_t)nrows * N, 0u); return; }
  if (nrows > 0)
    US_LAUNCH(env, "zero_rows", 4.0 * nrows * N, zero_rows_kernel, ceil_div<int64_t>(nrows * N, 256), 256, Y, nrows, N, ldy);
}

// scratch of the entry-balanced product: two carry rows per chunk (row index + one value per column of the lane layout)
static size_t carry_rows_bytes(int64_t nnz) {
  return ((size_t)ceil_div<int64_t>(nnz, chunk_entries(nnz)) * 2 * sizeof(int32_t) + 255) / 256 * 256;
}
size_t entry_balanced_scratch_bytes(int64_t nnz, int64_t N, int vec) {
  const int cbw = 64 * vec;
  return carry_rows_bytes(nnz) +
         (size_t)ceil_div<int64_t>(nnz, chunk_entries(nnz)) * 2 * ceil_div<int64_t>(N, cbw) * cbw * sizeof(float);
}

static void entry_balanced_spmm(Env &env, const us_formatted &A, const RowSrc &rs, const int32_t *col,
                                const char *name, int vec, const float *X, int64_t N, int64_t ldx, float *Y,
                                int64_t ldy) {
  // Y must already hold the values to add to (zeros for a plain product)
  const double xy = 4.0 * N * (A.ncols + A.nrows);
  const int chunk_len = chunk_entries(A.nnz);
  const int64_t nchunks = ceil_div<int64_t>(A.nnz, chunk_len);
  const size_t rows_pad = carry_rows_bytes(A.nnz);
  const int cbw = 64 * vec;
  const int64_t ncbv = ceil_div<int64_t>(N, cbw);
  char *ws = (char *)ensure_workspace(env, A, entry_balanced_scratch_bytes(A.nnz, N, vec));
  if (!env.ok()) return;
  int32_t *carry_row = (int32_t *)ws;
  float *carry = (float *)(ws + rows_pad);
  {
    LaunchScope ls(env, name, 12.0 * A.nnz + xy);
    const int64_t per_xcd = ceil_div<int64_t>(ceil_div<int64_t>(nchunks, 4), 8);
    const dim3 grid((unsigned)(per_xcd * 8), (unsigned)ncbv);
#define US_EB_LAUNCH(V, S) hipLaunchKernelGGL((coo_spmm_kernel<V, S>), grid, dim3(256), 0, env.stream, rs, col, (const float *)A.val, A.nnz, chunk_len, per_xcd, X, N, ldx, Y, ldy, carry_row, carry)
    if (rs.row) {
      if (vec == 4) US_EB_LAUNCH(4, false); else if (vec == 2) US_EB_LAUNCH(2, false); else US_EB_LAUNCH(1, false);
    } else {
      if (vec == 4) US_EB_LAUNCH(4, true); else if (vec == 2) US_EB_LAUNCH(2, true); else US_EB_LAUNCH(1, true);
    }
#undef US_EB_LAUNCH
    env.check(hipGetLastError());
  }
  if (env.ok()) {
    LaunchScope ls(env, "spmm_rows_fixup", 8.0 * nchunks);
    hipLaunchKernelGGL(coo_spmm_fixup_kernel, dim3((unsigned)ceil_div<int64_t>(nchunks * 2, 4), (unsigned)ncbv),
                       dim3(256), 0, env.stream, (const int32_t *)carry_row, (const float *)carry, nchunks * 2, ncbv,
                       cbw, N, Y, ldy);
    env.check(hipGetLastError());
  }
}

us_status spmm_impl(Env &env, const us_formatted &A, const float *X, int64_t N, int64_t ldx, float *Y, int64_t ldy,
                    bool accumulate) {
  const int64_t ncb = ceil_div<int64_t>(N, 64);
  const int acc = accumulate ? 1 : 0;
  // columns per lane for the gather kernels: vector loads need aligned rows
  const bool al16 = ((uintptr_t)X % 16 == 0) && ((uintptr_t)Y % 16 == 0);
  const int vec = (al16 && N % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && N >= 256) ? 4
                  : (al16 && N % 2 == 0 && ldx % 2 == 0 && ldy % 2 == 0 && N >= 128) ? 2 : 1;
  const double xy = 4.0 * N * (A.ncols + A.nrows);
  switch (A.pattern) {
    case P_BCSR: {
      if (A.bh == 4 && A.bw == 4) {
        const int64_t tiles = ceil_div<int64_t>(A.nmajor, 4), per_xcd = ceil_div<int64_t>(tiles, 8);
        if (env.ok()) {
          LaunchScope ls(env, "spmm_bcsr44_mfma", 4.0 * A.nval + 4.0 * A.nblk + 4.0 * (A.nmajor + 1) + xy);
          hipLaunchKernelGGL(bcsr44_spmm_mfma_kernel<BCSR_R>, dim3((unsigned)(per_xcd * 8), (unsigned)ncb), dim3(256), 0,
                             env.stream, (const int32_t *)A.level[1].ptr, (const int32_t *)A.level[1].idx,
                             (const float *)A.val, A.nmajor, per_xcd, A.nrows, A.ncols, X, N, ldx, Y, ldy, acc);
          env.check(hipGetLastError());
        }
      } else if (env.ok() && A.bh * A.bw <= 64) {
        LaunchScope ls(env, "spmm_bcsr", 4.0 * A.nval + 4.0 * A.nblk + xy);
        const int64_t tiles = ceil_div<int64_t>(A.nmajor, 4), per_xcd = ceil_div<int64_t>(tiles, 8);
        const dim3 grid((unsigned)(per_xcd * 8), (unsigned)ceil_div<int64_t>(N, 64 * vec));
#define US_BCSR_LAUNCH(V, H) hipLaunchKernelGGL((bcsr_spmm_rows_kernel<V, H>), grid, dim3(256), 0, env.stream, (const int32_t *)A.level[1].ptr, (const int32_t *)A.level[1].idx, (const float *)A.val, A.nmajor, (int)A.bh, (int)A.bw, per_xcd, A.nrows, A.ncols, X, N, ldx, Y, ldy, acc)
#define US_BCSR_BY_HEIGHT(V) do { if (A.bh <= 2) US_BCSR_LAUNCH(V, 2); else if (A.bh <= 4) US_BCSR_LAUNCH(V, 4); else if (A.bh <= 8) US_BCSR_LAUNCH(V, 8); else US_BCSR_LAUNCH(V, 16); } while (0)
        if (vec == 4) US_BCSR_BY_HEIGHT(4); else if (vec == 2) US_BCSR_BY_HEIGHT(2); else US_BCSR_BY_HEIGHT(1);
#undef US_BCSR_BY_HEIGHT
#undef US_BCSR_LAUNCH
        env.check(hipGetLastError());
      } else if (env.ok()) {   // blocks of more than 64 values: the plain loop
        LaunchScope ls(env, "spmm_bcsr", 4.0 * A.nval + 4.0 * A.nblk + xy);
        hipLaunchKernelGGL(bcsr_spmm_kernel, dim3((unsigned)ceil_div<int64_t>(A.nmajor, 4), (unsigned)ncb), dim3(256),
                           0, env.stream, (const int32_t *)A.level[1].ptr, (const int32_t *)A.level[1].idx,
                           (const float *)A.val, A.nmajor, (int)A.bh, (int)A.bw, A.nrows, A.ncols, X, N, ldx, Y, ldy, acc);
        env.check(hipGetLastError());
      }
      return env.status;
    }
    case P_BELL:
      if (env.ok()) {
        const double bytes = 4.0 * A.nval + 4.0 * A.level[2].nidx + xy;
        if (A.bh == 4 && A.bw == 4) {
          LaunchScope ls(env, "spmm_bell44_mfma", bytes);
          const int64_t tiles = ceil_div<int64_t>(A.nblk, 4), per_xcd = ceil_div<int64_t>(tiles, 8);
          hipLaunchKernelGGL(bell44_spmm_mfma_kernel, dim3((unsigned)(per_xcd * 8), (unsigned)ncb), dim3(256), 0, env.stream,
                             (const int32_t *)A.level[2].idx, (const float *)A.val, A.nmajor, A.nblk, per_xcd, A.nrows,
                             A.ncols, X, N, ldx, Y, ldy, acc);
        } else {
          LaunchScope ls(env, "spmm_bell", bytes);
          hipLaunchKernelGGL(bell_spmm_kernel, dim3((unsigned)ceil_div<int64_t>(A.nrows, 4), (unsigned)ncb), dim3(256), 0,
                             env.stream, (const int32_t *)A.level[2].idx, (const float *)A.val, A.nmajor, A.nblk, (int)A.bh,
                             (int)A.bw, A.nrows, A.ncols, X, N, ldx, Y, ldy, acc);
        }
        env.check(hipGetLastError());
      }
      return env.status;
    case P_ELL:
      if (env.ok()) {
        LaunchScope ls(env, "spmm_ell", 8.0 * A.nval + xy);
        const int64_t tiles = ceil_div<int64_t>(A.nrows, 32), per_xcd = ceil_div<int64_t>(tiles, 8);
        const dim3 grid((unsigned)(per_xcd * 8), (unsigned)ceil_div<int64_t>(N, 64 * vec));
        const int32_t *ec = A.level[2].idx;
        if (vec == 4) hipLaunchKernelGGL(ell_spmm_kernel<4>, grid, dim3(256), 0, env.stream, ec, (const float *)A.val, A.nmajor, A.nrows, per_xcd, X, N, ldx, Y, ldy, acc);
        else if (vec == 2) hipLaunchKernelGGL(ell_spmm_kernel<2>, grid, dim3(256), 0, env.stream, ec, (const float *)A.val, A.nmajor, A.nrows, per_xcd, X, N, ldx, Y, ldy, acc);
        else hipLaunchKernelGGL(ell_spmm_kernel<1>, grid, dim3(256), 0, env.stream, ec, (const float *)A.val, A.nmajor, A.nrows, per_xcd, X, N, ldx, Y, ldy, acc);
        env.check(hipGetLastError());
      }
      return env.status;
    case P_CSR:
    case P_DCSR:
    case P_CISR: {
      const StoredRows sr = stored_rows(A);
      if (A.swapped) {
        if (!accumulate) zero_rows(env, Y, A.nrows, N, ldy);
        if (env.ok() && A.nmajor > 0) {
          LaunchScope ls(env, "spmm_csc", 8.0 * A.nnz + xy);
          hipLaunchKernelGGL(csc_spmm_atomic_kernel, dim3((unsigned)ceil_div<int64_t>(A.nmajor, 4), (unsigned)ncb),
                             dim3(256), 0, env.stream, sr.ptr, sr.idx, (const float *)A.val, sr.row_ids, A.nmajor, X, N,
                             ldx, Y, ldy);
          env.check(hipGetLastError());
        }
        return env.status;
      }
      if (!accumulate) zero_rows(env, Y, A.nrows, N, ldy);
      if (A.nnz > 0) {
        RowSrc rs{nullptr, sr.ptr, sr.row_ids, A.nmajor};
        entry_balanced_spmm(env, A, rs, sr.idx, "spmm_csr", vec, X, N, ldx, Y, ldy);
      }
      return env.status;
    }
    case P_DIA:
      if (env.ok()) {
        LaunchScope ls(env, "spmm_dia", 4.0 * A.nval + xy);
        const int64_t tiles = ceil_div<int64_t>(A.nrows, 4 * DIA_R), per_xcd = ceil_div<int64_t>(tiles, 8);
        const dim3 grid((unsigned)(per_xcd * 8), (unsigned)ceil_div<int64_t>(N, 64 * vec));
        const int32_t *off = (const int32_t *)A.level[0].idx;
        const int by_col = A.swapped ? 1 : 0;
        if (vec == 4) hipLaunchKernelGGL(dia_spmm_rows_kernel<4>, grid, dim3(256), 0, env.stream, off, (const float *)A.val, A.nmajor, A.nrows, A.ncols, by_col, per_xcd, X, N, ldx, Y, ldy, acc);
        else if (vec == 2) hipLaunchKernelGGL(dia_spmm_rows_kernel<2>, grid, dim3(256), 0, env.stream, off, (const float *)A.val, A.nmajor, A.nrows, A.ncols, by_col, per_xcd, X, N, ldx, Y, ldy, acc);
        else hipLaunchKernelGGL(dia_spmm_rows_kernel<1>, grid, dim3(256), 0, env.stream, off, (const float *)A.val, A.nmajor, A.nrows, A.ncols, by_col, per_xcd, X, N, ldx, Y, ldy, acc);
        env.check(hipGetLastError());
      }
      return env.status;
    case P_CSB:
      if (!accumulate) zero_rows(env, Y, A.nrows, N, ldy);
      if (env.ok() && A.nnz > 0) {
        LaunchScope ls(env, "spmm_csb_atomic", 12.0 * A.nnz + xy);
        const int chunk_len = chunk_entries(A.nnz);
        const int64_t per_xcd = ceil_div<int64_t>(ceil_div<int64_t>(ceil_div<int64_t>(A.nnz, chunk_len), 4), 8);
        const dim3 grid((unsigned)(per_xcd * 8), (unsigned)ceil_div<int64_t>(N, 64 * vec));
#define US_CSB_LAUNCH(V) hipLaunchKernelGGL(csb_spmm_kernel<V>, grid, dim3(256), 0, env.stream, (const int32_t *)A.level[2].ptr, (const int32_t *)A.level[2].idx, (const int32_t *)A.level[3].idx, (const float *)A.val, A.nnz, chunk_len, per_xcd, A.nmajor, A.level[1].size, A.bh, A.bw, X, N, ldx, Y, ldy)
        if (vec == 4) US_CSB_LAUNCH(4); else if (vec == 2) US_CSB_LAUNCH(2); else US_CSB_LAUNCH(1);
#undef US_CSB_LAUNCH
        env.check(hipGetLastError());
      }
      return env.status;
    case P_BDIA:
      if (env.ok()) {
        LaunchScope ls(env, "spmm_bdia", 4.0 * A.nval + 4.0 * A.nblk + xy);
        const int64_t tiles = ceil_div<int64_t>(A.nmajor, 4), per_xcd = ceil_div<int64_t>(tiles, 8);
        const dim3 grid((unsigned)(per_xcd * 8), (unsigned)ceil_div<int64_t>(N, 64 * vec));
#define US_BDIA_LAUNCH(V, H) hipLaunchKernelGGL((bdia_spmm_rows_kernel<V, H>), grid, dim3(256), 0, env.stream, (const int32_t *)A.level[1].ptr, (const int32_t *)A.level[1].idx, (const float *)A.val, A.nmajor, (int)A.bh, per_xcd, A.nrows, A.ncols, X, N, ldx, Y, ldy, acc)
#define US_BDIA_BY_HEIGHT(V) do { if (A.bh <= 2) US_BDIA_LAUNCH(V, 2); else if (A.bh <= 4) US_BDIA_LAUNCH(V, 4); else if (A.bh <= 8) US_BDIA_LAUNCH(V, 8); else US_BDIA_LAUNCH(V, 16); } while (0)
        if (vec == 4) US_BDIA_BY_HEIGHT(4); else if (vec == 2) US_BDIA_BY_HEIGHT(2); else US_BDIA_BY_HEIGHT(1);
#undef US_BDIA_BY_HEIGHT
#undef US_BDIA_LAUNCH
        env.check(hipGetLastError());
      }
      return env.status;
    case P_COO: {
      if (!accumulate) zero_rows(env, Y, A.nrows, N, ldy);
      if (A.nnz == 0) return env.status;
      if (A.swapped) {
        if (env.ok()) {
          LaunchScope ls(env, "spmm_coo_atomic", 12.0 * A.nnz + xy);
          hipLaunchKernelGGL(coo_spmm_atomic_kernel, dim3((unsigned)ceil_div<int64_t>(A.nnz, 4), (unsigned)ncb),
                             dim3(256), 0, env.stream, (const int32_t *)A.level[1].idx, (const int32_t *)A.level[0].idx,
                             (const float *)A.val, A.nnz, X, N, ldx, Y, ldy);
          env.check(hipGetLastError());
        }
        return env.status;
      }
      RowSrc rs{A.level[0].idx, nullptr, nullptr, 0};
      entry_balanced_spmm(env, A, rs, A.level[1].idx, "spmm_coo", vec, X, N, ldx, Y, ldy);
      return env.status;
    }
    default: break;
  }
  return US_ERR_FORMAT_MISMATCH;
}

}  // namespace us
