// The Sort operator of the conversion algorithm (Figure 8: the step that orders T_format by its target tuple;
// Section 7.2.1 reports it as 65 % of COO->BDIA conversion time, Section 7.2.3 as 84 % for
// Serpens) as a least-significant-digit radix sort over packed target tuples.
//
// One digit pass = per-tile digit histogram, chunked scan of the (tile, digit) table, stable
// tile scatter (wavefront-ballot ranking, tile reordered through LDS so that every digit's run
// is written as one contiguous piece).  The first pass builds the keys from (row, col) on the
// fly (index-map evaluation: Swap, TileSplit), the last one can unpack them into index arrays,
// so keys never take an extra trip through HBM.
//
// Between passes an item travels as one 12-byte record {key low, key high, value}: the scatter
// is bound by the number of scattered store streams rather than by bytes (storing only the 5
// significant key bytes in two arrays was 25 % SLOWER than 8-byte keys), so key and payload
// share one stream.  Every pass also leaves the NEXT pass's digit of each item as a byte, so
// the next histogram reads 1 byte per item instead of the record.
//
// A single-kernel pass with a decoupled look-back over per-tile status words was tried and
// dropped: with ~770 tiles resident at once and status words that must cross the XCDs' L2s,
// the serial look-back (one device-scope load per predecessor and digit) ran 40x slower than
// the separate histogram + scan.  Digit totals accumulated with device atomics were dropped
// too: same-address atomics cost ~20 ns each here and serialised the histogram kernel.  Wider digits do not
// pay either: with 10 bits (4 passes instead of 5 for 40-bit keys, 48-byte runs per tile and digit) a scatter
// pass took 152 us instead of 107; with 7 bits it took 96 us, but there are then 6 of them.
//
// What the counters say about the scatter kernel (16.8 M entries, 100 us): ~810 VALU instructions per
// wavefront = 42 % of the VALU issue slots, waves waiting twice as long as they issue, 6 waves per SIMD
// (74 VGPRs, 43 KB of LDS per workgroup).  Forcing 8 waves per SIMD (16-bit wave counters for the LDS,
// 64 VGPRs) spilled 24 registers and took 157 us; 8192-entry tiles (16 entries per thread, runs twice as
// long, 4 waves per SIMD) took 123 us; 1024 threads x 4 entries (same tile, 48 VGPRs, 8 waves per SIMD) took
// 105 us, no different from the 106 us of this shape: occupancy is not what holds the kernel back, the
// scattered 200-byte pieces it writes are (7-bit digits, pieces twice as long: 96 us).
//
// A counting sort by row (device atomics for the row histogram, then an atomic cursor per row for the scatter,
// then a sort inside every row) is no way round the digit passes: on the 16.8 M entries and 2^20 rows of the
// power-law workload the histogram alone took 0.91 ms (18 G atomics per second to scattered addresses) and the
// cursor scatter 1.5 ms, against 0.68 ms for all five passes here.
#include "common.h"
#include "device.h"

namespace us {

constexpr int RS_T = 512, RS_IPT = 8, RS_TILE = RS_T * RS_IPT, RS_NW = RS_T / 64, RS_MAXBITS = 8, RS_BINS = 1 << RS_MAXBITS;
constexpr int RS_CHUNK = 32;  // tiles per workgroup of the chunk scan
constexpr int RS_HC = 16;     // histogram kernel: counters per digit

typedef uint64_t Key;  // keys live in registers and LDS as 64-bit words whatever their storage

__device__ __forceinline__ Key build_key(const KeySpec &ks, uint32_t r, uint32_t c) {
  uint32_t a = ks.swap ? c : r, b = ks.swap ? r : c;
  if (ks.mode == 0) return ((Key)a << ks.b_bits) | (Key)b;
  // (a coordinate out of range is reported, not sorted; its second field is still cut to b_bits so that it cannot
  // leak into the leading field, whose digits the first histogram may take from a / bh alone)
  const Key field = ((Key)1 << ks.b_bits) - 1;
  if (ks.mode == 2) {   // Skew(0,1,-1) then TileSplit(0,bh): (a/bh, b-a, a%bh), the diagonal biased to be >= 0
    uint32_t ab = a / ks.bh, ai = a - ab * ks.bh, dg = b - a + (ks.a_extent - 1);
    return ((((Key)ab << ks.b_bits) | ((Key)dg & field)) << ks.ih_bits) | (Key)ai;
  }
  uint32_t ab = a / ks.bh, ai = a - ab * ks.bh, bb = b / ks.bw, bi = b - bb * ks.bw;
  return (((((Key)ab << ks.b_bits) | ((Key)bb & field)) << ks.ih_bits | (Key)ai) << ks.iw_bits) | (Key)bi;
}

enum { IN_COO = 0, IN_SPLIT = 1, IN_KEY32 = 2 };
enum { OUT_SPLIT = 0, OUT_UNPACK = 1, OUT_KEY64 = 2, OUT_KEY32 = 3 };

struct __attribute__((packed, aligned(4))) Rec { uint32_t lo, hi, val; };

struct PassArgs {
  // input
  const int32_t *row, *col;        // IN_COO
  const uint32_t *lo_in;           // IN_KEY32: keys
  const Rec *rec_in;               // IN_SPLIT: records written by the previous pass
  const uint32_t *val_in;          // IN_COO / IN_KEY32
  const uint8_t *digit_in;         // this pass's digit of every input item, or null (first pass)
  // output
  Rec *rec_out;                    // OUT_SPLIT
  int32_t *major_out, *minor_out;  // OUT_UNPACK (key mode 0)
  uint64_t *key64_out; uint32_t *key32_out;
  uint32_t *val_out;
  uint8_t *digit_out;              // next pass's digit of every output item, or null (last pass)
  uint32_t n; int shift; uint32_t mask; uint32_t nblocks;
  int next_shift; uint32_t next_mask;
  uint32_t tiles_per_xcd;          // launch index -> tile mapping (see xcd_tile)
  uint32_t *hist;                  // [nblocks][RS_BINS] per-tile digit counts, then prefixes inside a chunk of tiles
  uint32_t *chunk;                 // [RS_BINS][nchunks] per-chunk digit counts, then prefixes over the chunks
  uint32_t *dtotal;                // [RS_BINS] digit totals of the whole input
  uint32_t nchunks;
  KeySpec ks;
  int hist_minor_only;             // IN_COO: this pass's digit lies inside the minor index of a (major, minor) key
  int coo_vec;                     // IN_COO: row, col and val are 16-byte aligned (full tiles are read four entries a load)
  int hist_major_shift;            // IN_COO, blocked keys: >= 0 when this pass's digit lies inside the leading field
                                   // a / bh of the key: digit = ((a / bh) >> hist_major_shift) & mask
  Flags *flags;
};

__device__ __forceinline__ bool coo_out_of_range(const KeySpec &ks, uint32_t r, uint32_t c) {
  return ((ks.swap ? c : r) >= ks.a_extent) | ((ks.swap ? r : c) >= ks.b_extent);
}

template <int IN>
__device__ __forceinline__ void load_item(const PassArgs &a, uint32_t i, Key *key, uint32_t *val, bool *bad) {
  if (IN == IN_COO) {
    const uint32_t r = (uint32_t)a.row[i], c = (uint32_t)a.col[i];
    *bad |= coo_out_of_range(a.ks, r, c);
    *key = build_key(a.ks, r, c);
    *val = a.val_in[i];
  } else if (IN == IN_KEY32) {
    *key = a.lo_in[i];
    *val = a.val_in[i];
  } else {
    Rec r = a.rec_in[i];
    *key = (Key)r.lo | ((Key)r.hi << 32);
    *val = r.val;
  }
}

// Workgroups are dealt round-robin to the 8 XCDs.  Mapping launch index i to tile
// (i % 8) * tiles_per_xcd + i / 8 lets each XCD work through one contiguous range of tiles, so
// the partial cache lines at the ends of neighbouring tiles' runs meet in the same L2.
__device__ __forceinline__ uint32_t xcd_tile(uint32_t i, uint32_t per_xcd) { return (i & 7u) * per_xcd + (i >> 3); }

template <int IN>
__global__ __launch_bounds__(RS_T) void radix_hist_kernel(PassArgs a) {
  // RS_HC counters per digit, picked by lane: neighbouring items often share a digit (within a group of
  // rows that share their low bits, one heavy row owns most entries), and LDS adds to one address
  // take their turns one lane at a time.
  __shared__ uint32_t s_hist[RS_BINS * RS_HC];
  for (int i = threadIdx.x; i < RS_BINS * RS_HC; i += RS_T) s_hist[i] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * RS_TILE;
  const uint32_t copy = threadIdx.x & (RS_HC - 1);
  uint32_t digit[RS_IPT];
  if (IN == IN_SPLIT && a.digit_in) {
    // the previous pass left this pass's digits as bytes: 8 per thread in one 8-byte load
    const uint32_t i = base + threadIdx.x * RS_IPT;
    if (i + RS_IPT <= a.n) {
      static_assert(RS_IPT == 4 || RS_IPT == 8, "digit bytes are read 4 or 8 at a time");
      uint32_t v[RS_IPT / 4];
#pragma unroll
      for (int q = 0; q < RS_IPT / 4; ++q) v[q] = reinterpret_cast<const uint32_t *>(a.digit_in + i)[q];
#pragma unroll
      for (int k = 0; k < RS_IPT; ++k) digit[k] = (v[k / 4] >> (8 * (k % 4))) & 0xFFu;
    } else {
#pragma unroll
      for (int k = 0; k < RS_IPT; ++k) digit[k] = i + k < a.n ? a.digit_in[i + k] : 0xFFFFFFFFu;
    }
  } else if (IN == IN_COO && a.hist_major_shift >= 0) {
    // the digit is a bit field of the block row alone: read the row indices only (the scatter of this pass reads
    // and validates both coordinates)
    const int32_t *major = a.ks.swap ? a.col : a.row;
    if (base + RS_TILE <= a.n && (reinterpret_cast<uintptr_t>(major) & 15u) == 0) {
      const uint4 *m4 = reinterpret_cast<const uint4 *>(major + base);   // full, aligned tile: four indices per load
      uint4 v[RS_IPT / 4];
#pragma unroll
      for (int q = 0; q < RS_IPT / 4; ++q) v[q] = m4[q * RS_T + threadIdx.x];
#pragma unroll
      for (int q = 0; q < RS_IPT / 4; ++q) {
        digit[4 * q + 0] = ((v[q].x / a.ks.bh) >> a.hist_major_shift) & a.mask;
        digit[4 * q + 1] = ((v[q].y / a.ks.bh) >> a.hist_major_shift) & a.mask;
        digit[4 * q + 2] = ((v[q].z / a.ks.bh) >> a.hist_major_shift) & a.mask;
        digit[4 * q + 3] = ((v[q].w / a.ks.bh) >> a.hist_major_shift) & a.mask;
      }
    } else {
#pragma unroll
      for (int k = 0; k < RS_IPT; ++k) {
        uint32_t i = base + k * RS_T + threadIdx.x;
        digit[k] = i < a.n ? ((((uint32_t)major[i] / a.ks.bh) >> a.hist_major_shift) & a.mask) : 0xFFFFFFFFu;
      }
    }
  } else if (IN == IN_COO && a.hist_minor_only) {
    // the digit is a bit field of the minor index alone: read that array only (the scatter of this pass
    // reads both and validates them; bits of an out-of-range minor index land in the key just the same)
    const int32_t *minor = a.ks.swap ? a.row : a.col;
    if (base + RS_TILE <= a.n && (reinterpret_cast<uintptr_t>(minor) & 15u) == 0) {
      // a full tile of a 16-byte aligned array: four indices per load (which thread counts which item is free)
      static_assert(RS_IPT % 4 == 0, "indices are read four at a time");
      const uint4 *m4 = reinterpret_cast<const uint4 *>(minor + base);
      uint4 v[RS_IPT / 4];
#pragma unroll
      for (int q = 0; q < RS_IPT / 4; ++q) v[q] = m4[q * RS_T + threadIdx.x];
#pragma unroll
      for (int q = 0; q < RS_IPT / 4; ++q) {
        digit[4 * q + 0] = (v[q].x >> a.shift) & a.mask;
        digit[4 * q + 1] = (v[q].y >> a.shift) & a.mask;
        digit[4 * q + 2] = (v[q].z >> a.shift) & a.mask;
        digit[4 * q + 3] = (v[q].w >> a.shift) & a.mask;
      }
    } else {
#pragma unroll
      for (int k = 0; k < RS_IPT; ++k) {
        uint32_t i = base + k * RS_T + threadIdx.x;
        digit[k] = i < a.n ? (((uint32_t)minor[i] >> a.shift) & a.mask) : 0xFFFFFFFFu;
      }
    }
  } else {
    bool bad = false;
    Key key[RS_IPT];
#pragma unroll
    for (int k = 0; k < RS_IPT; ++k) {   // all loads first: the memory system sees 8 requests per thread
      uint32_t i = base + k * RS_T + threadIdx.x;
      key[k] = 0;
      if (i < a.n) {
        uint32_t unused;
        load_item<IN>(a, i, &key[k], &unused, &bad);
      }
    }
#pragma unroll
    for (int k = 0; k < RS_IPT; ++k) {
      uint32_t i = base + k * RS_T + threadIdx.x;
      digit[k] = i < a.n ? ((uint32_t)(key[k] >> a.shift) & a.mask) : 0xFFFFFFFFu;
    }
    if (IN == IN_COO && bad) a.flags->index_range = 1;
  }
#pragma unroll
  for (int k = 0; k < RS_IPT; ++k)
    if (digit[k] != 0xFFFFFFFFu) atomicAdd(&s_hist[digit[k] * RS_HC + copy], 1u);
  __syncthreads();
  for (uint32_t d = threadIdx.x; d < RS_BINS; d += RS_T) {
    uint32_t sum = 0;
#pragma unroll
    for (uint32_t c = 0; c < RS_HC; ++c) sum += s_hist[d * RS_HC + ((c + d) & (RS_HC - 1))];
    a.hist[(size_t)blockIdx.x * RS_BINS + d] = sum;
  }
}

// Offsets of every (tile, digit) run without a single atomic:
//   chunk kernel: a workgroup takes RS_CHUNK consecutive tiles, thread d walks digit d through
//                 them (coalesced rows), leaving prefixes inside the chunk and the chunk total;
//   top kernel:   one wavefront per digit scans the chunk totals and leaves the digit total;
//   the scatter kernel adds the start of the digit (a 256-entry scan it does itself).
// Letting one workgroup of the histogram kernel count 8 tiles in a row and leave the prefixes itself (no chunk
// kernel) was no faster: 25 + 8.5 us a pass for the two kernels left, against 19 + 7 + 6.5 for these three.
__global__ __launch_bounds__(RS_BINS) void radix_scan_chunk_kernel(uint32_t *hist, uint32_t *chunk, uint32_t nblocks) {
  const uint32_t d = threadIdx.x;
  const uint32_t t0 = blockIdx.x * RS_CHUNK, t1 = min(t0 + RS_CHUNK, nblocks);
  uint32_t v[RS_CHUNK];
#pragma unroll
  for (int k = 0; k < RS_CHUNK; ++k) v[k] = t0 + k < t1 ? hist[(size_t)(t0 + k) * RS_BINS + d] : 0u;
  uint32_t run = 0;
#pragma unroll
  for (int k = 0; k < RS_CHUNK; ++k) {
    if (t0 + k < t1) hist[(size_t)(t0 + k) * RS_BINS + d] = run;
    run += v[k];
  }
  chunk[(size_t)d * gridDim.x + blockIdx.x] = run;   // digit-major
}

__global__ __launch_bounds__(256) void radix_scan_top_kernel(uint32_t *chunk, uint32_t nchunks, uint32_t *dtotal) {
  const uint32_t d = blockIdx.x * 4 + wave_id();
  const int lane = lane_id();
  uint32_t *row = chunk + (size_t)d * nchunks;
  uint32_t carry = 0;
  for (uint32_t c0 = 0; c0 < nchunks; c0 += 64) {
    const uint32_t c = c0 + lane;
    const uint32_t v = c < nchunks ? row[c] : 0u;
    const uint32_t inc = wave_inclusive_sum(v);
    if (c < nchunks) row[c] = carry + inc - v;
    carry += __shfl(inc, 63);
  }
  if (lane == 0) dtotal[d] = carry;
}

// Both scans in one workgroup for inputs of at most RS_SMALL tiles (one launch less per digit pass, which is
// what a conversion of a few hundred thousand entries spends its time on): thread d holds digit d of every tile.
constexpr int RS_SMALL = 64;
__global__ __launch_bounds__(RS_BINS) void radix_scan_small_kernel(uint32_t *hist, uint32_t *chunk, uint32_t *dtotal,
                                                                  uint32_t nblocks, uint32_t nchunks) {
  const uint32_t d = threadIdx.x;
  uint32_t v[RS_SMALL];
#pragma unroll
  for (int t = 0; t < RS_SMALL; ++t) v[t] = (uint32_t)t < nblocks ? hist[(size_t)t * RS_BINS + d] : 0u;
  uint32_t before_chunk = 0, run = 0;
#pragma unroll
  for (int t = 0; t < RS_SMALL; ++t) {
    if ((uint32_t)t < nblocks) {
      if (t % RS_CHUNK == 0) {
        before_chunk += run;
        run = 0;
        chunk[(size_t)d * nchunks + t / RS_CHUNK] = before_chunk;
      }
      hist[(size_t)t * RS_BINS + d] = run;
      run += v[t];
    }
  }
  dtotal[d] = before_chunk + run;
}

template <int IN, int OUT>
__global__ __launch_bounds__(RS_T) void radix_scatter_kernel(PassArgs a) {
  __shared__ uint32_t s_cnt[RS_NW][RS_BINS];  // per-wave digit counts, then per-wave bases
  __shared__ uint32_t s_start[RS_BINS];       // first in-tile position of each digit
  __shared__ uint32_t s_goff[RS_BINS];        // global position of the digit's run minus s_start
  __shared__ uint32_t s_wave[RS_T / 64 + 1];
  __shared__ Key s_key[RS_TILE];
  uint32_t *s_val = reinterpret_cast<uint32_t *>(s_key);

  const int lane = lane_id(), w = wave_id();
  const uint32_t nbins = a.mask + 1;
  const uint32_t tile = xcd_tile(blockIdx.x, a.tiles_per_xcd);
  if (tile >= a.nblocks) return;  // uniform: the launch is padded to 8 * tiles_per_xcd workgroups
  for (uint32_t i = threadIdx.x; i < RS_NW * RS_BINS; i += RS_T) (&s_cnt[0][0])[i] = 0;
  const uint32_t base = tile * RS_TILE;
  const uint32_t in_tile = min((uint32_t)RS_TILE, a.n - base);
  Key key[RS_IPT];
  uint32_t val[RS_IPT], pos[RS_IPT];
  bool bad = false;
  // wave w owns the contiguous slice [w*64*IPT, (w+1)*64*IPT) of the tile, lanes striped
  if (IN == IN_COO && a.coo_vec && in_tile == (uint32_t)RS_TILE) {
    // The caller's list has no order to keep, so which lane ranks which entry of the slice is free: four
    // consecutive entries per 16-byte load (item 4q + c of a lane is entry q*256 + 4*lane + c of the slice).
    static_assert(RS_IPT % 4 == 0, "entries are read four at a time");
    const uint32_t first = base + w * (64 * RS_IPT);
    const uint4 *r4 = reinterpret_cast<const uint4 *>(a.row + first), *c4 = reinterpret_cast<const uint4 *>(a.col + first);
    const uint4 *v4 = reinterpret_cast<const uint4 *>(a.val_in + first);
    uint4 rr[RS_IPT / 4], cc[RS_IPT / 4], vv[RS_IPT / 4];
#pragma unroll
    for (int q = 0; q < RS_IPT / 4; ++q) { rr[q] = r4[q * 64 + lane]; cc[q] = c4[q * 64 + lane]; vv[q] = v4[q * 64 + lane]; }
#pragma unroll
    for (int q = 0; q < RS_IPT / 4; ++q) {
      const uint32_t r[4] = {rr[q].x, rr[q].y, rr[q].z, rr[q].w}, c[4] = {cc[q].x, cc[q].y, cc[q].z, cc[q].w};
      const uint32_t v[4] = {vv[q].x, vv[q].y, vv[q].z, vv[q].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        bad |= coo_out_of_range(a.ks, r[e], c[e]);
        key[4 * q + e] = build_key(a.ks, r[e], c[e]);
        val[4 * q + e] = v[e];
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < RS_IPT; ++j) {
      uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
      key[j] = 0; val[j] = 0;
      if (t < in_tile) load_item<IN>(a, base + t, &key[j], &val[j], &bad);
    }
  }
  if (IN == IN_COO && bad) a.flags->index_range = 1;
  __syncthreads();

  // stable rank of every item among the items of its wave with the same digit.
  // peers = lanes holding the same digit = AND over the digit's bits of (bit ? ballot : ~ballot);
  // per bit that is one compare (the ballot), one sign-mask and one 3-input logic op per half.
  const uint32_t lane_lo = lane < 32 ? (1u << lane) - 1u : 0xFFFFFFFFu;   // lanes below this one
  const uint32_t lane_hi = lane < 32 ? 0u : (1u << (lane - 32)) - 1u;
#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    bool valid = t < in_tile;
    uint32_t d = (uint32_t)(key[j] >> a.shift) & a.mask;
    uint64_t vb = __ballot(valid);
    uint32_t plo = (uint32_t)vb, phi = (uint32_t)(vb >> 32);
#pragma unroll
    for (int b = 0; b < RS_MAXBITS; ++b) {
      const uint64_t bal = __ballot((d >> b) & 1u);
      const uint32_t keep = (uint32_t)((int32_t)(~d << (31 - b)) >> 31);   // all ones when bit b of d is 0
      plo &= (uint32_t)bal ^ keep;
      phi &= (uint32_t)(bal >> 32) ^ keep;
    }
    uint32_t before = __popc(plo & lane_lo) + __popc(phi & lane_hi);
    uint32_t count = __popc(plo) + __popc(phi);
    int leader = plo ? __ffs(plo) - 1 : (phi ? __ffs(phi) + 31 : 0);
    uint32_t old = 0;
    if (valid && lane == leader) {
      old = s_cnt[w][d];
      s_cnt[w][d] = old + count;
    }
    old = __shfl(old, leader);
    pos[j] = old + before;
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();

  // per digit: bases of the waves, tile total
  uint32_t tile_total = 0;
  if (threadIdx.x < nbins) {
#pragma unroll
    for (int ww = 0; ww < RS_NW; ++ww) {
      uint32_t c = s_cnt[ww][threadIdx.x];
      s_cnt[ww][threadIdx.x] = tile_total;
      tile_total += c;
    }
  }
  uint32_t dummy;
  const uint32_t start = block_exclusive_sum<RS_T>(tile_total, s_wave, &dummy);
  const uint32_t digit_start =
      block_exclusive_sum<RS_T>(threadIdx.x < RS_BINS ? a.dtotal[threadIdx.x] : 0u, s_wave, &dummy);
  if (threadIdx.x < nbins) {
    s_start[threadIdx.x] = start;
    s_goff[threadIdx.x] = digit_start + a.chunk[(size_t)threadIdx.x * a.nchunks + tile / RS_CHUNK] +
                           a.hist[(size_t)tile * RS_BINS + threadIdx.x] - start;
  }
  __syncthreads();

#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    if (t < in_tile) {
      uint32_t d = (uint32_t)(key[j] >> a.shift) & a.mask;
      pos[j] += s_start[d] + s_cnt[w][d];
      s_key[pos[j]] = key[j];
    }
  }
  __syncthreads();
  uint32_t gpos[RS_IPT];
  Key skey[RS_IPT];
#pragma unroll
  for (int k = 0; k < RS_IPT; ++k) {
    uint32_t i = k * RS_T + threadIdx.x;
    gpos[k] = 0; skey[k] = 0;
    if (i < in_tile) {
      Key kk = s_key[i];
      uint32_t g = s_goff[(uint32_t)(kk >> a.shift) & a.mask] + i;
      gpos[k] = g;
      if (OUT == OUT_UNPACK) {
        a.major_out[g] = (int32_t)(kk >> a.ks.b_bits);
        a.minor_out[g] = (int32_t)(kk & (((Key)1 << a.ks.b_bits) - 1));
      } else if (OUT == OUT_KEY64) {
        a.key64_out[g] = kk;
      } else if (OUT == OUT_KEY32) {
        a.key32_out[g] = (uint32_t)kk;
      } else {
        skey[k] = kk;   // written together with the value below
        if (a.digit_out) a.digit_out[g] = (uint8_t)((uint32_t)(kk >> a.next_shift) & a.next_mask);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    if (t < in_tile) s_val[pos[j]] = val[j];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < RS_IPT; ++k) {
    uint32_t i = k * RS_T + threadIdx.x;
    if (i < in_tile) {
      if (OUT == OUT_SPLIT) a.rec_out[gpos[k]] = Rec{(uint32_t)skey[k], (uint32_t)(skey[k] >> 32), s_val[i]};
      else a.val_out[gpos[k]] = s_val[i];
    }
  }
}


// ------------------------------------------------------------------ finishing sort inside LDS
// After the digit passes over the top bits of the key the list is cut into buckets of equal
// prefix that sit next to each other.  Keys are unique, so a bucket is small whenever the
// prefix is long enough, and it is finished where it fits: one workgroup loads the bucket,
// sorts the remaining low bits (at most 32) with the same stable ballot ranking, digit by
// digit, exchanging items through LDS only, and writes the final arrays.  Compared with
// carrying on with whole-array passes this replaces ceil(low_bits / 8) trips through HBM by
// one.
//
// A bucket above LS_CAP items (a heavy row of a power-law matrix, say) gets one more 8-bit
// split of its own first: its tiles are counted, scanned and scattered like a digit pass, but
// only its items move.  The pieces are then bundled, in order, into groups of at most LS_CAP
// items that the same LDS kernel finishes (it sorts by all low bits, so a group may span
// several pieces; a piece above LS_GROUP items is a group of its own).  A bucket beyond LS_MAXTILES tiles, or a piece above LS_CAP items, sets
// Flags::retry and the host sorts again with whole-array passes only.
// (Replacing the digit passes inside LDS by one 8-bit split plus counting smaller keys inside each piece
// was tried: the keys of a blocked layout cluster -- block columns inside a band, 16 entries per block --
// so pieces come out uneven whichever bits are taken, the count goes quadratic, and it lost.)
constexpr int LS_T = 256, LS_IPT = 16, LS_CAP = LS_T * LS_IPT;   // 4096 items, 32 KB of LDS
constexpr int LS_GROUP = LS_CAP / 2;     // pieces are bundled by the LS_GROUP-sized interval their start falls in
constexpr int LS_MAXTILES = 64;          // split buckets hold at most 64 * 4096 items

struct BigBucket { uint32_t bucket, first, size, tile_base; };
struct WorkItem { uint32_t first, size, bucket; };

struct LocalArgs {
  const Rec *rec_in;     // sorted by the top bits
  Rec *rec_split;        // big buckets after their extra split (same positions as in rec_in)
  const uint32_t *off;   // [nbuckets + 1] first record of every bucket
  uint32_t nbuckets, n;
  int low_bits;          // bits left to sort, <= 32
  int b_bits;            // OUT_UNPACK: minor index width
  int inner_bits;        // blocked tuples: key bits below the node (block row, block column | diagonal), the in-block indices
  uint32_t *node_count;  // per NODE_TILE output entries: nodes that start there (SortOut::node_count), or null
  // extra split of the big buckets
  uint32_t *counters;    // [0] big buckets, [1] their tiles, [2] groups
  BigBucket *big; uint32_t big_cap;
  uint32_t *tilemap; uint32_t tile_cap;   // tile -> index into big
  uint32_t *shist;       // [tile_cap][RS_BINS] digit counts per tile, then prefixes inside the bucket
  uint32_t *sdig;        // [big_cap][RS_BINS] first position of every piece inside its bucket
  WorkItem *work; uint32_t work_cap;
  // output
  int32_t *major_out, *minor_out;
  uint64_t *key64_out;
  uint32_t *val_out;
  Flags *flags;
};

__device__ __forceinline__ uint32_t split_digit(const LocalArgs &a, uint32_t lo) {
  const uint32_t low = a.low_bits >= 32 ? lo : (lo & ((1u << a.low_bits) - 1u));
  return a.low_bits > RS_MAXBITS ? (low >> (a.low_bits - RS_MAXBITS)) : low;   // top 8 of the low bits
}

// off[b] = first record whose prefix (key >> low_bits) is >= b, by bisection.  (A search that probes 64 places per
// step, one wavefront per bucket, ends after 3-5 rounds of loads instead of 26, but fetches 10 M scattered lines where
// the bisections share their upper levels: 41 us against 22 for the 32,769 buckets of 50 M records.)
__global__ __launch_bounds__(256) void bucket_offsets_kernel(const Rec *rec, uint32_t n, int low_bits, uint32_t nbuckets,
                                                            uint32_t *off) {
  const uint32_t b = blockIdx.x * 256 + threadIdx.x;
  if (b > nbuckets) return;
  uint32_t lo = 0, hi = n;   // first record whose prefix is >= b
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    const Rec r = rec[mid];
    const uint64_t prefix = (((uint64_t)r.hi << 32) | r.lo) >> low_bits;
    if (prefix < b) lo = mid + 1; else hi = mid;
  }
  off[b] = b == nbuckets ? n : lo;
}

// offsets come from searches over device data (garbage keys when a coordinate was out of range):
// nothing beyond this check is trusted to keep accesses inside [0, n)
__device__ __forceinline__ bool bucket_range(const LocalArgs &a, uint32_t b, uint32_t *first, uint32_t *size) {
  const uint32_t f = a.off[b], l = a.off[b + 1];
  if (l > a.n || f >= l) return false;
  *first = f; *size = l - f;
  return true;
}

__global__ __launch_bounds__(256) void big_list_kernel(LocalArgs a) {
  const uint32_t b = blockIdx.x * 256 + threadIdx.x;
  uint32_t first, size;
  if (b >= a.nbuckets || !bucket_range(a, b, &first, &size) || size <= (uint32_t)LS_CAP) return;
  const uint32_t ntiles = (size + RS_TILE - 1) / RS_TILE;
  if (ntiles > (uint32_t)LS_MAXTILES) { a.flags->retry = RETRY_SORT_LDS; return; }
  const uint32_t k = atomicAdd(&a.counters[0], 1u);
  const uint32_t tb = atomicAdd(&a.counters[1], ntiles);
  if (k >= a.big_cap || tb + ntiles > a.tile_cap) { a.flags->retry = RETRY_SORT_LDS; return; }   // overlapping garbage ranges only
  a.big[k] = BigBucket{b, first, size, tb};
  for (uint32_t j = 0; j < ntiles; ++j) a.tilemap[tb + j] = k;
}

// (the three kernels of the extra split walk their items with a stride of the grid: most inputs have no bucket to
// split, and a launch of one workgroup per possible tile then costs ~13 us of workgroups that start and leave)
constexpr uint32_t SEG_GRID = 1024;

__global__ __launch_bounds__(RS_T) void seg_hist_kernel(LocalArgs a) {
  __shared__ uint32_t s_hist[RS_BINS];
  const uint32_t ntiles = min(a.counters[1], a.tile_cap);
  for (uint32_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
    for (int i = threadIdx.x; i < RS_BINS; i += RS_T) s_hist[i] = 0;
    __syncthreads();
    const BigBucket B = a.big[min(a.tilemap[t], a.big_cap - 1)];
    const uint32_t begin = (t - B.tile_base) * RS_TILE, end = min(begin + (uint32_t)RS_TILE, B.size);
    for (uint32_t i = begin + threadIdx.x; i < end; i += RS_T) atomicAdd(&s_hist[split_digit(a, a.rec_in[B.first + i].lo)], 1u);
    __syncthreads();
    for (uint32_t d = threadIdx.x; d < RS_BINS; d += RS_T) a.shist[(size_t)t * RS_BINS + d] = s_hist[d];
    __syncthreads();
  }
}

// one workgroup per big bucket: prefixes of the (tile, digit) counts, piece starts, bundling into groups
__global__ __launch_bounds__(RS_BINS) void seg_scan_kernel(LocalArgs a) {
  __shared__ uint32_t s_wave[RS_BINS / 64 + 1];
  __shared__ uint32_t s_pos[RS_BINS + 1];    // piece starts, then group starts
  __shared__ uint32_t s_base;
  const uint32_t nbig = min(a.counters[0], a.big_cap), d = threadIdx.x;
  for (uint32_t k = blockIdx.x; k < nbig; k += gridDim.x) {
  const BigBucket B = a.big[k];
  const uint32_t ntiles = (B.size + RS_TILE - 1) / RS_TILE;
  uint32_t run = 0;
  for (uint32_t j = 0; j < ntiles; ++j) {
    uint32_t *h = a.shist + (size_t)(B.tile_base + j) * RS_BINS + d;
    const uint32_t v = *h;
    *h = run;
    run += v;
  }
  uint32_t total;
  const uint32_t start = block_exclusive_sum<RS_BINS>(run, s_wave, &total);
  a.sdig[(size_t)k * RS_BINS + d] = start;
  if (run > (uint32_t)LS_CAP) a.flags->retry = RETRY_SORT_LDS;
  s_pos[d] = start;
  if (d == 0) s_pos[RS_BINS] = B.size;
  __syncthreads();
  // piece d opens a group when its start falls in another LS_GROUP-sized interval than the one before (pieces of at
  // most LS_GROUP items bundled that way stay below LS_CAP together); a piece above LS_GROUP is a group of its own
  // (the piece behind it starts more than LS_GROUP further on, in another interval, hence in a new group)
  const bool head = d == 0 || run > (uint32_t)LS_GROUP || start / LS_GROUP != s_pos[d - 1] / LS_GROUP;
  uint32_t nheads;
  const uint32_t rank = block_exclusive_sum<RS_BINS>(head ? 1u : 0u, s_wave, &nheads);
  if (d == 0) s_base = atomicAdd(&a.counters[2], nheads);
  __syncthreads();
  if (head) s_pos[rank] = start;    // ranks <= d: slots below are no longer needed as piece starts
  if (d == 0) s_pos[nheads] = B.size;
  __syncthreads();
  if (head) {
    const uint32_t g = s_base + rank, gsize = s_pos[rank + 1] - start;
    if (g < a.work_cap) a.work[g] = WorkItem{B.first + start, gsize, B.bucket};
    else a.flags->retry = RETRY_SORT_LDS;
  }
  __syncthreads();   // s_pos and s_base are reused by the next bucket
  }
}

__global__ __launch_bounds__(RS_T) void seg_scatter_kernel(LocalArgs a) {
  __shared__ uint32_t s_next[RS_BINS];
  const uint32_t ntiles = min(a.counters[1], a.tile_cap);
  for (uint32_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const uint32_t k = min(a.tilemap[t], a.big_cap - 1);
    const BigBucket B = a.big[k];
    for (uint32_t d = threadIdx.x; d < RS_BINS; d += RS_T)
      s_next[d] = B.first + a.sdig[(size_t)k * RS_BINS + d] + a.shist[(size_t)t * RS_BINS + d];
    __syncthreads();
    const uint32_t begin = (t - B.tile_base) * RS_TILE, end = min(begin + (uint32_t)RS_TILE, B.size);
    for (uint32_t i = begin + threadIdx.x; i < end; i += RS_T) {
      const Rec r = a.rec_in[B.first + i];
      // the order inside a piece is settled by the full sort of its group, so any free slot will do
      const uint32_t at = atomicAdd(&s_next[split_digit(a, r.lo)], 1u);
      if (at < a.n) a.rec_split[at] = r;
    }
    __syncthreads();
  }
}

// Sort the cnt <= NT*IPT items in s_key / s_val [0, cnt) by the low `bits` bits of the keys, in place.
// Item t belongs to the thread with t = wave*(64*IPT) + j*64 + lane.  Between passes the items live
// in LDS only: registers hold them just for the exchange, which keeps the kernel near 64 VGPRs.
template <int NT, int IPT>
__device__ __forceinline__ void lds_sort(uint32_t cnt, int bits, uint32_t *s_key, uint32_t *s_val,
                                         uint32_t (*s_cnt)[RS_BINS], uint32_t *s_start, uint32_t *s_wave) {
  constexpr int NW = NT / 64;
  const int lane = lane_id(), w = wave_id();
  const uint32_t lane_lo = lane < 32 ? (1u << lane) - 1u : 0xFFFFFFFFu;
  const uint32_t lane_hi = lane < 32 ? 0u : (1u << (lane - 32)) - 1u;
  const int npass = (bits + RS_MAXBITS - 1) / RS_MAXBITS;
  const uint32_t t0 = w * (64 * IPT) + lane;
  int shift = 0;
  for (int p = 0; p < npass; ++p) {
    const int width = bits / npass + (p < bits % npass ? 1 : 0);
    const uint32_t mask = (1u << width) - 1u;
    for (uint32_t i = threadIdx.x; i < NW * RS_BINS; i += NT) (&s_cnt[0][0])[i] = 0;
    __syncthreads();
    uint32_t key[IPT], val[IPT], pos[IPT];
    // reads below are unguarded (t < NT*IPT always lies inside the arrays); a slot past cnt holds
    // stale data and is masked out of the ranking
#pragma unroll
    for (int j = 0; j < IPT; ++j) key[j] = s_key[t0 + j * 64];
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const uint32_t t = t0 + j * 64;
      const bool valid = t < cnt;
      const uint32_t d = (key[j] >> shift) & mask;
      const uint64_t vb = __ballot(valid);
      uint32_t plo = (uint32_t)vb, phi = (uint32_t)(vb >> 32);
#pragma unroll
      for (int b = 0; b < RS_MAXBITS; ++b) {
        const uint64_t bal = __ballot((d >> b) & 1u);
        const uint32_t keep = (uint32_t)((int32_t)(~d << (31 - b)) >> 31);
        plo &= (uint32_t)bal ^ keep;
        phi &= (uint32_t)(bal >> 32) ^ keep;
      }
      const uint32_t before = __popc(plo & lane_lo) + __popc(phi & lane_hi);
      // every peer reads the wave's running count of the digit, then the first peer advances it with
      // an add that returns nothing: LDS serves one wavefront's accesses in program order, so the
      // reads see the count before the add and nothing here waits for an LDS round trip
      const uint32_t old = valid ? s_cnt[w][d] : 0u;
      if (valid && before == 0) __hip_atomic_fetch_add(&s_cnt[w][d], __popc(plo) + __popc(phi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
      pos[j] = old + before;
      __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    uint32_t digit_total = 0;
    if (threadIdx.x < RS_BINS) {
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) {
        const uint32_t c = s_cnt[ww][threadIdx.x];
        s_cnt[ww][threadIdx.x] = digit_total;
        digit_total += c;
      }
    }
    uint32_t dummy;
    const uint32_t start = block_exclusive_sum<NT>(digit_total, s_wave, &dummy);
    if (threadIdx.x < RS_BINS) s_start[threadIdx.x] = start;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const uint32_t d = (key[j] >> shift) & mask;
      val[j] = s_val[t0 + j * 64];
      pos[j] += s_start[d] + s_cnt[w][d];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      if (t0 + j * 64 < cnt) {
        s_key[pos[j]] = key[j];
        s_val[pos[j]] = val[j];
      }
    }
    __syncthreads();
    shift += width;
  }
}

// The same result for the keys of a blocked tuple without sorting the entries: the entries of a bucket share few
// nodes (a block holds up to bh * bw of them), so the nodes are told apart with a hash table in LDS, only the
// distinct node keys are sorted, and an entry's place follows from its node's rank and from the entries of the
// node that come before it, counted in a bit map of the occupied in-block positions:
//   place = (entries of all nodes of lower rank) + (occupied positions of its node below its own).
// The ballot ranking of lds_sort costs ~80 VALU instructions per entry and 8-bit digit; here an entry costs one
// probe, two LDS atomics and a few population counts, whatever the width of the key.  Returns false (the same for
// every thread, LDS contents undefined) when the bucket holds more than RK_NODES nodes or its bit map does not
// fit: the caller then sorts the entries.  Two entries with one key share a bit: reported as a duplicate.
constexpr uint32_t RK_NODES = LS_CAP / 2;        // distinct nodes a bucket may hold; the table has twice as many slots
constexpr uint32_t RK_BITS = 32u * RK_NODES;      // bit map: RK_NODES words of LDS

__device__ __forceinline__ uint32_t rk_count(const uint32_t *bm, uint32_t node, int ib, uint32_t below) {
  // occupied positions of `node` below position `below` (below == 1 << ib: all of them)
  if (ib <= 5) {
    const uint32_t at = node << ib, w = bm[at >> 5] >> (at & 31u);
    return __popc(below >= 32u ? w : (w & ((1u << below) - 1u)));
  }
  const uint32_t base = node << (ib - 5), full = below >> 5;
  uint32_t c = 0;
  for (uint32_t q = 0; q < full; ++q) c += __popc(bm[base + q]);
  if (below & 31u) c += __popc(bm[base + full] & ((1u << (below & 31u)) - 1u));
  return c;
}

// A wavefront adds the nodes it has seen start in the (at most three) output tiles its work item touches to
// their counters: which[lane] = 0..2 for a lane that holds the first entry of a node, 3 otherwise.
__device__ __forceinline__ void add_heads(uint32_t which, uint32_t *h) {
  h[0] += (uint32_t)__popcll(__ballot(which == 0u));
  h[1] += (uint32_t)__popcll(__ballot(which == 1u));
  h[2] += (uint32_t)__popcll(__ballot(which == 2u));
}
__device__ __forceinline__ void flush_heads(uint32_t *tile_count, const uint32_t *h) {
  // (a tile with heads holds entries of this work item, so its index is below the number of tiles)
  if (lane_id() == 0) {
    if (h[0]) atomicAdd(&tile_count[0], h[0]);
    if (h[1]) atomicAdd(&tile_count[1], h[1]);
    if (h[2]) atomicAdd(&tile_count[2], h[2]);
  }
}

template <int IPT>
__device__ __forceinline__ bool rank_sort(const Rec *src, uint32_t first, uint32_t cnt, uint32_t low_mask, int low_bits,
                                          int ib, uint32_t *s_key, uint32_t *s_val, uint32_t (*s_cnt)[RS_BINS],
                                          uint32_t *s_start, uint32_t *s_wave, uint32_t *s_misc, uint32_t *tile_count,
                                          Flags *flags) {
  constexpr uint32_t EMPTY = 0xFFFFFFFFu;   // node keys have at most 31 bits
  uint32_t *tab = s_key, *dkey = s_val, *dslot = s_val + RK_NODES;
  static_assert(LS_CAP % (4 * LS_T) == 0, "table cleared with 16-byte stores");
  for (uint32_t i = threadIdx.x; i < (uint32_t)LS_CAP / 4; i += LS_T)
    reinterpret_cast<uint4 *>(tab)[i] = make_uint4(EMPTY, EMPTY, EMPTY, EMPTY);
  if (threadIdx.x == 0) { s_misc[0] = 0; s_misc[1] = 0; }
  s_start[threadIdx.x] = 0;   // ranks of up to LS_T nodes
  static_assert(RS_BINS == LS_T, "one rank per thread");
  uint32_t key[IPT], val[IPT], aux[IPT];
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    const uint32_t i = threadIdx.x + j * LS_T;
    key[j] = 0; val[j] = 0; aux[j] = 0;
    if (i < cnt) {
      const Rec r = src[first + i];
      key[j] = r.lo & low_mask;
      val[j] = r.val;
    }
  }
  __syncthreads();
  // every entry finds (or claims) the slot of its node; a claim also appends the node to the list of distinct
  // ones.  Slots are never given up, so a probe ends at the node's slot or at a free one, and the table cannot
  // fill: claims stop at RK_NODES + one per thread < LS_CAP
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    if (threadIdx.x + j * LS_T < cnt) {
      const uint32_t node = key[j] >> ib;
      uint32_t h = (node * 0x9E3779B1u) >> 20;   // 12 bits: LS_CAP slots
      while (__hip_atomic_load(&s_misc[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0u) {
        const uint32_t cur = __hip_atomic_load(&tab[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (cur == node) break;
        if (cur == EMPTY) {
          const uint32_t old = atomicCAS(&tab[h], EMPTY, node);
          if (old == EMPTY) {
            const uint32_t at = atomicAdd(&s_misc[0], 1u);
            if (at < RK_NODES) { dkey[at] = node; dslot[at] = h; }
            else __hip_atomic_store(&s_misc[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            break;
          }
          if (old == node) break;
        }
        h = (h + 1u) & (uint32_t)(LS_CAP - 1);
      }
      aux[j] = h;
    }
  }
  __syncthreads();
  const uint32_t nodes = s_misc[0];
  if (s_misc[1] != 0u || ((uint64_t)nodes << ib) > (uint64_t)RK_BITS) return false;
  // rank of every node among the distinct ones, left in its table slot
  if (nodes <= (uint32_t)LS_T) {
    // few: count the smaller keys.  A wavefront takes a quarter of the list against every node (one node per lane:
    // all lanes read the same word, a broadcast) and adds its count to the node's rank
    const uint32_t quarter = (nodes + 3u) / 4u, k0 = wave_id() * quarter, k1 = min(k0 + quarter, nodes);
    for (uint32_t n = lane_id(); n < nodes; n += 64) {
      const uint32_t mine = dkey[n];
      uint32_t r = 0;
#pragma unroll 8
      for (uint32_t k = k0; k < k1; ++k) r += dkey[k] < mine;
      if (r) atomicAdd(&s_start[n], r);
    }
    __syncthreads();
    if (threadIdx.x < nodes) tab[dslot[threadIdx.x]] = s_start[threadIdx.x];
  } else {
    const int nbits = low_bits > ib ? low_bits - ib : 1;
    if (nodes <= 2 * LS_T) lds_sort<LS_T, 2>(nodes, nbits, dkey, dslot, s_cnt, s_start, s_wave);
    else if (nodes <= 4 * LS_T) lds_sort<LS_T, 4>(nodes, nbits, dkey, dslot, s_cnt, s_start, s_wave);
    else lds_sort<LS_T, 8>(nodes, nbits, dkey, dslot, s_cnt, s_start, s_wave);
    for (uint32_t r = threadIdx.x; r < nodes; r += LS_T) tab[dslot[r]] = r;
  }
  __syncthreads();
  // (the list is no longer needed: its place takes a bit map of the occupied in-block positions, 1 << ib bits per
  // node, and the number of entries before every node)
  uint32_t *bm = s_val, *nstart = s_val + RK_NODES;
  const uint32_t nwords = ((nodes << ib) + 31u) >> 5;
  for (uint32_t w = threadIdx.x; w < nwords; w += LS_T) bm[w] = 0;
#pragma unroll
  for (int j = 0; j < IPT; ++j) aux[j] = tab[aux[j]];
  __syncthreads();
  const uint32_t imask = (1u << ib) - 1u;
  bool dup = false;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    if (threadIdx.x + j * LS_T < cnt) {
      const uint32_t bit = (aux[j] << ib) | (key[j] & imask);
      dup |= (atomicOr(&bm[bit >> 5], 1u << (bit & 31u)) >> (bit & 31u)) & 1u;
    }
  }
  if (dup) flags->duplicate = 1;
  __syncthreads();
  // entries before every node: consecutive nodes per thread, one if that covers them all
  constexpr int NPT = RK_NODES / LS_T;
  const int npt = nodes <= (uint32_t)LS_T ? 1 : NPT;
  uint32_t c[NPT], sum = 0, total;
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    const uint32_t r = threadIdx.x * npt + k;
    c[k] = (k < npt && r < nodes) ? rk_count(bm, r, ib, 1u << ib) : 0u;
    sum += c[k];
  }
  uint32_t run = block_exclusive_sum<LS_T>(sum, s_wave, &total);
#pragma unroll
  for (int k = 0; k < NPT; ++k) {
    if (k < npt) nstart[threadIdx.x * npt + k] = run;
    run += c[k];
  }
  __syncthreads();
  if (tile_count) {   // nodes that start in each of the output tiles the bucket touches
    uint32_t h[3] = {0, 0, 0};
    for (uint32_t base = 0; base < nodes; base += LS_T) {
      const uint32_t r = base + threadIdx.x;
      add_heads(r < nodes ? ((first + nstart[r]) >> NODE_TILE_SHIFT) - (first >> NODE_TILE_SHIFT) : 3u, h);
    }
    flush_heads(tile_count, h);
  }
#pragma unroll
  for (int j = 0; j < IPT; ++j)
    if (threadIdx.x + j * LS_T < cnt) aux[j] = nstart[aux[j]] + rk_count(bm, aux[j], ib, key[j] & imask);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    // (places collide only under a duplicate, which has been flagged; they stay below cnt either way)
    if (threadIdx.x + j * LS_T < cnt && aux[j] < cnt) {
      s_key[aux[j]] = key[j];
      s_val[aux[j]] = val[j];
    }
  }
  __syncthreads();
  return true;
}

template <int OUT>
__device__ __forceinline__ void local_emit(const LocalArgs &a, uint32_t bucket, uint32_t g, uint32_t k, uint32_t v) {
  const uint64_t full = ((uint64_t)bucket << a.low_bits) | (uint64_t)k;
  if (OUT == OUT_UNPACK) {
    a.major_out[g] = (int32_t)(full >> a.b_bits);
    a.minor_out[g] = (int32_t)(full & ((1ull << a.b_bits) - 1ull));
  } else {
    a.key64_out[g] = full;
  }
  a.val_out[g] = v;
}

// workgroup i < nbuckets: bucket i if it is small enough; workgroup nbuckets + g: group g of a split bucket.
// BLOCKED: keys of a blocked tuple, placed by node rank where the bucket allows it (rank_sort)
template <int OUT, bool BLOCKED>
__global__ __launch_bounds__(LS_T, 4) void local_sort_kernel(LocalArgs a) {
  __shared__ uint32_t s_key[LS_CAP];
  __shared__ uint32_t s_val[LS_CAP];
  __shared__ uint32_t s_cnt[LS_T / 64][RS_BINS];
  __shared__ uint32_t s_start[RS_BINS];
  __shared__ uint32_t s_wave[LS_T / 64 + 1];
  __shared__ uint32_t s_misc[2];
  // (one workgroup per possible group although most inputs have none: walking the groups with a stride instead put a
  // loop around the body that cost the common path a quarter of its speed, 329 -> 407 us on the FEM-like matrix)
  uint32_t first, cnt, bucket;
  const Rec *src;
  if (blockIdx.x < a.nbuckets) {
    bucket = blockIdx.x;
    if (!bucket_range(a, bucket, &first, &cnt) || cnt > (uint32_t)LS_CAP) return;
    src = a.rec_in;
  } else {
    const uint32_t g = blockIdx.x - a.nbuckets;
    if (g >= min(a.counters[2], a.work_cap)) return;
    const WorkItem wi = a.work[g];
    first = wi.first; cnt = wi.size; bucket = wi.bucket;
    if (cnt == 0 || cnt > (uint32_t)LS_CAP || first >= a.n || cnt > a.n - first) return;   // oversize pieces have set sort_retry
    src = a.rec_split;
  }
  const uint32_t low_mask = a.low_bits >= 32 ? 0xFFFFFFFFu : ((1u << a.low_bits) - 1u);
  // a work item of at most LS_CAP entries touches at most three output tiles, the first of them this one
  uint32_t *tile_count = (BLOCKED && a.node_count) ? a.node_count + (first >> NODE_TILE_SHIFT) : nullptr;
  bool placed = false;
  if (BLOCKED) {
    if (cnt <= 4 * LS_T) placed = rank_sort<4>(src, first, cnt, low_mask, a.low_bits, a.inner_bits, s_key, s_val, s_cnt, s_start, s_wave, s_misc, tile_count, a.flags);
    else if (cnt <= 8 * LS_T) placed = rank_sort<8>(src, first, cnt, low_mask, a.low_bits, a.inner_bits, s_key, s_val, s_cnt, s_start, s_wave, s_misc, tile_count, a.flags);
    else placed = rank_sort<16>(src, first, cnt, low_mask, a.low_bits, a.inner_bits, s_key, s_val, s_cnt, s_start, s_wave, s_misc, tile_count, a.flags);
  }
  if (!placed) {
    for (uint32_t i = threadIdx.x; i < cnt; i += LS_T) {
      const Rec r = src[first + i];
      s_key[i] = r.lo & low_mask;
      s_val[i] = r.val;
    }
    __syncthreads();
    if (cnt <= LS_T) lds_sort<LS_T, 1>(cnt, a.low_bits, s_key, s_val, s_cnt, s_start, s_wave);
    else if (cnt <= 2 * LS_T) lds_sort<LS_T, 2>(cnt, a.low_bits, s_key, s_val, s_cnt, s_start, s_wave);
    else if (cnt <= 4 * LS_T) lds_sort<LS_T, 4>(cnt, a.low_bits, s_key, s_val, s_cnt, s_start, s_wave);
    else if (cnt <= 8 * LS_T) lds_sort<LS_T, 8>(cnt, a.low_bits, s_key, s_val, s_cnt, s_start, s_wave);
    else lds_sort<LS_T, 16>(cnt, a.low_bits, s_key, s_val, s_cnt, s_start, s_wave);
  }
  bool dup = false;
  uint32_t h[3] = {0, 0, 0};
  const bool count_here = BLOCKED && tile_count && !placed;   // (rank_sort has counted its nodes itself)
  for (uint32_t base = 0; base < cnt; base += LS_T) {
    const uint32_t i = base + threadIdx.x;
    uint32_t which = 3u;
    if (i < cnt) {
      const uint32_t k = s_key[i];
      dup |= i > 0 && s_key[i - 1] == k;
      local_emit<OUT>(a, bucket, first + i, k, s_val[i]);
      // (the first entry of a work item starts a node: bucket and piece are told apart by bits of the node key,
      // which the host has checked before asking for the counts)
      if (count_here && (i == 0 || (k >> a.inner_bits) != (s_key[i - 1] >> a.inner_bits)))
        which = ((first + i) >> NODE_TILE_SHIFT) - (first >> NODE_TILE_SHIFT);
    }
    if (count_here) add_heads(which, h);
  }
  if (dup) a.flags->duplicate = 1;
  if (count_here) flush_heads(tile_count, h);
}

template <int IN>
static void launch_hist(Env &env, const PassArgs &a, double bytes) {
  US_LAUNCH(env, "radix_hist", bytes, (radix_hist_kernel<IN>), a.nblocks, RS_T, a);
}
template <int IN, int OUT>
static void launch_scatter(Env &env, const PassArgs &a, double bytes) {
  US_LAUNCH(env, "radix_scatter", bytes, (radix_scatter_kernel<IN, OUT>), a.tiles_per_xcd * 8u, RS_T, a);
}
template <int IN>
static void launch_scatter_out(Env &env, const PassArgs &a, int out_mode, double bytes) {
  switch (out_mode) {
    case OUT_UNPACK: launch_scatter<IN, OUT_UNPACK>(env, a, bytes); break;
    case OUT_KEY64: launch_scatter<IN, OUT_KEY64>(env, a, bytes); break;
    case OUT_KEY32: launch_scatter<IN, OUT_KEY32>(env, a, bytes); break;
    default: launch_scatter<IN, OUT_SPLIT>(env, a, bytes); break;
  }
}

// in_mode: IN_COO (row, col) or IN_KEY32 (key32_in).  Final output: unpacked (out.major set),
// 64-bit keys (out.key64) or 32-bit keys (out.key32).  Returns true when equal keys have been
// looked for (and flagged) on the way.
static bool sort_generic(Env &env, int in_mode, const int32_t *row, const int32_t *col, const uint32_t *key32_in,
                         const float *val, int64_t nnz, const KeySpec &ks, const SortOut &out_in, Flags *flags) {
  SortOut out = out_in;
  if (out.node_counted) *out.node_counted = false;
  if (nnz <= 0 || !env.ok()) {
    if (out.late && env.ok()) out.late(out);   // the caller still gets its (empty) arrays
    return false;
  }
  const int final_mode = (out.major || out.late) ? OUT_UNPACK : (out.key64 ? OUT_KEY64 : OUT_KEY32);
  const int total_bits = ks.total_bits > 0 ? ks.total_bits : 1;

  // Whole-array passes over the top `high_bits`, then the in-LDS finish over the rest: enough top
  // bits for buckets of 1024..2048 items on average, and at most 32 bits left over.
  int high_bits = total_bits, low_bits = 0;
  bool finish_local = false;
  // by default for blocked tuples only: block rows of FEM-like matrices fill evenly, while the rows of a
  // power-law graph do not (a heavy row's bucket needs extra splitting levels and the finish loses)
  // ... and for lists of at most RS_SMALL tiles whatever the tuple: there every launch costs more than the work it
  // does, and one digit pass + the finish is 9 launches where five digit passes are 15 (a row heavy enough to send
  // such a list back to the plain passes costs a tenth of a millisecond)
  const bool want_finish = env.lds_finish > 0 || (env.lds_finish < 0 && (ks.mode != 0 || nnz <= (int64_t)RS_SMALL * RS_TILE));
  if (want_finish && in_mode == IN_COO && final_mode != OUT_KEY32 && nnz >= 4096) {
    const int want = bits_for((uint64_t)(nnz - 1) / 2048);
    high_bits = want < total_bits ? want : total_bits;
    if (total_bits - high_bits > 32) high_bits = total_bits - 32;
    low_bits = total_bits - high_bits;
    finish_local = high_bits > 0 && high_bits <= want + 3;   // else: buckets of a few items each, not worth it
    if (!finish_local) { high_bits = total_bits; low_bits = 0; }
  }

  const int npass = ceil_div(high_bits, RS_MAXBITS);
  const uint32_t nblocks = (uint32_t)ceil_div<int64_t>(nnz, RS_TILE);
  const uint32_t nchunks = ceil_div<uint32_t>(nblocks, (uint32_t)RS_CHUNK);
  const int nrec = finish_local ? npass : npass - 1;   // passes that write records
  Rec *rbuf[2] = {nullptr, nullptr};
  uint8_t *dbuf[2] = {nullptr, nullptr};
  const uint32_t nbuckets = finish_local ? 1u << high_bits : 0u;
  LocalArgs la{};
  la.big_cap = (uint32_t)(nnz / LS_CAP) + 1;                 // a big bucket holds more than LS_CAP items
  la.tile_cap = (uint32_t)(nnz / RS_TILE) + la.big_cap;      // each has at most size/RS_TILE + 1 tiles
  la.work_cap = 2 * (uint32_t)(nnz / LS_GROUP) + la.big_cap; // ... and at most size/LS_GROUP + 1 groups that an interval opens, size/LS_GROUP that a large piece opens
  {  // everything below in one allocation
    auto g = [](size_t b) { return Env::granule(b); };
    size_t need = (nrec < 2 ? nrec : 2) * g(sizeof(Rec) * nnz) + (npass - 1 < 2 ? npass - 1 : 2) * g(nnz + 16) +
                  g(4ull * RS_BINS * nblocks) + g(4ull * RS_BINS * nchunks) + g(4ull * RS_BINS);
    if (finish_local)
      need += g(4ull * (nbuckets + 1)) + (npass >= 2 ? 0 : g(sizeof(Rec) * nnz)) + g(16) +
              g(sizeof(BigBucket) * la.big_cap) + g(4ull * la.tile_cap) + g(4ull * la.tile_cap * RS_BINS) +
              g(4ull * la.big_cap * RS_BINS) + g(sizeof(WorkItem) * la.work_cap);
    env.reserve(need);
  }
  for (int i = 0; i < 2 && i < nrec; ++i) rbuf[i] = env.temp<Rec>(nnz);
  for (int i = 0; i < 2 && i < npass - 1; ++i) dbuf[i] = env.temp<uint8_t>(nnz + 16);
  uint32_t *hist = env.temp<uint32_t>((size_t)RS_BINS * nblocks);
  uint32_t *chunk = env.temp<uint32_t>((size_t)RS_BINS * nchunks);
  uint32_t *dtotal = env.temp<uint32_t>(RS_BINS);
  if (!env.ok()) return false;

  int widths[16], shifts[16];
  for (int p = 0, sh = low_bits; p < npass; ++p) {
    widths[p] = high_bits / npass + (p < high_bits % npass ? 1 : 0);
    shifts[p] = sh;
    sh += widths[p];
  }
  const double kb = 8.0;  // key bytes between passes
  for (int p = 0; p < npass; ++p) {
    const bool first = p == 0, last_pass = p == npass - 1, last = last_pass && !finish_local;
    if (last && out.late) {
      out.late(out); out.late = nullptr;
      if (!env.ok()) return false;
    }
    PassArgs a{};
    a.row = first ? row : nullptr;
    a.col = first ? col : nullptr;
    a.lo_in = first ? key32_in : nullptr;
    a.rec_in = first ? nullptr : rbuf[(p - 1) & 1];
    a.val_in = first ? (const uint32_t *)val : nullptr;
    a.digit_in = first ? nullptr : dbuf[(p - 1) & 1];
    a.rec_out = last ? nullptr : rbuf[p & 1];
    a.digit_out = last_pass ? nullptr : dbuf[p & 1];
    a.val_out = last ? (uint32_t *)out.val : nullptr;
    a.major_out = last ? out.major : nullptr;
    a.minor_out = last ? out.minor : nullptr;
    a.key64_out = last ? out.key64 : nullptr;
    a.key32_out = last ? out.key32 : nullptr;
    a.n = (uint32_t)nnz; a.shift = shifts[p]; a.mask = (1u << widths[p]) - 1u; a.nblocks = nblocks;
    a.next_shift = last_pass ? 0 : shifts[p + 1];
    a.next_mask = last_pass ? 0u : (1u << widths[p + 1]) - 1u;
    a.tiles_per_xcd = ceil_div<uint32_t>(nblocks, 8u);
    a.hist = hist; a.chunk = chunk; a.dtotal = dtotal; a.nchunks = nchunks; a.ks = ks; a.flags = flags;
    a.hist_minor_only = first && in_mode == IN_COO && ks.mode == 0 && shifts[p] + widths[p] <= ks.b_bits && ks.b_bits <= 32;
    a.coo_vec = first && in_mode == IN_COO &&
                ((reinterpret_cast<uintptr_t>(row) | reinterpret_cast<uintptr_t>(col) | reinterpret_cast<uintptr_t>(val)) & 15u) == 0;
    const int lead_at = ks.b_bits + ks.ih_bits + ks.iw_bits;   // blocked keys: where the field a / bh starts
    a.hist_major_shift = (first && in_mode == IN_COO && ks.mode != 0 && shifts[p] >= lead_at) ? shifts[p] - lead_at : -1;

    const int in = first ? in_mode : IN_SPLIT;
    const int om = last ? final_mode : OUT_SPLIT;
    const double in_key = in == IN_COO ? 8.0 : (in == IN_KEY32 ? 4.0 : kb);
    const double out_key = om == OUT_UNPACK ? 8.0 : (om == OUT_KEY64 ? 8.0 : (om == OUT_KEY32 ? 4.0 : kb + 1.0));
    if (in == IN_COO) launch_hist<IN_COO>(env, a, (a.hist_minor_only || a.hist_major_shift >= 0 ? 4.0 : 8.0) * nnz);
    else if (in == IN_KEY32) launch_hist<IN_KEY32>(env, a, 4.0 * nnz);
    else launch_hist<IN_SPLIT>(env, a, 1.0 * nnz);
    if (nblocks <= (uint32_t)RS_SMALL) {
      US_LAUNCH(env, "radix_scan_small", 8.0 * RS_BINS * nblocks, radix_scan_small_kernel, 1, RS_BINS, hist, chunk, dtotal,
                nblocks, nchunks);
    } else {
      US_LAUNCH(env, "radix_scan_chunk", 8.0 * RS_BINS * nblocks, radix_scan_chunk_kernel, nchunks, RS_BINS, hist, chunk,
                nblocks);
      US_LAUNCH(env, "radix_scan_top", 8.0 * RS_BINS * nchunks, radix_scan_top_kernel, RS_BINS / 4, 256, chunk, nchunks,
                dtotal);
    }
    const double bytes = (in_key + 4.0 + out_key + 4.0) * nnz;
    if (in == IN_COO) launch_scatter_out<IN_COO>(env, a, om, bytes);
    else if (in == IN_KEY32) launch_scatter_out<IN_KEY32>(env, a, om, bytes);
    else launch_scatter_out<IN_SPLIT>(env, a, om, bytes);
  }
  if (!finish_local) return false;
  if (out.late) {
    out.late(out); out.late = nullptr;
    if (!env.ok()) return false;
  }

  la.nbuckets = nbuckets; la.n = (uint32_t)nnz; la.low_bits = low_bits; la.b_bits = ks.b_bits;
  uint32_t *off = env.temp<uint32_t>((size_t)nbuckets + 1);
  la.rec_in = rbuf[(npass - 1) & 1];
  la.rec_split = npass >= 2 ? rbuf[npass & 1] : env.temp<Rec>(nnz);
  la.counters = env.temp<uint32_t>(4);
  la.big = env.temp<BigBucket>(la.big_cap);
  la.tilemap = env.temp<uint32_t>(la.tile_cap);
  la.shist = env.temp<uint32_t>((size_t)la.tile_cap * RS_BINS);
  la.sdig = env.temp<uint32_t>((size_t)la.big_cap * RS_BINS);
  la.work = env.temp<WorkItem>(la.work_cap);
  if (!env.ok()) return false;
  la.off = off;
  la.major_out = out.major; la.minor_out = out.minor; la.key64_out = out.key64; la.val_out = (uint32_t *)out.val;
  la.flags = flags;
  // counters start at zero, and entries of `big` and `tilemap` that a garbage input (coordinates out of range) leaves
  // unwritten must still index safely: one fill when the three sit next to each other (carved from one block), else three
  {
    char *c0 = (char *)la.counters, *c1 = (char *)la.big, *c2 = (char *)la.tilemap;
    const size_t b0 = Env::granule(4 * sizeof(uint32_t)), b1 = Env::granule(sizeof(BigBucket) * la.big_cap);
    if (c1 == c0 + b0 && c2 == c1 + b1) {
      fill_u32(env, la.counters, (b0 + b1) / 4 + la.tile_cap, 0u);
    } else {
      fill_u32(env, la.counters, 4, 0u);
      fill_u32(env, (uint32_t *)la.big, (uint64_t)la.big_cap * 4, 0u);
      fill_u32(env, la.tilemap, la.tile_cap, 0u);
    }
  }
  US_LAUNCH(env, "bucket_offsets", 4.0 * nbuckets, bucket_offsets_kernel, ceil_div<uint32_t>(nbuckets + 1, 256u), 256,
            la.rec_in, la.n, low_bits, nbuckets, off);
  US_LAUNCH(env, "big_list", 8.0 * nbuckets, big_list_kernel, ceil_div<uint32_t>(nbuckets, 256u), 256, la);
  US_LAUNCH(env, "seg_hist", 0.0, seg_hist_kernel, min(la.tile_cap, SEG_GRID), RS_T, la);
  US_LAUNCH(env, "seg_scan", 0.0, seg_scan_kernel, min(la.big_cap, SEG_GRID), RS_BINS, la);
  US_LAUNCH(env, "seg_scatter", 0.0, seg_scatter_kernel, min(la.tile_cap, SEG_GRID), RS_T, la);
  // blocked tuples with in-block indices in the key (node keys of at most 31 bits): placement by node rank
  la.inner_bits = ks.mode == 1 ? ks.ih_bits + ks.iw_bits : (ks.mode == 2 ? ks.ih_bits : 0);
  const bool by_rank = la.inner_bits >= 1 && la.inner_bits <= 16;
  // nodes per output tile on the way: the first entry of every bucket and of every piece of a split bucket must
  // start a node, i.e. the bits that tell buckets and pieces apart must all belong to the node key
  const bool count_nodes = out.node_count && by_rank && final_mode == OUT_KEY64 && low_bits - RS_MAXBITS >= la.inner_bits;
  la.node_count = count_nodes ? out.node_count : nullptr;
  if (count_nodes) fill_u32(env, out.node_count, (uint64_t)ceil_div<int64_t>(nnz, NODE_TILE), 0u);
  if (out.node_counted) *out.node_counted = count_nodes;
  if (final_mode == OUT_UNPACK)
    US_LAUNCH(env, "local_sort", 24.0 * nnz, (local_sort_kernel<OUT_UNPACK, false>), nbuckets + la.work_cap, LS_T, la);
  else if (by_rank)
    US_LAUNCH(env, "local_sort", 24.0 * nnz, (local_sort_kernel<OUT_KEY64, true>), nbuckets + la.work_cap, LS_T, la);
  else
    US_LAUNCH(env, "local_sort", 24.0 * nnz, (local_sort_kernel<OUT_KEY64, false>), nbuckets + la.work_cap, LS_T, la);
  return true;
}

size_t sort_temp_bytes(int64_t nnz) {
  if (nnz <= 0) return 0;
  const size_t nblocks = (size_t)ceil_div<int64_t>(nnz, RS_TILE), nchunks = ceil_div<size_t>(nblocks, RS_CHUNK);
  return 2 * Env::granule(sizeof(Rec) * nnz) + 2 * Env::granule(nnz + 16) + Env::granule(4ull * RS_BINS * nblocks) +
         Env::granule(4ull * RS_BINS * nchunks) + Env::granule(4ull * RS_BINS);
}

bool sort_coo(Env &env, const int32_t *row, const int32_t *col, const float *val, int64_t nnz,
              const KeySpec &ks, const SortOut &out, Flags *flags_dev) {
  return sort_generic(env, IN_COO, row, col, nullptr, val, nnz, ks, out, flags_dev);
}

// stable ascending sort of 32-bit keys that carry a 32-bit payload
void sort_u32_payload(Env &env, const uint32_t *key, const uint32_t *payload, int64_t n, int bits, uint32_t *key_out,
                      uint32_t *payload_out, Flags *flags_dev) {
  if (n <= 0) return;
  KeySpec ks{};
  ks.total_bits = bits;
  SortOut so{};
  so.key32 = key_out; so.val = (float *)payload_out;   // the value slot carries 32 bits untouched
  sort_generic(env, IN_KEY32, nullptr, nullptr, key, (const float *)payload, n, ks, so, flags_dev);
}

}  // namespace us
