// The Sort operator of the conversion algorithm (Figure 8: "apply Sort to T_format";
// Section 7.2.1 reports it as 65 % of COO->BDIA conversion time, Section 7.2.3 as 84 % for
// Serpens) as a least-significant-digit radix sort over packed target tuples.
//
// One digit pass = per-tile digit histogram, per-digit scan over the tiles, stable tile
// scatter (wavefront-ballot ranking, tile reordered through LDS so that every digit's run is
// written as one contiguous piece).  The first pass builds the keys from (row, col) on the
// fly (index-map evaluation: Swap, TileSplit), the last one can unpack them into index
// arrays, so keys never take an extra trip through HBM.
//
// A single-kernel pass with a decoupled look-back over per-tile status words was tried and
// dropped: with ~770 tiles resident at once and status words that must cross the XCDs' L2s,
// the serial look-back (one device-scope load per predecessor and digit) ran 40x slower than
// the separate histogram + scan.
#include "common.h"
#include "device.h"

namespace us {

constexpr int RS_T = 512, RS_IPT = 8, RS_TILE = RS_T * RS_IPT, RS_NW = RS_T / 64, RS_MAXBITS = 8, RS_BINS = 1 << RS_MAXBITS;

template <typename K>
__device__ __forceinline__ K build_key(const KeySpec &ks, uint32_t r, uint32_t c) {
  uint32_t a = ks.swap ? c : r, b = ks.swap ? r : c;
  if (ks.mode == 0) return ((K)a << ks.b_bits) | (K)b;
  uint32_t ab = a / ks.bh, ai = a - ab * ks.bh, bb = b / ks.bw, bi = b - bb * ks.bw;
  return (((((K)ab << ks.b_bits) | (K)bb) << ks.ih_bits | (K)ai) << ks.iw_bits) | (K)bi;
}

template <typename K>
struct PassArgs {
  const int32_t *row, *col;      // COO input (first pass) or null
  const K *key_in;               // packed input otherwise
  const uint32_t *val_in;
  K *key_out; uint32_t *val_out; // packed output, or
  int32_t *major_out, *minor_out;  // unpacked output (last pass, mode 0)
  uint32_t n; int shift; uint32_t mask; uint32_t nblocks;
  const uint8_t *digit_in;       // this pass's digit of every input item (written by the previous pass) or null
  uint8_t *digit_out;            // next pass's digit of every output item, or null
  int next_shift; uint32_t next_mask;
  uint32_t tiles_per_xcd;        // launch index -> tile mapping (see xcd_tile)
  uint32_t *hist;                // [nblocks][RS_BINS] per-tile digit counts, then prefixes inside a chunk of tiles
  uint32_t *chunk;               // [RS_BINS][nchunks] per-chunk digit counts, then prefixes over the chunks
  uint32_t *dtotal;              // [RS_BINS] digit totals of the whole input
  uint32_t nchunks;
  KeySpec ks;
  Flags *flags;
};

template <typename K, bool FROM_COO>
__device__ __forceinline__ K load_key(const PassArgs<K> &a, uint32_t i) {
  if (FROM_COO) return build_key<K>(a.ks, (uint32_t)a.row[i], (uint32_t)a.col[i]);
  return a.key_in[i];
}

// Workgroups are dealt round-robin to the 8 XCDs.  Mapping launch index i to tile
// (i % 8) * tiles_per_xcd + i / 8 lets each XCD work through one contiguous range of tiles, so
// the partial cache lines at the ends of neighbouring tiles' runs meet in the same L2.
__device__ __forceinline__ uint32_t xcd_tile(uint32_t i, uint32_t per_xcd) { return (i & 7u) * per_xcd + (i >> 3); }

template <typename K, bool FROM_COO>
__global__ __launch_bounds__(RS_T) void radix_hist_kernel(PassArgs<K> a) {
  __shared__ uint32_t s_hist[RS_BINS];
  for (int i = threadIdx.x; i < RS_BINS; i += RS_T) s_hist[i] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * RS_TILE;
  uint32_t digit[RS_IPT];
  if (!FROM_COO && a.digit_in) {
    // the previous pass left this pass's digits as bytes: 8 per thread in one 8-byte load
    const uint32_t i = base + threadIdx.x * RS_IPT;
    if (i + RS_IPT <= a.n) {
      uint2 v = *reinterpret_cast<const uint2 *>(a.digit_in + i);
#pragma unroll
      for (int k = 0; k < 4; ++k) { digit[k] = (v.x >> (8 * k)) & 0xFFu; digit[4 + k] = (v.y >> (8 * k)) & 0xFFu; }
    } else {
#pragma unroll
      for (int k = 0; k < RS_IPT; ++k) digit[k] = i + k < a.n ? a.digit_in[i + k] : 0xFFFFFFFFu;
    }
  } else {
    bool bad = false;
    K key[RS_IPT];
#pragma unroll
    for (int k = 0; k < RS_IPT; ++k) {   // all loads first: the memory system sees 8 requests per thread
      uint32_t i = base + k * RS_T + threadIdx.x;
      key[k] = 0;
      if (i < a.n) {
        if (FROM_COO) {
          uint32_t r = (uint32_t)a.row[i], c = (uint32_t)a.col[i];
          uint32_t ra = a.ks.swap ? c : r, cb = a.ks.swap ? r : c;
          bad |= (ra >= a.ks.a_extent) | (cb >= a.ks.b_extent);
          key[k] = build_key<K>(a.ks, r, c);
        } else {
          key[k] = a.key_in[i];
        }
      }
    }
#pragma unroll
    for (int k = 0; k < RS_IPT; ++k) {
      uint32_t i = base + k * RS_T + threadIdx.x;
      digit[k] = i < a.n ? ((uint32_t)(key[k] >> a.shift) & a.mask) : 0xFFFFFFFFu;
    }
    if (FROM_COO && bad) a.flags->index_range = 1;
  }
#pragma unroll
  for (int k = 0; k < RS_IPT; ++k)
    if (digit[k] != 0xFFFFFFFFu) atomicAdd(&s_hist[digit[k]], 1u);
  __syncthreads();
  for (uint32_t d = threadIdx.x; d < RS_BINS; d += RS_T) a.hist[(size_t)blockIdx.x * RS_BINS + d] = s_hist[d];
}

// Offsets of every (tile, digit) run without a single atomic (same-address device atomics cost
// ~20 ns each on this part and would serialise thousands of tiles):
//   chunk kernel: a workgroup takes RS_CHUNK consecutive tiles, thread d walks digit d through
//                 them (coalesced rows), leaving prefixes inside the chunk and the chunk total;
//   top kernel:   one wavefront per digit scans the chunk totals and leaves the digit total;
//   the scatter kernel adds the start of the digit (a 256-entry scan it does itself).
constexpr int RS_CHUNK = 32;

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

// one wavefront per digit: exclusive scan of the chunk totals of that digit, digit total
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

template <typename K, bool FROM_COO, bool UNPACK>
__global__ __launch_bounds__(RS_T) void radix_scatter_kernel(PassArgs<K> a) {
  __shared__ uint32_t s_cnt[RS_NW][RS_BINS];  // per-wave digit counts, then per-wave bases
  __shared__ uint32_t s_start[RS_BINS];       // first in-tile position of each digit
  __shared__ uint32_t s_goff[RS_BINS];        // global position of the digit's run minus s_start
  __shared__ uint32_t s_wave[RS_T / 64 + 1];
  __shared__ K s_key[RS_TILE];
  uint32_t *s_val = reinterpret_cast<uint32_t *>(s_key);

  const int lane = lane_id(), w = wave_id();
  const uint32_t nbins = a.mask + 1;
  for (uint32_t i = threadIdx.x; i < RS_NW * RS_BINS; i += RS_T) (&s_cnt[0][0])[i] = 0;

  const uint32_t tile = xcd_tile(blockIdx.x, a.tiles_per_xcd);
  if (tile >= a.nblocks) return;  // uniform: the launch is padded to 8 * tiles_per_xcd workgroups
  const uint32_t base = tile * RS_TILE;
  const uint32_t in_tile = min((uint32_t)RS_TILE, a.n - base);
  K key[RS_IPT];
  uint32_t val[RS_IPT], pos[RS_IPT];
  // wave w owns the contiguous slice [w*64*IPT, (w+1)*64*IPT) of the tile, lanes striped
#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    if (t < in_tile) {
      key[j] = load_key<K, FROM_COO>(a, base + t);
      val[j] = FROM_COO ? ((const uint32_t *)a.val_in)[base + t] : a.val_in[base + t];
    } else {
      key[j] = 0; val[j] = 0;
    }
  }
  __syncthreads();

  // stable rank of every item among the items of its wave with the same digit
#pragma unroll
  for (int j = 0; j < RS_IPT; ++j) {
    uint32_t t = w * (64 * RS_IPT) + j * 64 + lane;
    bool valid = t < in_tile;
    uint32_t d = (uint32_t)(key[j] >> a.shift) & a.mask;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < RS_MAXBITS; ++b) {
      uint64_t bal = __ballot((d >> b) & 1u);
      peers &= ((d >> b) & 1u) ? bal : ~bal;
    }
    uint32_t before = __popcll(peers & lanes_below());
    int leader = __ffsll((unsigned long long)peers) - 1;
    uint32_t old = 0;
    if (valid && lane == leader) {
      old = s_cnt[w][d];
      s_cnt[w][d] = old + (uint32_t)__popcll(peers);
    }
    old = __shfl(old, leader < 0 ? 0 : leader);
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
#pragma unroll
  for (int k = 0; k < RS_IPT; ++k) {
    uint32_t i = k * RS_T + threadIdx.x;
    if (i < in_tile) {
      K kk = s_key[i];
      uint32_t g = s_goff[(uint32_t)(kk >> a.shift) & a.mask] + i;
      gpos[k] = g;
      if (UNPACK) {
        a.major_out[g] = (int32_t)(kk >> a.ks.b_bits);
        a.minor_out[g] = (int32_t)(kk & (((K)1 << a.ks.b_bits) - 1));
      } else {
        a.key_out[g] = kk;
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
    if (i < in_tile) a.val_out[gpos[k]] = s_val[i];
  }
}

template <typename K>
static void sort_generic(Env &env, const int32_t *row, const int32_t *col, const K *key_in, const float *val,
                         int64_t nnz, const KeySpec &ks, const SortOut &out, Flags *flags) {
  if (nnz <= 0 || !env.ok()) return;
  const bool unpack = out.major != nullptr;
  const int total_bits = ks.total_bits > 0 ? ks.total_bits : 1;
  const int npass = ceil_div(total_bits, RS_MAXBITS);
  const uint32_t nblocks = (uint32_t)ceil_div<int64_t>(nnz, RS_TILE);
  K *kbuf[2] = {nullptr, nullptr};
  uint32_t *vbuf[2] = {nullptr, nullptr};
  for (int i = 0; i < 2 && i < npass - 1; ++i) {
    kbuf[i] = env.temp<K>(nnz);
    vbuf[i] = env.temp<uint32_t>(nnz);
  }
  uint8_t *dbuf[2] = {nullptr, nullptr};   // digit bytes handed from one pass to the next
  for (int i = 0; i < 2 && i < npass - 1; ++i) dbuf[i] = env.temp<uint8_t>(nnz + 16);
  const uint32_t nchunks = ceil_div<uint32_t>(nblocks, (uint32_t)RS_CHUNK);
  uint32_t *hist = env.temp<uint32_t>((size_t)RS_BINS * nblocks);
  uint32_t *chunk = env.temp<uint32_t>((size_t)RS_BINS * nchunks);
  uint32_t *dtotal = env.temp<uint32_t>(RS_BINS);
  if (!env.ok()) return;

  K *packed_out = sizeof(K) == 8 ? (K *)out.key64 : (K *)out.key32;
  int widths[16], shifts[16];
  for (int p = 0, sh = 0; p < npass; ++p) {
    widths[p] = total_bits / npass + (p < total_bits % npass ? 1 : 0);
    shifts[p] = sh;
    sh += widths[p];
  }
  const uint32_t tiles_per_xcd = ceil_div<uint32_t>(nblocks, 8u);
  for (int p = 0; p < npass; ++p) {
    const int width = widths[p], shift = shifts[p];
    const bool first = p == 0, last = p == npass - 1;
    PassArgs<K> a{};
    a.digit_in = first ? nullptr : dbuf[(p - 1) & 1];
    a.digit_out = last ? nullptr : dbuf[p & 1];
    a.next_shift = last ? 0 : shifts[p + 1];
    a.next_mask = last ? 0u : (1u << widths[p + 1]) - 1u;
    a.tiles_per_xcd = tiles_per_xcd;
    const bool from_coo = first && row != nullptr;
    a.row = from_coo ? row : nullptr;
    a.col = from_coo ? col : nullptr;
    a.key_in = first ? key_in : kbuf[(p - 1) & 1];
    a.val_in = first ? (const uint32_t *)val : vbuf[(p - 1) & 1];
    a.key_out = last ? (unpack ? nullptr : packed_out) : kbuf[p & 1];
    a.val_out = last ? (uint32_t *)out.val : vbuf[p & 1];
    a.major_out = last ? out.major : nullptr;
    a.minor_out = last ? out.minor : nullptr;
    a.n = (uint32_t)nnz; a.shift = shift; a.mask = (1u << width) - 1u; a.nblocks = nblocks;
    a.hist = hist; a.chunk = chunk; a.dtotal = dtotal; a.nchunks = nchunks; a.ks = ks; a.flags = flags;
    const double kb = sizeof(K);
    if (from_coo) US_LAUNCH(env, "radix_hist", 8.0 * nnz, (radix_hist_kernel<K, true>), nblocks, RS_T, a);
    else US_LAUNCH(env, "radix_hist", (first ? kb : 1.0) * nnz, (radix_hist_kernel<K, false>), nblocks, RS_T, a);
    US_LAUNCH(env, "radix_scan_chunk", 8.0 * RS_BINS * nblocks, radix_scan_chunk_kernel, nchunks, RS_BINS, hist, chunk,
              nblocks);
    US_LAUNCH(env, "radix_scan_top", 8.0 * RS_BINS * nchunks, radix_scan_top_kernel, RS_BINS / 4, 256, chunk, nchunks,
              dtotal);
    const double rd = (from_coo ? 12.0 : kb + 4.0) * nnz;
    const double wr = ((last && unpack) ? 12.0 : kb + 4.0 + (last ? 0.0 : 1.0)) * nnz;
    const uint32_t sgrid = tiles_per_xcd * 8u;
    if (from_coo && last && unpack) US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, true, true>), sgrid, RS_T, a);
    else if (from_coo && last) US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, true, false>), sgrid, RS_T, a);
    else if (from_coo) US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, true, false>), sgrid, RS_T, a);
    else if (last && unpack) US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, false, true>), sgrid, RS_T, a);
    else US_LAUNCH(env, "radix_scatter", rd + wr, (radix_scatter_kernel<K, false, false>), sgrid, RS_T, a);
  }
}

void sort_coo(Env &env, const int32_t *row, const int32_t *col, const float *val, int64_t nnz,
              const KeySpec &ks, const SortOut &out, Flags *flags_dev) {
  const bool k32 = ks.total_bits <= 32 && out.key64 == nullptr;
  if (k32) sort_generic<uint32_t>(env, row, col, nullptr, val, nnz, ks, out, flags_dev);
  else sort_generic<uint64_t>(env, row, col, nullptr, val, nnz, ks, out, flags_dev);
}

// ascending sort of 32-bit keys (no payload of interest)
void sort_u32(Env &env, const uint32_t *key, int64_t n, int bits, uint32_t *out, Flags *flags_dev) {
  if (n <= 0) return;
  KeySpec ks{};
  ks.total_bits = bits;
  float *dummy_in = env.temp<float>(n), *dummy_out = env.temp<float>(n);
  if (!env.ok()) return;
  SortOut so{};
  so.key32 = out; so.val = dummy_out;
  sort_generic<uint32_t>(env, nullptr, nullptr, key, dummy_in, n, ks, so, flags_dev);
}

void sort_keys(Env &env, const uint64_t *key, const float *val, int64_t nnz, const KeySpec &ks,
               const SortOut &out, Flags *flags_dev) {
  sort_generic<uint64_t>(env, nullptr, nullptr, key, val, nnz, ks, out, flags_dev);
}

}  // namespace us
