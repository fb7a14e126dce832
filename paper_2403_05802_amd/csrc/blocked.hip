// Blocked layouts from one sort by the blocked tuple (TileSplit in the key build): BCSR and the blocked DIA of
// Figure 3c (dense inner levels filled from the sorted list), and CSB (a dense grid of compressed blocks).
#include "convert_internal.h"
#include "device.h"

namespace us {

// ------------------------------------------------------------------ BCSR
// After sorting by (d0/bh, d1/bw, d0%bh, d1%bw) the entries of a block are contiguous.
// Merge(0,1): head flag where the block prefix changes, scan -> block id.
constexpr int BE_T = 256, BE_IPT = 8, BE_TILE = BE_T * BE_IPT;
static_assert(BE_TILE == NODE_TILE, "the sort counts nodes per tile of the emit kernel");

__global__ __launch_bounds__(BE_T) void bcsr_count_kernel(const uint64_t *key, int64_t n, int inner_bits,
                                                         uint32_t *partial, Flags *flags) {
  __shared__ uint32_t s_wave[BE_T / 64 + 1];
  int64_t base = (int64_t)blockIdx.x * BE_TILE;
  uint32_t heads = 0;
  bool dup = false;
#pragma unroll
  for (int k = 0; k < BE_IPT; ++k) {
    int64_t i = base + k * BE_T + threadIdx.x;
    if (i < n) {
      uint64_t cur = key[i], prev = i > 0 ? key[i - 1] : ~0ull;
      dup |= (i > 0) & (cur == prev);
      heads += (i == 0) | ((cur >> inner_bits) != (prev >> inner_bits));
    }
  }
  if (dup) flags->duplicate = 1;
  uint32_t total;
  block_exclusive_sum<BE_T>(heads, s_wave, &total);
  if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

__global__ __launch_bounds__(BE_T) void bcsr_emit_kernel(const uint64_t *key, const float *val, int64_t n,
                                                        KeySpec ks, int32_t col_bias, const uint32_t *partial,
                                                        int32_t *blk_row, int32_t *blk_col, float *bval) {
  __shared__ uint32_t s_wave[BE_T / 64 + 1];
  const int inner_bits = ks.ih_bits + ks.iw_bits;
  const int lane = lane_id();
  // a wavefront owns 64*BE_IPT consecutive entries, lanes striped (coalesced loads); block ids
  // come from ballots of the head flags, so no per-thread serial run is needed
  const int64_t wbase = (int64_t)blockIdx.x * BE_TILE + (int64_t)wave_id() * (64 * BE_IPT);
  uint64_t k[BE_IPT];
  uint64_t hb[BE_IPT];   // ballot of head flags of item j
  uint32_t wave_total = 0;
  uint64_t last_prev = (wbase > 0 && wbase <= n) ? key[wbase - 1] : ~0ull;  // key before the wave's slice
#pragma unroll
  for (int j = 0; j < BE_IPT; ++j) {
    const int64_t i = wbase + j * 64 + lane;
    k[j] = i < n ? key[i] : ~0ull;
  }
#pragma unroll
  for (int j = 0; j < BE_IPT; ++j) {
    const int64_t i = wbase + j * 64 + lane;
    uint64_t prev = __shfl_up(k[j], 1);
    if (lane == 0) prev = last_prev;
    const bool head = (i < n) && ((i == 0) | ((k[j] >> inner_bits) != (prev >> inner_bits)));
    hb[j] = __ballot(head);
    wave_total += (uint32_t)__popcll(hb[j]);
    last_prev = __shfl(k[j], 63);
  }
  uint32_t total;
  uint32_t wave_base = block_exclusive_sum<BE_T>(lane == 0 ? wave_total : 0u, s_wave, &total);
  uint32_t run = __shfl(wave_base, 0) + partial[blockIdx.x];  // blocks before this wave's slice
  const uint32_t bsz = ks.bh * ks.bw;
#pragma unroll
  for (int j = 0; j < BE_IPT; ++j) {
    const int64_t i = wbase + j * 64 + lane;
    if (i < n) {
      const bool head = (hb[j] >> lane) & 1ull;
      const uint32_t blk = run + (uint32_t)__popcll(hb[j] & (lanes_below() | (1ull << lane))) - 1;
      const uint32_t bi = (uint32_t)(k[j] & ((1ull << ks.iw_bits) - 1));
      const uint32_t ai = (uint32_t)((k[j] >> ks.iw_bits) & ((1ull << ks.ih_bits) - 1));
      const uint64_t bk = k[j] >> inner_bits;
      if (head) {
        blk_col[blk] = (int32_t)(bk & ((1ull << ks.b_bits) - 1)) - col_bias;
        blk_row[blk] = (int32_t)(bk >> ks.b_bits);
      }
      bval[(size_t)blk * bsz + ai * ks.bw + bi] = val[i];
    }
    run += (uint32_t)__popcll(hb[j]);
  }
}

// Blocked ELL from the block lists of BCSR: block b of block row br sits in slot k = b - ptr[br] (the enum query over
// the blocks of a block row, ascending block column); its block column goes to ecol[k * nbr + br] and its values to
// the slot-major slab.  A thread per value; slab and ecol start out as padding (0 and -1).
__global__ __launch_bounds__(256) void bell_fill_kernel(const int32_t *ptr, const int32_t *blk_row, const int32_t *blk_col,
                                                       const float *bval, int64_t nvals, int bsz, int64_t nbr, int64_t K,
                                                       int32_t *ecol, float *eval, Flags *flags) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= nvals) return;
  const int64_t b = e / bsz;
  const int in = (int)(e - b * bsz);
  const int64_t br = blk_row[b], k = b - ptr[br];
  if (k >= K) { flags->ell_overflow = 1; return; }   // a block row with more blocks than a fixed width allows
  if (in == 0) ecol[k * nbr + br] = blk_col[b];
  eval[(k * nbr + br) * bsz + in] = bval[e];
}

// Key layout of the two blocked families: BCSR (d0/bh, d1/bw, d0%bh, d1%bw) and BDIA
// (d0/bh, d1-d0 biased by nrows-1, d0%bh).
KeySpec blocked_keyspec(const Plan &plan, int64_t nrows, int64_t ncols) {
  const int64_t nbr = ceil_div<int64_t>(nrows, plan.bh);
  KeySpec ks{};
  ks.swap = 0; ks.bh = (uint32_t)plan.bh; ks.bw = (uint32_t)plan.bw;
  ks.a_extent = (uint32_t)nrows; ks.b_extent = (uint32_t)ncols;
  ks.ih_bits = bits_for(plan.bh - 1);
  if (plan.pattern == P_BDIA) {
    ks.mode = 2; ks.b_bits = bits_for(nrows + ncols - 2); ks.iw_bits = 0;
  } else {
    ks.mode = 1; ks.b_bits = bits_for(ceil_div<int64_t>(ncols, plan.bw) - 1); ks.iw_bits = bits_for(plan.bw - 1);
  }
  ks.total_bits = bits_for(nbr - 1) + ks.b_bits + ks.ih_bits + ks.iw_bits;
  return ks;
}

// Sorted keys -> ptr/idx of the merged node level and the zero-filled dense inner levels.
us_status emit_blocked(Env &env, const Plan &plan, const us_format_desc &desc, int64_t nrows, int64_t ncols,
                       const KeySpec &ks, const uint64_t *skey, const float *sval, int64_t n, Flags *flags,
                       us_formatted **out, uint32_t *node_count) {
  const int64_t nbr = ceil_div<int64_t>(nrows, plan.bh);
  const int64_t nb = ceil_div<int64_t>(n > 0 ? n : 1, BE_TILE);
  // nodes that start in every tile: counted by the sort already (node_count), or here (which also looks for equal keys)
  uint32_t *partial = node_count ? node_count : env.temp<uint32_t>(nb);
  if (!env.ok()) return env.status;
  if (!node_count)
    US_LAUNCH(env, "bcsr_count", 8.0 * n, bcsr_count_kernel, nb, BE_T, skey, n, ks.ih_bits + ks.iw_bits, partial, flags);
  // (one workgroup scanning 24,576 tile counts took 29 us; reduce + scan of the sums + apply takes three short launches)
  if (nb > 8192) exclusive_scan_i32(env, (const int32_t *)partial, (int32_t *)partial, nb, &flags->scalar[0]);
  else scan_partials_launch(env, partial, nb, &flags->scalar[0]);
  Flags h{};
  if (!read_flags(env, flags, &h)) return env.status;
  if (flag_status(h) != US_OK) return flag_status(h);
  const int64_t nblk = h.scalar[0], bsz = plan.bh * plan.bw;
  if (nblk * bsz >= (1ll << 31)) return US_ERR_OVERFLOW;
  const bool bdia = plan.pattern == P_BDIA;
  if (plan.pattern == P_BELL) {
    // the block lists of BCSR in temporaries, the most blocks a block row holds, then the slot-major slabs
    int32_t *ptr = env.temp<int32_t>(nbr + 1), *bidx = env.temp<int32_t>(nblk), *blk_row = env.temp<int32_t>(nblk);
    float *bval = env.temp<float>(nblk * bsz);
    if (!env.ok()) return env.status;
    if (nblk * bsz != n) fill_u32(env, (uint32_t *)bval, nblk * bsz, 0u);
    if (n > 0)
      US_LAUNCH(env, "bcsr_emit", 12.0 * n + 4.0 * n, bcsr_emit_kernel, nb, BE_T, skey, sval, n, ks, (int32_t)0,
                (const uint32_t *)partial, blk_row, bidx, bval);
    lower_bound_ptr(env, blk_row, nblk, nbr, ptr);
    int64_t K = plan.ell_width;
    if (K == 0) {
      fill_u32(env, (uint32_t *)&flags->scalar[1], 1, 0u);
      max_group_len(env, ptr, nbr, &flags->scalar[1]);
      if (!read_flags(env, flags, &h)) return env.status;
      K = h.scalar[1];
    }
    if (K * nbr * bsz >= (1ll << 31)) return US_ERR_OVERFLOW;
    us_formatted *f = new us_formatted();
    f->desc = desc; f->pattern = P_BELL;
    f->nrows = nrows; f->ncols = ncols; f->nnz = n;
    f->nlevels = 5;
    f->level[0].size = K; f->level[1].size = nbr; f->level[3].size = plan.bh; f->level[4].size = plan.bw;
    const int64_t nslots = K * nbr;
    if (env.one_result) env.reserve_out(Env::granule(4 * (size_t)nslots) + Env::granule(4 * (size_t)(nslots * bsz)));
    f->level[2].idx = env.owned<int32_t>(nslots); f->level[2].nidx = nslots;
    f->val = env.owned<float>(nslots * bsz); f->nval = nslots * bsz;
    f->nmajor = K; f->bh = plan.bh; f->bw = plan.bw; f->nblk = nbr;
    if (!env.ok()) { free_formatted(env, f); return env.status; }
    fill_u32(env, (uint32_t *)f->level[2].idx, nslots, 0xFFFFFFFFu);
    fill_u32(env, (uint32_t *)f->val, nslots * bsz, 0u);
    if (nblk > 0)
      US_LAUNCH(env, "bell_fill", 8.0 * nblk * bsz + 12.0 * nblk, bell_fill_kernel, ceil_div<int64_t>(nblk * bsz, 256), 256,
                (const int32_t *)ptr, (const int32_t *)blk_row, (const int32_t *)bidx, (const float *)bval, nblk * bsz,
                (int)bsz, nbr, K, f->level[2].idx, f->val, flags);
    if (!read_flags(env, flags, &h)) { free_formatted(env, f); return env.status; }
    if (flag_status(h) != US_OK) { free_formatted(env, f); return flag_status(h); }
    *out = f;
    return US_OK;
  }
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = plan.pattern;
  f->nrows = nrows; f->ncols = ncols; f->nnz = n;
  f->nlevels = bdia ? 3 : 4;
  f->level[0].size = nbr;
  if (env.one_result)   // the sizes are known now: one block for the three arrays
    env.reserve_out(Env::granule(4 * (size_t)(nbr + 1)) + Env::granule(4 * (size_t)nblk) + Env::granule(4 * (size_t)(nblk * bsz)));
  f->level[1].ptr = env.owned<int32_t>(nbr + 1); f->level[1].nptr = nbr + 1;
  f->level[1].idx = env.owned<int32_t>(nblk); f->level[1].nidx = nblk;
  f->level[2].size = plan.bh;
  if (!bdia) f->level[3].size = plan.bw;
  f->val = env.owned<float>(nblk * bsz); f->nval = nblk * bsz;
  f->nmajor = nbr; f->bh = plan.bh; f->bw = plan.bw; f->nblk = nblk;
  int32_t *blk_row = env.temp<int32_t>(nblk);
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  // (the flags just read say that the keys are distinct and in range: with as many entries as slots every slot
  // receives a value and nothing needs clearing first)
  if (nblk * bsz != n) fill_u32(env, (uint32_t *)f->val, nblk * bsz, 0u);
  if (n > 0)
    US_LAUNCH(env, "bcsr_emit", 12.0 * n + 4.0 * n, bcsr_emit_kernel, nb, BE_T, skey, sval, n, ks,
              (int32_t)(bdia ? nrows - 1 : 0), (const uint32_t *)partial, blk_row, f->level[1].idx, f->val);
  lower_bound_ptr(env, blk_row, nblk, nbr, f->level[1].ptr);
  env.sync();
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  *out = f;
  return US_OK;
}

us_status convert_blocked(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc,
                          Flags *flags, us_formatted **out) {
  const int64_t n = coo.nnz;
  const KeySpec ks = blocked_keyspec(plan, coo.nrows, coo.ncols);
  if (ks.total_bits > 64) return US_ERR_OVERFLOW;
  uint64_t *skey = env.temp<uint64_t>(n);
  float *sval = env.temp<float>(n);
  uint32_t *node_count = env.temp<uint32_t>(ceil_div<int64_t>(n > 0 ? n : 1, BE_TILE));
  if (!env.ok()) return env.status;
  SortOut so{};
  bool counted = false;
  so.key64 = skey; so.val = sval; so.node_count = node_count; so.node_counted = &counted;
  const bool dups_checked = sort_coo(env, coo.row, coo.col, coo.val, n, ks, so, flags);
  return emit_blocked(env, plan, desc, coo.nrows, coo.ncols, ks, skey, sval, n, flags, out,
                      counted && dups_checked ? node_count : nullptr);
}

// CSB (Section 2.1: a dense collection of blocks stored compressed): the entries in BCSR tuple order, a ptr
// over all blocks of the dense grid, and the two in-block indices of every entry.
__global__ __launch_bounds__(256) void csb_unpack_kernel(const uint64_t *key, int64_t n, KeySpec ks, int64_t nbc,
                                                        int32_t *blk, int32_t *in_row, int32_t *in_col, Flags *flags) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const uint64_t k = key[i];
  if (i > 0 && key[i - 1] == k) flags->duplicate = 1;
  const uint64_t bk = k >> (ks.ih_bits + ks.iw_bits);
  blk[i] = (int32_t)((int64_t)(bk >> ks.b_bits) * nbc + (int64_t)(bk & ((1ull << ks.b_bits) - 1)));
  in_row[i] = (int32_t)((k >> ks.iw_bits) & ((1ull << ks.ih_bits) - 1));
  in_col[i] = (int32_t)(k & ((1ull << ks.iw_bits) - 1));
}

us_status convert_csb(Env &env, const us_coo &coo, const Plan &plan, const us_format_desc &desc, Flags *flags,
                      us_formatted **out) {
  const int64_t n = coo.nnz;
  const int64_t nbr = ceil_div<int64_t>(coo.nrows, plan.bh), nbc = ceil_div<int64_t>(coo.ncols, plan.bw);
  if (nbr * nbc + 1 >= (1ll << 31)) return US_ERR_OVERFLOW;
  Plan pk = plan; pk.pattern = P_BCSR;   // same target tuple as BCSR
  const KeySpec ks = blocked_keyspec(pk, coo.nrows, coo.ncols);
  uint64_t *skey = env.temp<uint64_t>(n);
  int32_t *blk = env.temp<int32_t>(n);
  us_formatted *f = new us_formatted();
  f->desc = desc; f->pattern = P_CSB;
  f->nrows = coo.nrows; f->ncols = coo.ncols; f->nnz = n;
  f->nlevels = 4;
  f->level[0].size = nbr; f->level[1].size = nbc;
  f->level[2].ptr = env.owned<int32_t>(nbr * nbc + 1); f->level[2].nptr = nbr * nbc + 1;
  f->level[2].idx = env.owned<int32_t>(n); f->level[2].nidx = n;
  f->level[3].idx = env.owned<int32_t>(n); f->level[3].nidx = n;
  f->val = env.owned<float>(n); f->nval = n;
  f->nmajor = nbr * nbc; f->bh = plan.bh; f->bw = plan.bw; f->nblk = nbr * nbc;
  if (!env.ok()) { free_formatted(env, f); return env.status; }
  SortOut so{};
  so.key64 = skey; so.val = f->val;
  sort_coo(env, coo.row, coo.col, coo.val, n, ks, so, flags);
  if (n > 0)
    US_LAUNCH(env, "csb_unpack", 20.0 * n, csb_unpack_kernel, ceil_div<int64_t>(n, 256), 256, (const uint64_t *)skey, n, ks,
              nbc, blk, f->level[2].idx, f->level[3].idx, flags);
  lower_bound_ptr(env, blk, n, nbr * nbc, f->level[2].ptr);
  Flags h{};
  if (!read_flags(env, flags, &h)) { free_formatted(env, f); return env.status; }
  if (flag_status(h) != US_OK) { free_formatted(env, f); return flag_status(h); }
  *out = f;
  return US_OK;
}

}  // namespace us
