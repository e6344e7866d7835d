// Schedule ("tile table") construction on the device.
//
// From the int32 seq_offsets of a jagged batch (paper, section 2.2) this kernel lists every
// owner tile of every sequence together with the streamed segments it has to be computed
// against, and orders the list by non-increasing cost so that the hardware dispatcher, which
// hands out workgroups in index order, sees the heavy tiles first (longest-processing-time
// order; the cost of a causal tile grows with its position in the sequence).  Tiles that lie
// wholly above the diagonal never appear.  For a context-parallel rank (section 2.3) each
// side of a sequence consists of the two mini-chunks the rank owns.
//
// Nothing here needs the host to know the offsets: the grid of the attention kernels is
// sized from an upper bound on the item count and surplus workgroups exit at once, so no
// device-to-host copy or synchronisation is involved (section 3 measures what such
// synchronisations cost).
#include "hstu_common.h"

namespace hstu {

namespace {

constexpr int PLAN_THREADS = 1024;
constexpr int NBINS = 2048;

// The (up to two) segments one side of one sequence consists of.
struct Side {
  int nseg;
  int len[2];
  int pos[2];
  int rows;  // len[0] + len[1]
};

__device__ inline Side make_side(int L, int cp, int rank) {
  Side s;
  if (rank < 0) {
    s.nseg = 1; s.len[0] = L; s.pos[0] = 0; s.len[1] = 0; s.pos[1] = 0;
  } else {
    // mini-chunk m covers positions [m*c, min((m+1)*c, L)), c = ceil(L / (2*cp))
    const long long c = ((long long)L + 2 * cp - 1) / (2 * cp);
    const int m0 = rank, m1 = 2 * cp - 1 - rank;
    long long b0 = m0 * c, e0 = (m0 + 1) * c, b1 = m1 * c, e1 = (m1 + 1) * c;
    b0 = b0 < L ? b0 : L; e0 = e0 < L ? e0 : L; b1 = b1 < L ? b1 : L; e1 = e1 < L ? e1 : L;
    s.nseg = 2;
    s.len[0] = (int)(e0 - b0); s.pos[0] = (int)b0;
    s.len[1] = (int)(e1 - b1); s.pos[1] = (int)b1;
    if (s.len[1] > 0 && s.pos[1] == s.pos[0] + s.len[0]) {  // adjacent chunks: one segment
      s.len[0] += s.len[1]; s.len[1] = 0; s.nseg = 1;
    }
    if (s.len[1] == 0) s.nseg = 1;
  }
  s.rows = s.len[0] + s.len[1];
  return s;
}

__device__ inline int clampi(long long x, int lo, int hi) {
  return x < lo ? lo : (x > hi ? hi : (int)x);
}

// Sanitised [start, end) of sequence b in the global layout: whatever the device array
// holds, 0 <= start <= end <= total_rows.
__device__ inline void seq_range(const int32_t* off, int b, int total_rows, int& s, int& e) {
  s = clampi(off[b], 0, total_rows);
  e = clampi(off[b + 1], s, total_rows);
}

constexpr int STILE = 64;  // rows per tile of the streamed side (what the kernels stage in LDS)

__device__ inline int tiles_of(const Side& s, int tile) {
  return (s.len[0] + tile - 1) / tile + (s.len[1] + tile - 1) / tile;
}

// Inclusive scan of one value per thread across the block; returns the inclusive prefix and
// leaves the block total in *total.  `buf` has at least PLAN_THREADS / 64 ints.  Shuffles
// inside each wavefront, then one pass over the wavefront totals.
__device__ inline int block_scan(int v, int* buf, int* total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int x = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int y = __shfl_up(x, d, 64);
    if (lane >= d) x += y;
  }
  if (lane == 63) buf[wave] = x;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < PLAN_THREADS / 64; ++w) {
    const int t = buf[w];
    if (w < wave) base += t;
    tot += t;
  }
  *total = tot;
  __syncthreads();
  return x + base;
}

// atomicAdd(&hist[bin], 1) for every active lane, returning the old value, with the lanes of a
// wave that hit the same bin combined into one atomic (batches of short sequences put thousands
// of items into a handful of bins, and same-address LDS atomics serialise).  Up to four distinct
// bins per wave are combined, the rest fall back to one atomic per lane.  Must be called by all
// lanes of the wave.
__device__ inline int combined_atomic_inc(int* hist, int bin, bool active) {
  const int lane = threadIdx.x & 63;
  int pos = -1;
  for (int round = 0; round < 4; ++round) {
    const unsigned long long todo = __ballot(active && pos < 0);
    if (todo == 0) break;
    const int leader = __ffsll((long long)todo) - 1;
    const int lb = __shfl(bin, leader, 64);
    const bool mine = active && pos < 0 && bin == lb;
    const unsigned long long same = __ballot(mine);
    int base = 0;
    if (lane == leader) base = atomicAdd(&hist[lb], __popcll(same));
    base = __shfl(base, leader, 64);
    if (mine) pos = base + __popcll(same & ((1ull << lane) - 1ull));
  }
  if (active && pos < 0) pos = atomicAdd(&hist[bin], 1);
  return pos;
}

// Per-sequence arrays are kept in LDS when the batch fits (the common case) so that the binary
// searches and base lookups of the later passes do not pay global-memory latency.
constexpr int LDS_BATCH = 6143;

__device__ __forceinline__ void plan_body(const PlanArgs& a);

__global__ void __launch_bounds__(PLAN_THREADS) plan_kernel(PlanArgs a0, PlanArgs a1, PlanArgs a2) {
  plan_body(blockIdx.x == 0 ? a0 : (blockIdx.x == 1 ? a1 : a2));
}

__device__ __forceinline__ void plan_body(const PlanArgs& a) {
  __shared__ int scan_buf[PLAN_THREADS / 64];
  __shared__ int s_off[LDS_BATCH + 2], s_owner[LDS_BATCH + 1], s_streamed[LDS_BATCH + 1];
  __shared__ int s_tile[LDS_BATCH + 2], s_stile[LDS_BATCH + 2];
  const bool in_lds = a.batch <= LDS_BATCH;
  // the arrays the later passes read: LDS copies when they fit, the workspace otherwise
  const int* r_off = in_lds ? s_off : a.off;
  const int* r_owner = in_lds ? s_owner : a.owner_base;
  const int* r_streamed = in_lds ? s_streamed : a.streamed_base;
  const int* r_tile = in_lds ? s_tile : a.tile_base;
  const int* r_stile = in_lds ? s_stile : a.stile_base;
  __shared__ int hist[NBINS];
  __shared__ int num_items_s;
  __shared__ int num_stiles_s;
  const int tid = threadIdx.x;

  // ---- pass 1: per-sequence bases (prefix sums over the batch) --------------------------
  int carry_owner = 0, carry_streamed = 0, carry_tiles = 0, carry_stiles = 0;
  for (int b0 = 0; b0 < a.batch; b0 += PLAN_THREADS) {
    const int b = b0 + tid;
    int orows = 0, srows = 0, ntile = 0, nstile = 0, s = 0, e = 0;
    if (b < a.batch) {
      seq_range(a.off, b, a.total_rows, s, e);
      const Side so = make_side(e - s, a.cp, a.owner_rank);
      const Side ss = make_side(e - s, a.cp, a.streamed_rank);
      orows = so.rows; srows = ss.rows; ntile = tiles_of(so, a.tile); nstile = tiles_of(ss, STILE);
    }
    int tot;
    const int io = block_scan(orows, scan_buf, &tot);   const int tot_o = tot;
    const int is = block_scan(srows, scan_buf, &tot);   const int tot_s = tot;
    const int it = block_scan(ntile, scan_buf, &tot);   const int tot_t = tot;
    const int iu = block_scan(nstile, scan_buf, &tot);  const int tot_u = tot;
    if (b < a.batch) {
      // global layouts keep the caller's offsets; local layouts are packed rank rows
      const int ob = a.owner_rank < 0 ? s : carry_owner + io - orows;
      const int sb = a.streamed_rank < 0 ? s : carry_streamed + is - srows;
      const int tb = carry_tiles + it - ntile, ub = carry_stiles + iu - nstile;
      if (in_lds) {
        s_off[b] = a.off[b]; s_owner[b] = ob; s_streamed[b] = sb; s_tile[b] = tb; s_stile[b] = ub;
        if (b == a.batch - 1) s_off[b + 1] = a.off[b + 1];
      } else {
        a.owner_base[b] = ob; a.streamed_base[b] = sb; a.tile_base[b] = tb; a.stile_base[b] = ub;
      }
    }
    carry_owner += tot_o; carry_streamed += tot_s; carry_tiles += tot_t; carry_stiles += tot_u;
  }
  if (tid == 0) {
    if (in_lds) { s_tile[a.batch] = carry_tiles; s_stile[a.batch] = carry_stiles; }
    else { a.tile_base[a.batch] = carry_tiles; a.stile_base[a.batch] = carry_stiles; }
    num_items_s = carry_tiles < a.max_items ? carry_tiles : a.max_items;
    num_stiles_s = carry_stiles < a.max_stiles ? carry_stiles : a.max_stiles;
  }
  for (int i = tid; i < NBINS; i += PLAN_THREADS) hist[i] = 0;
  __syncthreads();
  const int num_items = num_items_s;
  const int num_stiles = num_stiles_s;

  // ---- pass 1b: the 64-row tiles of the streamed side (what the transposed copies are cut into)
  for (int i = tid; a.want_ttile && i < num_stiles; i += PLAN_THREADS) {
    int lo = 0, hi = a.batch;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (r_stile[mid] <= i) lo = mid; else hi = mid;
    }
    const int b = lo;
    int s, e;
    seq_range(r_off, b, a.total_rows, s, e);
    const Side ss = make_side(e - s, a.cp, a.streamed_rank);
    int t = i - r_stile[b];
    const int nt0 = (ss.len[0] + STILE - 1) / STILE;
    const int g = t < nt0 ? 0 : 1;
    if (g) t -= nt0;
    const int row0 = r_streamed[b] + (g ? ss.len[0] : 0) + t * STILE;
    int nrows = ss.len[g] - t * STILE;
    if (nrows > STILE) nrows = STILE;
    nrows = clampi((long long)a.streamed_rows - row0, 0, nrows);
    a.ttile[2 * i] = row0;
    a.ttile[2 * i + 1] = nrows;
  }

  // ---- pass 2: describe every item, histogram its cost -----------------------------------
  int carry_sub = 0, carry_red = 0, carry_slot = 0;  // running totals of parts, split tiles, slots
  for (int i0 = 0; i0 < num_items; i0 += PLAN_THREADS) {
    const int i = i0 + tid;
    const bool active = i < num_items;
    int bin = 0;
    Item it = {};
    int pvis[2] = {0, 0};
    if (active) {
    int lo = 0, hi = a.batch;  // largest b with tile_base[b] <= i
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (r_tile[mid] <= i) lo = mid; else hi = mid;
    }
    const int b = lo;
    int s, e;
    seq_range(r_off, b, a.total_rows, s, e);
    const Side so = make_side(e - s, a.cp, a.owner_rank);
    const Side ss = make_side(e - s, a.cp, a.streamed_rank);
    int t = i - r_tile[b];
    const int nt0 = (so.len[0] + a.tile - 1) / a.tile;
    const int u = t < nt0 ? 0 : 1;
    if (u) t -= nt0;
    it.row0 = r_owner[b] + (u ? so.len[0] : 0) + t * a.tile;
    it.nrows = so.len[u] - t * a.tile;
    if (it.nrows > a.tile) it.nrows = a.tile;
    it.pos0 = so.pos[u] + t * a.tile;
    // never beyond the rows the caller declared for its buffers
    it.nrows = clampi((long long)a.owner_rows - it.row0, 0, it.nrows);
    // The visible streamed segments, compacted to the front.  Written without run-time array
    // indices so that the item stays in registers (indexed, it would live in scratch memory).
    int vrow[2] = {0, 0}, vlen[2] = {0, 0}, vpos[2] = {0, 0}, vcol[2] = {0, 0}, vcost[2] = {0, 0};
    int vvis[2] = {0, 0};
    bool von[2] = {false, false};
    int srow = r_streamed[b];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      if (g < ss.nseg) {
        const int len = clampi((long long)a.streamed_rows - srow, 0, ss.len[g]);
        int vis;  // streamed rows that at least one owner row sees
        if (!a.causal) {
          vis = len;
        } else if (a.side == 0) {  // keys at positions <= last query position
          vis = clampi((long long)it.pos0 + it.nrows - ss.pos[g], 0, len);
        } else {                   // queries at positions >= first key position
          vis = len - clampi((long long)it.pos0 - ss.pos[g], 0, len);
        }
        von[g] = it.nrows > 0 && vis > 0;
        vrow[g] = srow; vlen[g] = len; vpos[g] = ss.pos[g];
        vcol[g] = STILE * (r_stile[b] + (g ? (ss.len[0] + STILE - 1) / STILE : 0));
        vcost[g] = (vis + 31) >> 5;
        vvis[g] = vis;
        srow += ss.len[g];
      }
    }
    const bool first1 = !von[0] && von[1];  // only the second segment is visible: it moves to slot 0
    it.nseg = (von[0] ? 1 : 0) + (von[1] ? 1 : 0);
    it.cost = (von[0] ? vcost[0] : 0) + (von[1] ? vcost[1] : 0);
    it.seg_row0[0] = von[0] ? vrow[0] : (first1 ? vrow[1] : 0);
    it.seg_len[0] = von[0] ? vlen[0] : (first1 ? vlen[1] : 0);
    it.seg_pos0[0] = von[0] ? vpos[0] : (first1 ? vpos[1] : 0);
    it.seg_tcol0[0] = von[0] ? vcol[0] : (first1 ? vcol[1] : 0);
    const bool second = von[0] && von[1];
    it.seg_row0[1] = second ? vrow[1] : 0;
    it.seg_len[1] = second ? vlen[1] : 0;
    it.seg_pos0[1] = second ? vpos[1] : 0;
    it.seg_tcol0[1] = second ? vcol[1] : 0;
    it.part = 0;
    it.pad[0] = it.pad[1] = 0;
    // visible rows of the (compacted) segments, for cutting the tile into parts
    pvis[0] = von[0] ? vvis[0] : (first1 ? vvis[1] : 0);
    pvis[1] = second ? vvis[1] : 0;
    }
    if (a.split_max <= 1 && a.cost_shift >= 30) {  // natural order: nothing to sort
      if (active) { a.items[i] = it; a.order[i] = i; }
      continue;
    }
    if (a.split_max <= 1) {
      if (active) a.items[i] = it;
      bin = it.cost >> a.cost_shift;
      if (bin > NBINS - 1) bin = NBINS - 1;
      combined_atomic_inc(hist, NBINS - 1 - bin, active);  // reversed: heavy items get the low indices
      continue;
    }
    // ---- heavy owner tiles are cut along their streamed rows into ns parts of whole 64-row
    // tiles; each part becomes an item of its own that writes an fp32 partial result
    const int nt0 = (pvis[0] + STILE - 1) / STILE, nt = nt0 + (pvis[1] + STILE - 1) / STILE;
    int ns = active ? it.cost / a.split_blocks : 0;
    if (ns > a.split_max) ns = a.split_max;
    if (ns > nt) ns = nt;
    if (active && ns < 1) ns = 1;
    int tot_n, tot_r, tot_p;
    const int u0 = carry_sub + block_scan(ns, scan_buf, &tot_n) - ns;
    const int isr = ns > 1 ? 1 : 0;
    const int r0 = carry_red + block_scan(isr, scan_buf, &tot_r) - isr;
    const int p0 = carry_slot + block_scan(isr ? ns : 0, scan_buf, &tot_p) - (isr ? ns : 0);
    carry_sub += tot_n; carry_red += tot_r; carry_slot += tot_p;
    if (isr) {
      a.red[4 * r0] = it.row0; a.red[4 * r0 + 1] = it.nrows; a.red[4 * r0 + 2] = p0; a.red[4 * r0 + 3] = ns;
    }
    for (int k = 0; k < a.split_max; ++k) {
      const bool on = k < ns;
      Item sub = it;
      if (on && ns > 1) {
        const int lo = (int)((long long)k * nt / ns), hi = (int)((long long)(k + 1) * nt / ns);
        int srow2[2], slen2[2], spos2[2], scol2[2], scost = 0, n2 = 0;
        bool son[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const int base = c ? nt0 : 0, ntc = c ? nt - nt0 : nt0;
          const int l = clampi(lo - base, 0, ntc), h = clampi(hi - base, 0, ntc);
          son[c] = h > l;
          const int skip = l * STILE;
          int len = it.seg_len[c] - skip;
          if (len > (h - l) * STILE) len = (h - l) * STILE;
          int vis = pvis[c] - skip;
          if (vis > (h - l) * STILE) vis = (h - l) * STILE;
          srow2[c] = it.seg_row0[c] + skip; slen2[c] = len; spos2[c] = it.seg_pos0[c] + skip;
          scol2[c] = it.seg_tcol0[c] + skip;
          if (son[c]) { scost += (vis + 31) >> 5; ++n2; }
        }
        const bool f1 = !son[0] && son[1], both = son[0] && son[1];
        sub.nseg = n2; sub.cost = scost; sub.part = p0 + k + 1;
        sub.seg_row0[0] = son[0] ? srow2[0] : (f1 ? srow2[1] : 0);
        sub.seg_len[0] = son[0] ? slen2[0] : (f1 ? slen2[1] : 0);
        sub.seg_pos0[0] = son[0] ? spos2[0] : (f1 ? spos2[1] : 0);
        sub.seg_tcol0[0] = son[0] ? scol2[0] : (f1 ? scol2[1] : 0);
        sub.seg_row0[1] = both ? srow2[1] : 0;
        sub.seg_len[1] = both ? slen2[1] : 0;
        sub.seg_pos0[1] = both ? spos2[1] : 0;
        sub.seg_tcol0[1] = both ? scol2[1] : 0;
      }
      const bool emit = on && u0 + k < a.max_items;
      if (emit) a.items[u0 + k] = sub;
      bin = sub.cost >> a.cost_shift;
      if (bin > NBINS - 1) bin = NBINS - 1;
      combined_atomic_inc(hist, NBINS - 1 - bin, emit);
    }
  }
  // items the kernels will see (the scans' totals are the same in every thread)
  const int items_final = a.split_max > 1 ? (carry_sub < a.max_items ? carry_sub : a.max_items) : num_items;
  __syncthreads();

  const bool sorted = !(a.split_max <= 1 && a.cost_shift >= 30);
  // ---- pass 3: bin start positions (exclusive scan over the reversed histogram) ----------
  if (sorted) {
    const int h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
    int tot;
    const int inc = block_scan(h0 + h1, scan_buf, &tot);
    hist[2 * tid] = inc - h0 - h1;
    hist[2 * tid + 1] = inc - h1;
  }
  __syncthreads();

  // ---- pass 4: scatter item indices into schedule order ----------------------------------
  for (int i0 = 0; sorted && i0 < items_final; i0 += PLAN_THREADS) {
    const int i = i0 + tid;
    const bool active = i < items_final;
    int bin = active ? a.items[i].cost >> a.cost_shift : 0;
    if (bin > NBINS - 1) bin = NBINS - 1;
    const int pos = combined_atomic_inc(hist, NBINS - 1 - bin, active);
    if (active) a.order[pos] = i;
  }
  if (tid == 0) {
    a.header[0] = items_final;
    a.header[1] = num_stiles;
    a.header[2] = a.split_max > 1 ? carry_red : 0;
  }
}

}  // namespace

namespace {

constexpr int REORDER_THREADS = 256;

// Load-balance reorder (section 2.3).  One workgroup per (64-row tile of the rank's local layout,
// tensor).  The workgroup finds its tile from the offsets by itself: every thread sums the tile
// and row counts of a contiguous share of the sequences, a scan over the 256 partial sums tells
// which thread's share holds tile blockIdx.x, and that thread walks its share to the sequence.
// No table is built beforehand, so the call is this one launch and needs no workspace.  Inside
// a tile the rows are consecutive in both layouts: the tile is one contiguous span on either
// side and the copy runs at full memory width, 16 bytes per lane, four loads in flight.
__global__ void __launch_bounds__(REORDER_THREADS) reorder_kernel(ReorderArgs a) {
  __shared__ int wave_tiles[REORDER_THREADS / 64], wave_rows[REORDER_THREADS / 64];
  __shared__ int found[3];  // first local row, rows, first global row of this workgroup's tile
  const int i = blockIdx.x / a.split, part = blockIdx.x % a.split;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) found[1] = 0;
  const int per = (a.batch + REORDER_THREADS - 1) / REORDER_THREADS;
  const int b_lo = tid * per < a.batch ? tid * per : a.batch;
  const int b_hi = b_lo + per < a.batch ? b_lo + per : a.batch;
  int tiles = 0, rows = 0;
  for (int b = b_lo; b < b_hi; ++b) {
    int s, e;
    seq_range(a.off, b, a.total_rows, s, e);
    const Side sd = make_side(e - s, a.cp, a.rank);
    tiles += tiles_of(sd, STILE);
    rows += sd.rows;
  }
  int xt = tiles, xr = rows;  // inclusive prefixes across the block
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int yt = __shfl_up(xt, d, 64), yr = __shfl_up(xr, d, 64);
    if (lane >= d) { xt += yt; xr += yr; }
  }
  if (lane == 63) { wave_tiles[wave] = xt; wave_rows[wave] = xr; }
  __syncthreads();
  for (int w = 0; w < wave; ++w) { xt += wave_tiles[w]; xr += wave_rows[w]; }
  int tile0 = xt - tiles, row0 = xr - rows;  // first tile and first local row of this thread's share
  if (i >= tile0 && i < xt) {
    for (int b = b_lo; b < b_hi; ++b) {
      int s, e;
      seq_range(a.off, b, a.total_rows, s, e);
      const Side sd = make_side(e - s, a.cp, a.rank);
      const int nt = tiles_of(sd, STILE);
      if (i < tile0 + nt) {
        int t = i - tile0;
        const int nt0 = (sd.len[0] + STILE - 1) / STILE;
        const int g = t < nt0 ? 0 : 1;
        if (g) t -= nt0;
        const int local = row0 + (g ? sd.len[0] : 0) + t * STILE;
        int n = sd.len[g] - t * STILE;
        if (n > STILE) n = STILE;
        found[0] = local;
        found[1] = clampi((long long)a.local_rows - local, 0, n);
        found[2] = s + sd.pos[g] + t * STILE;
        break;
      }
      tile0 += nt; row0 += sd.rows;
    }
  }
  __syncthreads();
  // this workgroup's share of the tile: rows [part, part + 1) * STILE / split of it
  const int sub = STILE / a.split, first = part * sub;
  const int64_t nrows = found[1] - first < sub ? found[1] - first : sub;
  if (nrows <= 0) return;  // beyond the last tile, or beyond the declared local rows
  const int64_t local_row = found[0] + first, global_row = found[2] + first;
  const int64_t rb = a.row_bytes[blockIdx.y];
  const char* src = a.src[blockIdx.y] + (a.scatter ? local_row : global_row) * rb;
  char* dst = a.dst[blockIdx.y] + (a.scatter ? global_row : local_row) * rb;
  constexpr int N = REORDER_THREADS;
  if (rb % 16 != 0) {  // narrow rows (a multiple of 4 bytes, e.g. one timestamp per row): word copies
    const int64_t words = nrows * rb / 4;
    for (int64_t c = tid; c < words; c += N) ((uint32_t*)dst)[c] = ((const uint32_t*)src)[c];
    return;
  }
  const int64_t chunks = nrows * rb / 16;
  typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
  // plain loads and stores: non-temporal ones gain 5 % on copies larger than the last-level
  // cache and lose 15 % on the smaller ones that the batches here produce
  constexpr int U = 4;
  int64_t c = tid;
  for (; c + (U - 1) * N < chunks; c += U * N) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = *(const u32x4*)(src + (c + u * N) * 16);
#pragma unroll
    for (int u = 0; u < U; ++u) *(u32x4*)(dst + (c + u * N) * 16) = v[u];
  }
  for (; c < chunks; c += N) *(u32x4*)(dst + c * 16) = *(const u32x4*)(src + c * 16);
}

}  // namespace

hipError_t launch_reorder(const ReorderArgs& a, int64_t max_tiles, hipStream_t stream) {
  if (a.count < 1 || a.count > 4 || max_tiles < 1 || max_tiles >= (1ll << 31)) return hipErrorInvalidValue;
  if (a.split < 1 || STILE % a.split != 0 || max_tiles * a.split >= (1ll << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(reorder_kernel, dim3((unsigned)(max_tiles * a.split), (unsigned)a.count),
                     dim3(REORDER_THREADS), 0, stream, a);
  return hipGetLastError();
}

namespace {

// Sum of the partial results of one split owner tile and head, in slot order.
__global__ void __launch_bounds__(256) reduce_partials_kernel(Plan plan, const float* partial, void* out,
                                                              int H, int d, int tile_rows,
                                                              int accumulate, int out_f32) {
  const int r = blockIdx.x / H, h = blockIdx.x % H;
  if (r >= plan.header[2]) return;
  const int row0 = plan.red[4 * r], nrows = plan.red[4 * r + 1], slot0 = plan.red[4 * r + 2],
            ns = plan.red[4 * r + 3];
  const int64_t slot_stride = (int64_t)H * tile_rows * d;
  const float* src = partial + ((int64_t)slot0 * H + h) * tile_rows * d;
  const int n4 = nrows * d / 4;
  for (int i = threadIdx.x; i < n4; i += 256) {
    float4 acc = *(const float4*)(src + (int64_t)i * 4);
    for (int k = 1; k < ns; ++k) {
      const float4 v = *(const float4*)(src + k * slot_stride + (int64_t)i * 4);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const int row = (i * 4) / d, col = (i * 4) % d;
    const int64_t e = ((int64_t)(row0 + row) * H + h) * d + col;
    if (out_f32) {
      float4* o = (float4*)((float*)out + e);
      if (accumulate) { const float4 p = *o; acc.x += p.x; acc.y += p.y; acc.z += p.z; acc.w += p.w; }
      *o = acc;
    } else {
      __bf16* o = (__bf16*)out + e;
      float x[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (accumulate) x[c] += (float)o[c];
        o[c] = (__bf16)x[c];
      }
    }
  }
}

}  // namespace

hipError_t launch_reduce_partials(const Plan& plan, int64_t max_tiles, const float* partial, void* out,
                                  int num_heads, int d, int tile_rows, int accumulate, int out_f32,
                                  hipStream_t stream) {
  if (max_tiles < 1 || max_tiles * num_heads >= (1ll << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)(max_tiles * num_heads)), dim3(256), 0,
                     stream, plan, partial, out, num_heads, d, tile_rows, accumulate, out_f32);
  return hipGetLastError();
}

namespace {

// Timestamp records (see TsRecord): one thread per row.  The sequence of a row is found by
// bisection of the offsets; rows outside every sequence (offsets that do not end at the row
// count) get a range of their own timestamp only.  Without offsets a row's range covers the
// next 32 rows of the array.
__global__ void __launch_bounds__(256) ts_records_kernel(const int32_t* __restrict__ ts,
                                                         const int32_t* __restrict__ off, int batch,
                                                         int total, TsRecord* __restrict__ rec,
                                                         double* __restrict__ acc, int nb) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (acc)
    for (int i = r; i < nb; i += gridDim.x * 256) acc[i] = 0.0;
  if (r >= total + 64) return;
  TsRecord x = {0, 0, 0, 0};
  if (r < total) {
    int end = total;
    if (off) {
      int lo = 0, hi = batch;  // off[lo] <= r < off[hi] when the offsets are well-formed
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= r) lo = mid; else hi = mid;
      }
      end = off[hi];
      end = end < total ? end : total;
    }
    const int last = r + 32 < end ? r + 32 : end;
    x.ts = x.lo = x.hi = ts[r];
    for (int i = r + 1; i < last; ++i) {
      const int t = ts[i];
      x.lo = t < x.lo ? t : x.lo;
      x.hi = t > x.hi ? t : x.hi;
    }
  }
  rec[r] = x;
}

}  // namespace

namespace {

__global__ void __launch_bounds__(256) dw_finish_kernel(const double* __restrict__ acc,
                                                        float* __restrict__ d_w, int nb, double scale,
                                                        int accumulate) {
  for (int i = threadIdx.x; i < nb; i += 256) {
    const float x = (float)(acc[i] * scale);
    d_w[i] = accumulate ? d_w[i] + x : x;
  }
}

}  // namespace

hipError_t launch_dw_finish(const double* acc, float* d_w, int nb, double scale, int accumulate,
                            hipStream_t stream) {
  if (!acc || !d_w || nb < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(dw_finish_kernel, dim3(1), dim3(256), 0, stream, acc, d_w, nb, scale, accumulate);
  return hipGetLastError();
}

hipError_t launch_ts_records(const int32_t* ts, const int32_t* off, int batch, int64_t total_rows,
                             TsRecord* rec, double* acc, int nb, hipStream_t stream) {
  if ((off && batch < 1) || total_rows < 0 || total_rows + 64 >= (1ll << 31)) return hipErrorInvalidValue;
  const unsigned blocks = (unsigned)((total_rows + 64 + 255) / 256);
  hipLaunchKernelGGL(ts_records_kernel, dim3(blocks), dim3(256), 0, stream, ts, off, batch,
                     (int)total_rows, rec, acc, nb);
  return hipGetLastError();
}

namespace {

// Packed tiles (see PackedPlanArgs): one thread per row.  The sequence of a row is found by
// bisection of the offsets; whatever the offsets hold, a row's bounds contain the row and stay
// inside [0, total_rows], and items cover rows below min(off[batch], total_rows) only.
__global__ void __launch_bounds__(256) packed_plan_kernel(PackedPlanArgs a) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  const int T = a.total_rows;
  int teff = a.off[a.batch];
  teff = teff < 0 ? 0 : (teff < T ? teff : T);
  if (r == 0) {
    const int ntiles = (teff + a.tile - 1) / a.tile;
    for (int side = 0; side < 2; ++side) {
      a.header[side][0] = ntiles;
      a.header[side][1] = 0;
      a.header[side][2] = 0;
    }
  }
  if (r >= T) return;
  auto seq_of = [&](int row) {
    int lo = 0, hi = a.batch;  // off[lo] <= row < off[hi] when the offsets are well-formed
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (a.off[mid] <= row) lo = mid; else hi = mid;
    }
    return lo;
  };
  auto clamp_end = [&](int e, int at_least) { e = e < T ? e : T; return e > at_least ? e : at_least; };
  const int b = seq_of(r);
  int s0 = a.off[b];
  s0 = s0 < 0 ? 0 : (s0 < r ? s0 : r);
  a.row_seq[r] = make_int2(s0, clamp_end(a.off[b + 1], r + 1));
  if (r % a.tile != 0 || r >= teff) return;
  const int t = r / a.tile;
  const int r1 = r + a.tile < teff ? r + a.tile : teff;
  const int e1 = clamp_end(a.off[seq_of(r1 - 1) + 1], r1);  // end of the last sequence of the tile
  Item it = {};
  it.row0 = r;
  it.nrows = r1 - r;
  it.pos0 = r;
  it.nseg = 1;
  // owners are queries: keys from the start of the first sequence to the tile's end (causal) or
  // to the end of the last sequence
  it.seg_row0[0] = s0;
  it.seg_pos0[0] = s0;
  it.seg_len[0] = (a.causal ? r1 : e1) - s0;
  a.items[0][t] = it;
  a.order[0][t] = t;
  // owners are keys: queries from the tile's start (causal) or the start of the first sequence
  // to the end of the last sequence
  const int q0 = a.causal ? r : s0;
  it.seg_row0[0] = q0;
  it.seg_pos0[0] = q0;
  it.seg_len[0] = e1 - q0;
  a.items[1][t] = it;
  a.order[1][t] = t;
}

}  // namespace

hipError_t launch_packed_plan(const PackedPlanArgs& a, hipStream_t stream) {
  if (a.batch < 1 || a.total_rows < 1 || a.tile < 64 || a.tile % 64 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(packed_plan_kernel, dim3((unsigned)((a.total_rows + 255) / 256)), dim3(256), 0,
                     stream, a);
  return hipGetLastError();
}

hipError_t launch_plans(const PlanArgs* a, int count, hipStream_t stream) {
  static_assert(NBINS == 2 * PLAN_THREADS, "pass 3 handles two bins per thread");
  if (count < 1 || count > 3) return hipErrorInvalidValue;
  hipLaunchKernelGGL(plan_kernel, dim3(count), dim3(PLAN_THREADS), 0, stream, a[0],
                     a[count > 1 ? 1 : 0], a[count - 1]);
  return hipGetLastError();
}

}  // namespace hstu
