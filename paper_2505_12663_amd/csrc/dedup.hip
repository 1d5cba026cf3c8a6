// ID tagging (Eq. 8) and stage-1 deduplication (Sec. 3.3) for gfx950.
//
// Dedup = stable LSD radix sort of (key, position) pairs, 8 bits per pass, followed by a
// head-flag scan.  Digits in which all keys agree are found on the device (OR/AND reduction of
// the keys) and their passes skipped: tagged keys carry a few identifier bits at the top and a
// 40..48-bit ID at the bottom, so 2-3 of the 8 passes vanish.  Each pass is three kernels
// (per-tile histogram, per-digit scan over tiles, scatter) - no kernel waits on another block.
// The scatter ranks a tile's keys with wave-wide ballots (no LDS atomics), reorders the tile in
// LDS and writes runs of equal digit contiguously.
#include <mutex>

#include "common.hpp"

using namespace mtgr;

namespace {

constexpr int kThreads = 256;
constexpr int kItems = 16;                    // keys per thread
constexpr int kTile = kThreads * kItems;      // 4096 keys per block
constexpr int kWaves = kThreads / kWave;      // 4
constexpr int kRadix = 256;
constexpr int kPasses = 8;
constexpr int kScThreads = 512;               // scatter kernel: same tile, more and lighter threads
constexpr int kScItems = kTile / kScThreads;
constexpr int kScWaves = kScThreads / kWave;

struct DdHeader {
    unsigned long long or_mask, and_mask;
    int active[kPasses];
    int src[kPasses];   // 0 = caller's keys (implicit position), 1 = buffer A, 2 = buffer B
    int dst[kPasses];
    int final_sel;
    int pad;
    long long n_unique;
};

struct DdBuffers {
    const uint64_t* in_keys;
    uint64_t* ka;
    uint64_t* kb;
    uint32_t* ia;
    uint32_t* ib;
};

__device__ inline const uint64_t* sel_keys(const DdBuffers& b, int s) { return s == 0 ? b.in_keys : (s == 1 ? b.ka : b.kb); }
__device__ inline const uint32_t* sel_idx(const DdBuffers& b, int s) { return s == 1 ? b.ia : (s == 2 ? b.ib : nullptr); }

// ---------------------------------------------------------------------------- tagging
// last field whose start is <= e (s_off[0] <= e < s_off[n_fields])
__device__ inline int field_of(const int64_t* s_off, int n_fields, int64_t e) {
    int lo = 0, hi = n_fields;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_off[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

// A wave tags 256 consecutive IDs per round (4 coalesced loads).  Almost every such range lies
// inside one field, so two searches per wave (first and last element) replace one per element.
__global__ __launch_bounds__(kThreads) void k_tag(const uint64_t* __restrict__ x, const int64_t* __restrict__ field_off,
                                                 const uint8_t* __restrict__ field_tag, int n_fields, int64_t n,
                                                 int shift, int id_bits, uint64_t* __restrict__ key_out,
                                                 unsigned long long* err_count) {
    extern __shared__ int64_t s_off[]; // n_fields + 1 offsets
    for (int f = threadIdx.x; f <= n_fields; f += kThreads) s_off[f] = field_off[f];
    __syncthreads();
    constexpr int kPer = 4;
    const uint64_t low_mask = (1ull << (id_bits < shift ? id_bits : shift)) - 1ull;   // IDs beyond it are counted and wrapped
    const int lane = lane_id();
    const int64_t wave_stride = (int64_t)gridDim.x * kWaves * (kWave * kPer);
    unsigned errs = 0;
    for (int64_t base = ((int64_t)blockIdx.x * kWaves + threadIdx.x / kWave) * (kWave * kPer); base < n; base += wave_stride) {
        const int64_t last = base + kWave * kPer - 1 < n ? base + kWave * kPer - 1 : n - 1;
        int f_edge = 0;
        if (lane == 0) f_edge = field_of(s_off, n_fields, base);
        if (lane == kWave - 1) f_edge = field_of(s_off, n_fields, last);
        const int f_first = __shfl(f_edge, 0, kWave), f_last = __shfl(f_edge, kWave - 1, kWave);
        uint64_t v[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int64_t e = base + u * kWave + lane;
            v[u] = x[e < n ? e : n - 1];      // no load behind a branch: see k_dd_masks
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int64_t e = base + u * kWave + lane;
            if (e >= n) continue;
            const int f = (f_first == f_last) ? f_first : field_of(s_off, n_fields, e);
            uint64_t val = v[u];
            if (val > low_mask) {
                ++errs;
                val &= low_mask;
            }
            key_out[e] = ((uint64_t)field_tag[f] << shift) | val;
        }
    }
    for (int o = 32; o > 0; o >>= 1) errs += __shfl_xor(errs, o, kWave);
    if (errs && lane == 0) atomicAdd(err_count, (unsigned long long)errs);
}

__global__ void k_zero64(unsigned long long* p) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0ull;
}

// Tile handled by a block: workgroups are handed to the 8 XCDs (each with its own L2) in turn; giving every XCD
// a contiguous range of tiles lets its L2 merge the partial-sector accesses that neighbouring tiles make to the
// rows of tile_hist and to the ends of their digit runs in the scatter's output.  The grid is
// 8 * ceil(n_tiles / 8) blocks; a block whose tile does not exist leaves at once.
constexpr unsigned kXcds = 8;
__device__ inline unsigned tile_of_block(unsigned n_tiles) {
    const unsigned per = (n_tiles + kXcds - 1) / kXcds;
    return (blockIdx.x % kXcds) * per + blockIdx.x / kXcds;
}
inline unsigned xcd_grid(unsigned n_tiles) { return kXcds * ((n_tiles + kXcds - 1) / kXcds); }

// ---------------------------------------------------------------------------- which digits vary
__device__ inline unsigned digit_of(uint64_t k, int pass) { return (unsigned)(k >> (8 * pass)) & 0xFFu; }

// Add a wave's 64 digits to an LDS histogram.  From the second pass on equal keys sit next to
// each other, and a popular key fills whole tiles: 64 lanes adding to one counter would be served
// one after the other.  Neighbouring lanes with the same digit are therefore counted as one run
// and added once, by the run's first lane.  d >= kRadix means "no key".
__device__ inline void hist_add_runs(unsigned* s_hist, unsigned d, int lane) {
    const unsigned prev = __shfl_up(d, 1, kWave);
    const bool head = lane == 0 || d != prev;
    const uint64_t heads = __ballot(head);
    if (head && d < (unsigned)kRadix) {
        const uint64_t rest = (heads >> lane) >> 1;
        const unsigned len = rest ? (unsigned)__ffsll((unsigned long long)rest) : (unsigned)(kWave - lane);
        atomicAdd(&s_hist[d], len);
    }
}

// One block per tile: OR / AND of the tile's keys -> partial[2*tile], partial[2*tile+1] (no atomics),
// and, since the keys are in registers anyway, the tile's histogram of the lowest digit in the
// layout the first radix pass expects (that pass then needs no histogram kernel of its own).
__global__ __launch_bounds__(kThreads) void k_dd_masks(const uint64_t* __restrict__ key, int64_t n, unsigned n_tiles,
                                                      unsigned long long* __restrict__ partial,
                                                      unsigned* __restrict__ tile_hist) {
    __shared__ unsigned long long s_o[kWaves], s_a[kWaves];
    __shared__ unsigned s_hist[kRadix];
    const unsigned tile = tile_of_block(n_tiles);
    if (tile >= n_tiles) return;
    s_hist[threadIdx.x] = 0u;
    __syncthreads();
    const int lane = lane_id();
    uint64_t o = 0ull, a = ~0ull;
    const int64_t base = (int64_t)tile * kTile + (threadIdx.x / kWave) * (kWave * kItems) + lane;
    unsigned d[kItems];
    // The loads of a thread go out together, none behind a branch (an element past the end reads the last key
    // instead): a load inside a conditional makes the compiler wait for it on the spot, one round trip per item.
    uint64_t kv[kItems];
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t e = base + it * kWave;
        kv[it] = key[e < n ? e : n - 1];
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t e = base + it * kWave;
        d[it] = kRadix;
        if (e < n) {
            o |= kv[it];
            a &= kv[it];
            d[it] = digit_of(kv[it], 0);
        }
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) hist_add_runs(s_hist, d[it], lane);
    for (int s = 32; s > 0; s >>= 1) {
        o |= shfl64(o, lane ^ s);
        a &= shfl64(a, lane ^ s);
    }
    if (lane == 0) {
        s_o[threadIdx.x / kWave] = o;
        s_a[threadIdx.x / kWave] = a;
    }
    __syncthreads();
    tile_hist[(size_t)threadIdx.x * n_tiles + tile] = s_hist[threadIdx.x];
    if (threadIdx.x == 0) {
        for (int w = 1; w < kWaves; ++w) {
            o |= s_o[w];
            a &= s_a[w];
        }
        partial[2 * tile] = o;
        partial[2 * tile + 1] = a;
    }
}

// one block: combine the partial masks, then lay out the passes
__global__ __launch_bounds__(kThreads) void k_dd_plan(DdHeader* h, const unsigned long long* __restrict__ partial,
                                                     int n_partial) {
    __shared__ unsigned long long s_o[kWaves], s_a[kWaves];
    uint64_t o = 0ull, a = ~0ull;
    for (int i = threadIdx.x; i < n_partial; i += kThreads) {
        o |= partial[2 * i];
        a &= partial[2 * i + 1];
    }
    for (int s = 32; s > 0; s >>= 1) {
        o |= shfl64(o, lane_id() ^ s);
        a &= shfl64(a, lane_id() ^ s);
    }
    if (lane_id() == 0) {
        s_o[threadIdx.x / kWave] = o;
        s_a[threadIdx.x / kWave] = a;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    for (int w = 1; w < kWaves; ++w) {
        o |= s_o[w];
        a &= s_a[w];
    }
    h->or_mask = o;
    h->and_mask = a;
    h->n_unique = 0;
    const unsigned long long varying = o ^ a;
    int cur = 0;
    for (int p = 0; p < kPasses; ++p) {
        const bool act = ((varying >> (8 * p)) & 0xFFull) != 0ull;
        h->active[p] = act;
        h->src[p] = cur;
        const int d = (cur == 1) ? 2 : 1;
        h->dst[p] = d;
        if (act) cur = d;
    }
    h->final_sel = cur;
}

// ---------------------------------------------------------------------------- radix pass

// tile element e = wave*1024 + item*64 + lane
__global__ __launch_bounds__(kThreads) void k_rs_hist(DdBuffers b, const DdHeader* __restrict__ h, int pass, int64_t n,
                                                     unsigned n_tiles, unsigned* __restrict__ tile_hist) {
    if (!h->active[pass]) return;
    __shared__ unsigned s_hist[kRadix];
    const unsigned tile = tile_of_block(n_tiles);
    if (tile >= n_tiles) return;
    s_hist[threadIdx.x] = 0u;
    __syncthreads();
    const uint64_t* keys = sel_keys(b, h->src[pass]);
    const int64_t base = (int64_t)tile * kTile + (threadIdx.x / kWave) * (kWave * kItems) + (threadIdx.x % kWave);
    const int lane = lane_id();
    unsigned d[kItems];
    uint64_t kv[kItems];
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t e = base + it * kWave;
        kv[it] = keys[e < n ? e : n - 1];     // all loads first, unconditional: see k_dd_masks
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t e = base + it * kWave;
        d[it] = e < n ? digit_of(kv[it], pass) : kRadix; // kRadix = no key
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) hist_add_runs(s_hist, d[it], lane);
    __syncthreads();
    tile_hist[(size_t)threadIdx.x * n_tiles + tile] = s_hist[threadIdx.x];
}

// block d: exclusive scan of digit d's counts over the tiles; total -> digit_total[d].
// Every thread owns a run of consecutive tiles, so the block-wide scan happens once.
__global__ __launch_bounds__(kThreads) void k_rs_scan(const DdHeader* __restrict__ h, int pass, unsigned n_tiles,
                                                     unsigned* __restrict__ tile_hist,
                                                     unsigned* __restrict__ digit_total) {
    if (!h->active[pass]) return;
    __shared__ unsigned s_wave[kWaves];
    unsigned* row = tile_hist + (size_t)blockIdx.x * n_tiles;
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const unsigned per = (n_tiles + kThreads - 1) / kThreads;
    const unsigned lo = threadIdx.x * per;
    const unsigned hi = lo + per < n_tiles ? lo + per : n_tiles;
    unsigned sum = 0;
    for (unsigned i = lo; i < hi; ++i) sum += row[i];
    unsigned incl = sum;
    for (int o = 1; o < kWave; o <<= 1) {
        unsigned t = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += t;
    }
    if (lane == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    unsigned run = incl - sum;
    for (int w = 0; w < wave; ++w) run += s_wave[w];
    for (unsigned i = lo; i < hi; ++i) {
        const unsigned v = row[i];
        row[i] = run;
        run += v;
    }
    if (threadIdx.x == kThreads - 1) digit_total[blockIdx.x] = run;
}

// tile element e = wave*(64*kScItems) + item*64 + lane
__global__ __launch_bounds__(kScThreads) void k_rs_scatter(DdBuffers b, const DdHeader* __restrict__ h, int pass,
                                                        int64_t n, unsigned n_tiles,
                                                        const unsigned* __restrict__ tile_hist,
                                                        const unsigned* __restrict__ digit_total) {
    if (!h->active[pass]) return;
    // LDS: the reordered tile (48 KB) and, before it is filled, the counters in the same memory;
    // only the per-digit output offsets live apart.  49 KB per block lets three blocks share a CU.
    __shared__ __attribute__((aligned(16))) unsigned char s_raw[kTile * 12];
    __shared__ unsigned s_delta[kRadix];         // global position - tile position for digit d (mod 2^32)
    uint64_t* s_key = reinterpret_cast<uint64_t*>(s_raw);
    uint32_t* s_idx = reinterpret_cast<uint32_t*>(s_raw + (size_t)kTile * 8);
    unsigned (*s_cnt)[kRadix] = reinterpret_cast<unsigned (*)[kRadix]>(s_raw);            // [kScWaves][kRadix]
    unsigned* s_start = reinterpret_cast<unsigned*>(s_raw) + kScWaves * kRadix;             // [kRadix]
    unsigned* s_wt = s_start + kRadix;                                                    // [kWaves]
    unsigned* s_wg = s_wt + kScWaves;                                                       // [kWaves]

    const int src = h->src[pass], dst = h->dst[pass];
    const uint64_t* in_k = sel_keys(b, src);
    const uint32_t* in_i = sel_idx(b, src);
    uint64_t* out_k = dst == 1 ? b.ka : b.kb;
    uint32_t* out_i = dst == 1 ? b.ia : b.ib;

    const unsigned tile = tile_of_block(n_tiles);
    if (tile >= n_tiles) return;
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int64_t tile_base = (int64_t)tile * kTile;
    const int tile_n = (int)((n - tile_base) < kTile ? (n - tile_base) : kTile);
    for (int i = threadIdx.x; i < kScWaves * kRadix; i += kScThreads) s_cnt[0][i] = 0u;
    __syncthreads();

    uint64_t key[kScItems];
    uint32_t idx[kScItems];
    unsigned rnk[kScItems];
    const int e0 = wave * (kWave * kScItems) + lane;
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        const int e = e0 + it * kWave;
        const int ec = e < tile_n ? e : tile_n - 1;     // all loads first, unconditional: see k_dd_masks
        key[it] = in_k[tile_base + ec];
        idx[it] = in_i ? in_i[tile_base + ec] : (uint32_t)(tile_base + e);
    }
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        const bool ok = e0 + it * kWave < tile_n;
        key[it] = ok ? key[it] : ~0ull;
        idx[it] = ok ? idx[it] : 0xFFFFFFFFu;
    }
    // rank of every key among the keys of equal digit that precede it in this wave's 1024
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        const unsigned d = digit_of(key[it], pass); // padding keys are all ones: digit 255, at the tile's end
        const Peers peers = match_digit<8>(d);
        const unsigned before = s_cnt[wave][d], r = peers.rank();
        rnk[it] = before + r;
        if (r == 0) s_cnt[wave][d] = before + peers.count();
    }
    __syncthreads();
    // thread d < 256: per-wave exclusive offsets of digit d, tile total, global base
    unsigned run = 0, incl_t = 0, incl_g = 0, tot_g = 0;
    if (threadIdx.x < kRadix) {
        const unsigned d = threadIdx.x;
        for (int w = 0; w < kScWaves; ++w) {
            const unsigned c = s_cnt[w][d];
            s_cnt[w][d] = run;
            run += c;
        }
        // exclusive scans over the 256 digits: tile totals (-> s_start) and global totals
        incl_t = run;
        incl_g = tot_g = digit_total[d];
        for (int o = 1; o < kWave; o <<= 1) {
            unsigned a = __shfl_up(incl_t, o, kWave), g = __shfl_up(incl_g, o, kWave);
            if (lane >= o) {
                incl_t += a;
                incl_g += g;
            }
        }
        if (lane == kWave - 1) {
            s_wt[wave] = incl_t;
            s_wg[wave] = incl_g;
        }
    }
    __syncthreads();
    if (threadIdx.x < kRadix) {
        const unsigned d = threadIdx.x;
        unsigned off_t = 0, off_g = 0;
        for (int w = 0; w < wave; ++w) {
            off_t += s_wt[w];
            off_g += s_wg[w];
        }
        const unsigned start = off_t + incl_t - run;
        const unsigned gbase = off_g + incl_g - tot_g;
        s_start[d] = start;
        s_delta[d] = gbase + tile_hist[(size_t)d * n_tiles + tile] - start;
    }
    __syncthreads();
    // position of every key in the sorted tile, taken before the tile overwrites the counters
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        const unsigned d = digit_of(key[it], pass);
        rnk[it] += s_start[d] + s_cnt[wave][d];
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        s_key[rnk[it]] = key[it];
        s_idx[rnk[it]] = idx[it];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < tile_n; e += kScThreads) {
        const uint64_t k = s_key[e];
        const unsigned g = s_delta[digit_of(k, pass)] + (unsigned)e;   // < n < 2^31
        out_k[g] = k;
        out_i[g] = s_idx[e];
    }
}

// ---------------------------------------------------------------------------- heads -> unique
// head(j) = key differs from its predecessor in sorted order

__global__ __launch_bounds__(kThreads) void k_heads_count(DdBuffers b, const DdHeader* __restrict__ h, int64_t n,
                                                         unsigned* __restrict__ tile_heads) {
    const uint64_t* keys = sel_keys(b, h->final_sel);
    __shared__ unsigned s_w[kWaves];
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int64_t base = (int64_t)blockIdx.x * kTile + wave * (kWave * kItems) + lane;
    unsigned cnt = 0;
    uint64_t cur[kItems], prev[kItems];
#pragma unroll
    for (int it = 0; it < kItems; ++it) {          // all loads first, unconditional: see k_dd_masks
        const int64_t j = base + it * kWave;
        const int64_t jc = j < n ? j : n - 1;
        cur[it] = keys[jc];
        prev[it] = keys[jc > 0 ? jc - 1 : 0];
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t j = base + it * kWave;
        if (j < n) cnt += (j == 0 || cur[it] != prev[it]) ? 1u : 0u;
    }
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, kWave);
    if (lane == 0) s_w[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) tile_heads[blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

// single block: exclusive scan of the per-tile head counts; total = number of distinct keys
__global__ __launch_bounds__(1024) void k_heads_scan(unsigned* __restrict__ tile_heads, unsigned n_tiles, DdHeader* h,
                                                    int64_t* n_unique_out) {
    __shared__ unsigned s_wave[16];
    __shared__ unsigned s_carry;
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    if (threadIdx.x == 0) s_carry = 0u;
    __syncthreads();
    for (unsigned base = 0; base < n_tiles; base += 1024) {
        const unsigned i = base + threadIdx.x;
        const unsigned v = i < n_tiles ? tile_heads[i] : 0u;
        unsigned incl = v;
        for (int o = 1; o < kWave; o <<= 1) {
            unsigned t = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += t;
        }
        if (lane == kWave - 1) s_wave[wave] = incl;
        __syncthreads();
        unsigned woff = 0;
        for (int w = 0; w < wave; ++w) woff += s_wave[w];
        const unsigned carry = s_carry;
        if (i < n_tiles) tile_heads[i] = carry + woff + incl - v;
        __syncthreads();
        if (threadIdx.x == 1023) s_carry = carry + woff + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        h->n_unique = (long long)s_carry;
        *n_unique_out = (int64_t)s_carry;
    }
}

__global__ __launch_bounds__(kThreads) void k_emit(DdBuffers b, const DdHeader* __restrict__ h, int64_t n,
                                                  const unsigned* __restrict__ tile_heads, uint64_t* __restrict__ uniq,
                                                  int32_t* __restrict__ inverse, int32_t* __restrict__ perm,
                                                  int32_t* __restrict__ seg_off, int32_t* __restrict__ seg_of) {
    const int sel = h->final_sel;
    const uint64_t* keys = sel_keys(b, sel);
    const uint32_t* idxs = sel_idx(b, sel);
    __shared__ unsigned s_w[kWaves];
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int64_t base = (int64_t)blockIdx.x * kTile + wave * (kWave * kItems) + lane;
    // pass 1: heads per wave
    uint64_t key[kItems], prev[kItems];
    uint32_t pos[kItems];
    unsigned headbits = 0; // bit it = element is a head
    unsigned cnt = 0;
#pragma unroll
    for (int it = 0; it < kItems; ++it) {          // all loads first, unconditional: see k_dd_masks
        const int64_t j = base + it * kWave;
        const int64_t jc = j < n ? j : n - 1;
        key[it] = keys[jc];
        prev[it] = keys[jc > 0 ? jc - 1 : 0];
        pos[it] = idxs ? idxs[jc] : (uint32_t)j;
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t j = base + it * kWave;
        const bool head = j < n && (j == 0 || key[it] != prev[it]);
        headbits |= head ? (1u << it) : 0u;
        cnt += head ? 1u : 0u;
    }
    unsigned wave_total = cnt;
    for (int o = 32; o > 0; o >>= 1) wave_total += __shfl_xor(wave_total, o, kWave);
    if (lane == 0) s_w[wave] = wave_total;
    __syncthreads();
    unsigned running = tile_heads[blockIdx.x];
    for (int w = 0; w < wave; ++w) running += s_w[w];
    // pass 2: element order inside the wave is (it, lane)
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t j = base + it * kWave;
        const bool head = (headbits >> it) & 1u;
        const uint64_t m = __ballot(head);
        const unsigned seg = running + (unsigned)rank_in(m, lane) + (head ? 1u : 0u) - 1u; // heads up to and incl. j, minus 1
        running += (unsigned)__popcll(m);
        if (j < n) {
            const uint32_t p = pos[it];
            if (inverse) inverse[p] = (int32_t)seg;
            // the mapping is read again a gigabyte of traffic later (expand, reduce): no cache allocation
            if (perm) __builtin_nontemporal_store((int32_t)p, &perm[j]);
            if (seg_of) __builtin_nontemporal_store((int32_t)seg, &seg_of[j]);
            if (head) {
                uniq[seg] = key[it];
                if (seg_off) seg_off[seg] = (int32_t)j;
            }
            if (j == n - 1 && seg_off) seg_off[seg + 1] = (int32_t)n;
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_counts(const int32_t* __restrict__ seg_off, const DdHeader* __restrict__ h,
                                                    int32_t* __restrict__ counts) {
    const int64_t u = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (u < h->n_unique) counts[u] = seg_off[u + 1] - seg_off[u];
}

__global__ void k_empty_result(int64_t* n_unique, int32_t* seg_off) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *n_unique = 0;
        if (seg_off) seg_off[0] = 0;
    }
}

constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct DdLayout {
    size_t header, masks, ka, kb, ia, ib, tile_hist, digit_total, tile_heads, seg_off, total;
    unsigned n_tiles;
};
constexpr DdLayout dd_layout(int64_t n) {
    DdLayout L{};
    L.n_tiles = (unsigned)((n + kTile - 1) / kTile);
    size_t o = 0;
    L.header = o; o = align_up(o + sizeof(DdHeader), 256);
    L.masks = o; o = align_up(o + (size_t)L.n_tiles * 16, 256);
    L.ka = o; o = align_up(o + (size_t)n * 8, 256);
    L.kb = o; o = align_up(o + (size_t)n * 8, 256);
    L.ia = o; o = align_up(o + (size_t)n * 4, 256);
    L.ib = o; o = align_up(o + (size_t)n * 4, 256);
    L.tile_hist = o; o = align_up(o + (size_t)kRadix * L.n_tiles * 4, 256);
    L.digit_total = o; o = align_up(o + kRadix * 4, 256);
    L.tile_heads = o; o = align_up(o + (size_t)L.n_tiles * 4, 256);
    L.seg_off = o; o = align_up(o + (size_t)(n + 1) * 4, 256);
    L.total = o;
    return L;
}

// Scratch of the allocation-free entry point: the workspace of a deduplication of up to
// EMB_DEDUP_NOALLOC_MAX_KEYS keys, resident on every device the library runs on until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the resolved address.
constexpr size_t kScratchBytes = dd_layout(EMB_DEDUP_NOALLOC_MAX_KEYS).total;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// address of `scratch` on the current device, resolved once per device
int scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return EMB_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return EMB_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return EMB_OK;
}

} // namespace

extern "C" {

int emb_tag_keys(const uint64_t* x, const int64_t* field_off, const uint8_t* field_tag, int n_fields,
                 int64_t n, int tag_bits, uint64_t* key_out, int64_t* err_count, void* stream) {
    return mtgr::tag_keys_limited(x, field_off, field_tag, n_fields, n, tag_bits, 63, key_out, err_count, stream);
}

} // extern "C"

int mtgr::tag_keys_limited(const uint64_t* x, const int64_t* field_off, const uint8_t* field_tag, int n_fields,
                           int64_t n, int tag_bits, int id_bits, uint64_t* key_out, int64_t* err_count, void* stream) {
    if (n < 0 || n_fields < 0 || n_fields > 4096 || tag_bits < 0 || tag_bits > 16 || id_bits < 1 || !err_count) return EMB_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_zero64, dim3(1), dim3(64), 0, s, reinterpret_cast<unsigned long long*>(err_count));
    MTGR_LAUNCH_CHECK();
    if (n == 0) return EMB_OK;
    if (!x || !field_off || !field_tag || !key_out || n_fields == 0) return EMB_ERR_INVALID_ARG;
    unsigned grid = (unsigned)((n + kThreads * 4 - 1) / (kThreads * 4));
    if (grid > 65536u) grid = 65536u;
    hipLaunchKernelGGL(k_tag, dim3(grid), dim3(kThreads), (size_t)(n_fields + 1) * sizeof(int64_t), s, x, field_off,
                       field_tag, n_fields, n, 63 - tag_bits, id_bits, key_out, reinterpret_cast<unsigned long long*>(err_count));
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

extern "C" {

size_t emb_dedup_workspace_bytes(int64_t n) {
    if (n < 0) return 0;
    return dd_layout(n < 1 ? 1 : n).total;
}

int emb_dedup_noalloc(const uint64_t* key, int64_t n, uint64_t* uniq, int32_t* inverse, int32_t* counts,
                      int32_t* perm, int32_t* seg_off, int32_t* seg_of, int64_t* n_unique, void* stream) {
    if (n > EMB_DEDUP_NOALLOC_MAX_KEYS) return EMB_ERR_TOO_LARGE;
    void* ws = nullptr;
    const int rc = scratch_of_current_device(&ws);
    if (rc != EMB_OK) return rc;
    return emb_dedup(key, n, uniq, inverse, counts, perm, seg_off, seg_of, n_unique, ws, kScratchBytes, stream);
}

int emb_dedup(const uint64_t* key, int64_t n, uint64_t* uniq, int32_t* inverse, int32_t* counts,
              int32_t* perm, int32_t* seg_off, int32_t* seg_of, int64_t* n_unique, void* workspace,
              size_t workspace_bytes, void* stream) {
    if (n < 0 || n > 0x7FFFFFFFll || !n_unique) return EMB_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n == 0) {
        hipLaunchKernelGGL(k_empty_result, dim3(1), dim3(64), 0, s, n_unique, seg_off);
        MTGR_LAUNCH_CHECK();
        return EMB_OK;
    }
    if (!key || !uniq) return EMB_ERR_INVALID_ARG;
    const DdLayout L = dd_layout(n);
    if (!workspace || workspace_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return EMB_ERR_WORKSPACE;
    char* w = static_cast<char*>(workspace);
    DdHeader* hdr = reinterpret_cast<DdHeader*>(w + L.header);
    DdBuffers b;
    b.in_keys = key;
    b.ka = reinterpret_cast<uint64_t*>(w + L.ka);
    b.kb = reinterpret_cast<uint64_t*>(w + L.kb);
    b.ia = reinterpret_cast<uint32_t*>(w + L.ia);
    b.ib = reinterpret_cast<uint32_t*>(w + L.ib);
    unsigned* tile_hist = reinterpret_cast<unsigned*>(w + L.tile_hist);
    unsigned* digit_total = reinterpret_cast<unsigned*>(w + L.digit_total);
    unsigned* tile_heads = reinterpret_cast<unsigned*>(w + L.tile_heads);
    int32_t* seg = seg_off ? seg_off : reinterpret_cast<int32_t*>(w + L.seg_off);
    const unsigned n_tiles = L.n_tiles;

    unsigned long long* masks = reinterpret_cast<unsigned long long*>(w + L.masks);
    hipLaunchKernelGGL(k_dd_masks, dim3(xcd_grid(n_tiles)), dim3(kThreads), 0, s, key, n, n_tiles, masks, tile_hist);
    hipLaunchKernelGGL(k_dd_plan, dim3(1), dim3(kThreads), 0, s, hdr, masks, (int)n_tiles);
    MTGR_LAUNCH_CHECK();
    for (int p = 0; p < kPasses; ++p) {
        if (p > 0) // the lowest digit's histogram came with the mask reduction
            hipLaunchKernelGGL(k_rs_hist, dim3(xcd_grid(n_tiles)), dim3(kThreads), 0, s, b, hdr, p, n, n_tiles, tile_hist);
        hipLaunchKernelGGL(k_rs_scan, dim3(kRadix), dim3(kThreads), 0, s, hdr, p, n_tiles, tile_hist, digit_total);
        hipLaunchKernelGGL(k_rs_scatter, dim3(xcd_grid(n_tiles)), dim3(kScThreads), 0, s, b, hdr, p, n, n_tiles, tile_hist, digit_total);
        MTGR_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(k_heads_count, dim3(n_tiles), dim3(kThreads), 0, s, b, hdr, n, tile_heads);
    hipLaunchKernelGGL(k_heads_scan, dim3(1), dim3(1024), 0, s, tile_heads, n_tiles, hdr, n_unique);
    hipLaunchKernelGGL(k_emit, dim3(n_tiles), dim3(kThreads), 0, s, b, hdr, n, tile_heads, uniq, inverse, perm, seg, seg_of);
    MTGR_LAUNCH_CHECK();
    if (counts) {
        hipLaunchKernelGGL(k_counts, dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, seg, hdr, counts);
        MTGR_LAUNCH_CHECK();
    }
    return EMB_OK;
}

} // extern "C"
