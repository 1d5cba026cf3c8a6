// ID tagging (Eq. 8) and stage-1 deduplication (Sec. 3.3) in one call, for gfx950.
//
// emb_tag_dedup sorts 8-byte records (raw ID << pos_bits | position) instead of (tagged key, position)
// pairs of 12 bytes.  The table identifier of Eq. 8 is a function of the position (IDs arrive field by
// field), so it is not stored: the one radix pass whose digit reaches into the identifier bits looks it
// up from the position, and after the sort the records of identifier t occupy a known range of the
// sorted order.  The caller declares how many bits a raw ID can have (id_bits), which fixes the
// number of radix passes on the host: ceil((id_bits + tag_bits) / 9) passes of at most 9 bits, no
// pass is launched for bits that cannot vary, and the tagged keys are never written unless asked for.
// Stable LSD passes keep equal IDs in position order.  Per pass: per-tile histogram, per-digit scan
// over tiles, scatter (wave-ballot ranking, tile reordered in LDS, digit runs written contiguously).
#include "common.hpp"

using namespace mtgr;

namespace {

constexpr int kThreads = 256;
constexpr int kItems = 16;                    // records per thread
constexpr int kTile = kThreads * kItems;      // 4096 records per block (8192 measured 9-13 % slower for the whole call)
constexpr int kWaves = kThreads / kWave;      // 4
constexpr int kScThreads = 512;               // scatter kernel: same tile, more and lighter threads
constexpr int kScItems = kTile / kScThreads;
constexpr int kScWaves = kScThreads / kWave;
constexpr int kMaxBits = 9;                   // widest digit
constexpr int kMaxRadix = 1 << kMaxBits;
constexpr int kMaxPasses = 8;                 // 63 key bits / 9, rounded up
constexpr int kMaxFields = 1024;              // field table kept in LDS by the kernels that need the identifier

// What every kernel of one call needs, by value.
struct PkArgs {
    const uint64_t* x;          // raw IDs
    const int64_t* field_off;   // [n_fields + 1]
    const uint8_t* field_tag;   // [n_fields]
    int n_fields;
    int64_t n;
    unsigned n_tiles;
    int id_bits;                // raw IDs are below 2^id_bits (larger ones are counted and wrapped)
    int tag_shift;              // 63 - tag_bits: position of the identifier in the tagged key
    int pos_bits;               // low bits of a record that hold the position
    uint64_t* rec_a;
    uint64_t* rec_b;
    unsigned* tile_hist;        // [radix][n_tiles]
    unsigned* digit_total;      // [radix]
    unsigned* tile_heads;       // [n_tiles]
    unsigned* tag_start;        // [257] first sorted position of every identifier
};

struct PassPlan {
    int shift;                  // lowest bit of the digit within the virtual key (identifier << id_bits | id)
    int bits;                   // digit width
};

// Tile handled by a block.  Workgroups are handed to the 8 XCDs (each with its own L2) in turn, so with
// tile = blockIdx the neighbours of a tile run under other L2s.  Neighbouring tiles share memory sectors:
// their entries of one digit's row of tile_hist are adjacent 4-byte words, and their runs of one digit are
// adjacent in the scatter's output.  Giving every XCD a contiguous range of tiles lets its L2 merge those
// partial-sector accesses (36 MB of sector traffic per histogram and per scatter otherwise, for 4.5 MB of
// counters).  The grid is 8 * ceil(n_tiles / 8) blocks; a block whose tile does not exist leaves at once.
constexpr unsigned kXcds = 8;
__device__ inline unsigned tile_of_block(unsigned n_tiles) {
    const unsigned per = (n_tiles + kXcds - 1) / kXcds;
    return (blockIdx.x % kXcds) * per + blockIdx.x / kXcds;
}
inline unsigned xcd_grid(unsigned n_tiles) { return kXcds * ((n_tiles + kXcds - 1) / kXcds); }

// last field whose start is <= e (s_off[0] <= e < s_off[n_fields])
__device__ inline int field_of(const int64_t* s_off, int n_fields, int64_t e) {
    int lo = 0, hi = n_fields;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_off[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

// LDS copy of the field table: offsets, then identifiers
struct FieldTable {
    const int64_t* off;
    const uint8_t* tag;
    int n_fields;
    __device__ inline unsigned tag_of(int64_t pos) const { return tag[field_of(off, n_fields, pos)]; }
};
__device__ inline FieldTable load_fields(const PkArgs& a, unsigned char* smem, int n_threads) {
    int64_t* s_off = reinterpret_cast<int64_t*>(smem);
    uint8_t* s_tag = reinterpret_cast<uint8_t*>(s_off + a.n_fields + 1);
    for (int f = threadIdx.x; f <= a.n_fields; f += n_threads) s_off[f] = a.field_off[f];
    for (int f = threadIdx.x; f < a.n_fields; f += n_threads) s_tag[f] = a.field_tag[f];
    return FieldTable{s_off, s_tag, a.n_fields};
}
__host__ __device__ inline size_t field_table_bytes(int n_fields) { return (size_t)(n_fields + 1) * 8 + (size_t)((n_fields + 7) & ~7); }

// digit of a record in the given pass; WITH_TAG: the digit reaches into the identifier bits
template <bool WITH_TAG>
__device__ inline unsigned digit_of(uint64_t rec, const PkArgs& a, PassPlan p, const FieldTable& ft) {
    uint64_t k = rec >> a.pos_bits;
    if (WITH_TAG) k |= (uint64_t)ft.tag_of((int64_t)(rec & ((1ull << a.pos_bits) - 1ull))) << a.id_bits;
    return (unsigned)(k >> p.shift) & ((1u << p.bits) - 1u);
}

// Add a wave's 64 digits to an LDS histogram; neighbouring lanes with the same digit are counted as
// one run and added once (a popular ID would otherwise serialise 64 lanes on one counter).
// d >= kMaxRadix means "no record".
__device__ inline void hist_add_runs(unsigned* s_hist, unsigned d, int lane) {
    const unsigned prev = __shfl_up(d, 1, kWave);
    const bool head = lane == 0 || d != prev;
    const uint64_t heads = __ballot(head);
    if (head && d < (unsigned)kMaxRadix) {
        const uint64_t rest = (heads >> lane) >> 1;
        const unsigned len = rest ? (unsigned)__ffsll((unsigned long long)rest) : (unsigned)(kWave - lane);
        atomicAdd(&s_hist[d], len);
    }
}

// raw ID -> ID within id_bits (and within 63 - tag_bits, Eq. 8); out-of-range IDs are counted and wrapped
__device__ inline uint64_t checked_id(uint64_t v, const PkArgs& a, unsigned* errs) {
    const int bits = a.id_bits < a.tag_shift ? a.id_bits : a.tag_shift;
    const uint64_t mask = (1ull << bits) - 1ull;
    if (v > mask) {
        ++*errs;
        v &= mask;
    }
    return v;
}

// ---------------------------------------------------------------------------- set-up
// One block: sorted-order start of every identifier (counts of the fields that carry it, prefix-summed).
__global__ __launch_bounds__(256) void k_pk_plan(PkArgs a, unsigned long long* err_count) {
    __shared__ unsigned s_cnt[256];
    s_cnt[threadIdx.x] = 0u;
    __syncthreads();
    for (int f = threadIdx.x; f < a.n_fields; f += 256)
        atomicAdd(&s_cnt[a.field_tag[f]], (unsigned)(a.field_off[f + 1] - a.field_off[f]));
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned run = 0;
        for (int t = 0; t < 256; ++t) {
            a.tag_start[t] = run;
            run += s_cnt[t];
        }
        a.tag_start[256] = run;
        *err_count = 0ull;
    }
}

// ---------------------------------------------------------------------------- histograms
// First pass: the records do not exist yet; the digit comes straight from the raw IDs, which are also
// range-checked here (once per call), and the tagged keys are written when the caller wants them.
template <bool WITH_TAG>
__global__ __launch_bounds__(kThreads) void k_pk_hist0(PkArgs a, PassPlan p, uint64_t* __restrict__ key_out,
                                                      unsigned long long* err_count) {
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
    __shared__ unsigned s_hist[kMaxRadix];
    const unsigned tile = tile_of_block(a.n_tiles);
    if (tile >= a.n_tiles) return;
    for (int i = threadIdx.x; i < kMaxRadix; i += kThreads) s_hist[i] = 0u;
    const FieldTable ft = load_fields(a, s_dyn, kThreads);
    __syncthreads();
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int64_t wave_base = (int64_t)tile * kTile + wave * (kWave * kItems);
    // identifier of the wave's 1024 positions: one field lookup when they lie in one field
    const bool need_tag = WITH_TAG || key_out != nullptr;
    int f_first = 0, f_last = 0;
    if (need_tag && wave_base < a.n) {
        const int64_t last = wave_base + kWave * kItems - 1 < a.n ? wave_base + kWave * kItems - 1 : a.n - 1;
        f_first = field_of(ft.off, ft.n_fields, wave_base);
        f_last = field_of(ft.off, ft.n_fields, last);
    }
    unsigned errs = 0;
    // Two batches of eight IDs per lane: all loads of a batch go out before anything waits, and a digit goes to the
    // histogram as soon as it is known.  (Sixteen IDs and sixteen digits held at once cost the kernel a quarter of
    // its resident waves - 74 registers - and with them a second round of blocks.)
    constexpr int kHalf = kItems / 2;
#pragma unroll 1
    for (int h = 0; h < 2; ++h) {
        const int64_t e0 = wave_base + h * (kHalf * kWave) + lane;
        uint64_t raw[kHalf];
#pragma unroll
        for (int it = 0; it < kHalf; ++it) raw[it] = e0 + it * kWave < a.n ? a.x[e0 + it * kWave] : 0ull;
#pragma unroll
        for (int it = 0; it < kHalf; ++it) {
            const int64_t e = e0 + it * kWave;
            unsigned d = kMaxRadix;
            if (e < a.n) {
                const uint64_t id = checked_id(raw[it], a, &errs);
                uint64_t k = id;
                if (need_tag) {
                    const unsigned tag = ft.tag[f_first == f_last ? f_first : field_of(ft.off, ft.n_fields, e)];
                    if (key_out) key_out[e] = ((uint64_t)tag << a.tag_shift) | id;
                    if (WITH_TAG) k |= (uint64_t)tag << a.id_bits;
                }
                d = (unsigned)(k >> p.shift) & ((1u << p.bits) - 1u);
            }
            hist_add_runs(s_hist, d, lane);
        }
    }
    for (int o = 32; o > 0; o >>= 1) errs += __shfl_xor(errs, o, kWave);
    if (errs && lane == 0) atomicAdd(err_count, (unsigned long long)errs);
    __syncthreads();
    for (int i = threadIdx.x; i < (1 << p.bits); i += kThreads) a.tile_hist[(size_t)i * a.n_tiles + tile] = s_hist[i];
}

template <bool WITH_TAG>
__global__ __launch_bounds__(kThreads) void k_pk_hist(PkArgs a, PassPlan p, const uint64_t* __restrict__ src) {
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
    __shared__ unsigned s_hist[kMaxRadix];
    const unsigned tile = tile_of_block(a.n_tiles);
    if (tile >= a.n_tiles) return;
    for (int i = threadIdx.x; i < kMaxRadix; i += kThreads) s_hist[i] = 0u;
    FieldTable ft{nullptr, nullptr, 0};
    if (WITH_TAG) ft = load_fields(a, s_dyn, kThreads);
    __syncthreads();
    const int lane = lane_id();
    const int64_t base = (int64_t)tile * kTile + (threadIdx.x / kWave) * (kWave * kItems) + lane;
    uint64_t r[kItems];
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t e = base + it * kWave;
        r[it] = e < a.n ? src[e] : ~0ull;
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t e = base + it * kWave;
        const unsigned d = e < a.n ? digit_of<WITH_TAG>(r[it], a, p, ft) : (unsigned)kMaxRadix;
        hist_add_runs(s_hist, d, lane);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < (1 << p.bits); i += kThreads) a.tile_hist[(size_t)i * a.n_tiles + tile] = s_hist[i];
}

// block d: exclusive scan of digit d's counts over the tiles; total -> digit_total[d].
// Every thread owns a run of consecutive tiles, so the block-wide scan happens once.
__global__ __launch_bounds__(kThreads) void k_pk_scan(PkArgs a) {
    __shared__ unsigned s_wave[kWaves];
    unsigned* row = a.tile_hist + (size_t)blockIdx.x * a.n_tiles;
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const unsigned per = (a.n_tiles + kThreads - 1) / kThreads;
    const unsigned lo = threadIdx.x * per < a.n_tiles ? threadIdx.x * per : a.n_tiles;
    const unsigned hi = lo + per < a.n_tiles ? lo + per : a.n_tiles;
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
    if (threadIdx.x == kThreads - 1) a.digit_total[blockIdx.x] = run;
}

// ---------------------------------------------------------------------------- scatter
// tile element e = wave*(64*kScItems) + item*64 + lane.  FIRST: records are built from the raw IDs.
template <int BITS, bool FIRST, bool WITH_TAG>
__global__ __launch_bounds__(kScThreads) void k_pk_scatter(PkArgs a, PassPlan p, const uint64_t* __restrict__ src,
                                                          uint64_t* __restrict__ dst) {
    constexpr int kRadix = 1 << BITS;
    // LDS: the reordered tile (32 KB) and, before it is filled, the counters in the same memory;
    // only the per-digit output offsets live apart.
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
    __shared__ __attribute__((aligned(16))) unsigned char s_raw[kTile * 8];
    __shared__ unsigned s_delta[kRadix];         // global position - tile position for digit d (mod 2^32)
    static_assert(kScWaves * kRadix * 4 + kRadix * 4 + 2 * kScWaves * 4 <= kTile * 8, "counters must fit under the tile");
    static_assert(kScThreads >= kRadix, "one thread per digit computes the digit's offsets");
    uint64_t* s_rec = reinterpret_cast<uint64_t*>(s_raw);
    unsigned (*s_cnt)[kRadix] = reinterpret_cast<unsigned (*)[kRadix]>(s_raw);            // [kScWaves][kRadix]
    unsigned* s_start = reinterpret_cast<unsigned*>(s_raw) + kScWaves * kRadix;             // [kRadix]
    unsigned* s_wt = s_start + kRadix;                                                    // [kScWaves]
    unsigned* s_wg = s_wt + kScWaves;                                                     // [kScWaves]

    const unsigned tile = tile_of_block(a.n_tiles);
    if (tile >= a.n_tiles) return;
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int64_t tile_base = (int64_t)tile * kTile;
    const int tile_n = (int)((a.n - tile_base) < kTile ? (a.n - tile_base) : kTile);
    for (int i = threadIdx.x; i < kScWaves * kRadix; i += kScThreads) s_cnt[0][i] = 0u;
    FieldTable ft{nullptr, nullptr, 0};
    if (WITH_TAG) ft = load_fields(a, s_dyn, kScThreads);
    __syncthreads();

    uint64_t rec[kScItems];
    unsigned dig[kScItems];
    unsigned rnk[kScItems];
    const int e0 = wave * (kWave * kScItems) + lane;
    unsigned unused_errs = 0;
    // all loads first and none behind a branch (an element past the tile's end reads the tile's last one instead):
    // a load inside a conditional makes the compiler wait for it on the spot, one round trip per item
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        const int e = e0 + it * kWave;
        rec[it] = src[tile_base + (e < tile_n ? e : tile_n - 1)];
    }
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        const int e = e0 + it * kWave;
        const bool ok = e < tile_n;
        if (FIRST) rec[it] = ok ? (checked_id(rec[it], a, &unused_errs) << a.pos_bits) | (uint64_t)(tile_base + e) : ~0ull;
        else rec[it] = ok ? rec[it] : ~0ull;
    }
    // rank of every record among the records of equal digit that precede it in this wave's share
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        const int e = e0 + it * kWave;
        // padding records take the highest digit and sit at the tile's end
        const unsigned d = e < tile_n ? digit_of<WITH_TAG>(rec[it], a, p, ft) : (unsigned)(kRadix - 1);
        dig[it] = d;
        const Peers peers = match_digit<BITS>(d);
        const unsigned before = s_cnt[wave][d], r = peers.rank();
        rnk[it] = before + r;
        if (r == 0) s_cnt[wave][d] = before + peers.count();
    }
    __syncthreads();
    // thread d < kRadix: per-wave exclusive offsets of digit d, tile total, global base
    unsigned run = 0, incl_t = 0, incl_g = 0, tot_g = 0;
    if (threadIdx.x < kRadix) {
        const unsigned d = threadIdx.x;
        for (int w = 0; w < kScWaves; ++w) {
            const unsigned c = s_cnt[w][d];
            s_cnt[w][d] = run;
            run += c;
        }
        // exclusive scans over the digits: tile totals (-> s_start) and global totals
        incl_t = run;
        incl_g = tot_g = d < (1u << p.bits) ? a.digit_total[d] : 0u;
        for (int o = 1; o < kWave; o <<= 1) {
            unsigned t = __shfl_up(incl_t, o, kWave), g = __shfl_up(incl_g, o, kWave);
            if (lane >= o) {
                incl_t += t;
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
        s_delta[d] = gbase + (d < (1u << p.bits) ? a.tile_hist[(size_t)d * a.n_tiles + tile] : 0u) - start;
    }
    __syncthreads();
    // position of every record in the sorted tile, taken before the tile overwrites the counters
#pragma unroll
    for (int it = 0; it < kScItems; ++it) rnk[it] += s_start[dig[it]] + s_cnt[wave][dig[it]];
    __syncthreads();
    // the digit rides along in the record's place only if it cannot be recomputed cheaply: keep it in a
    // parallel 16-bit array above the tile when the identifier is part of it
    uint16_t* s_dig = reinterpret_cast<uint16_t*>(s_dyn + ((field_table_bytes(WITH_TAG ? a.n_fields : 0) + 15) & ~(size_t)15));
#pragma unroll
    for (int it = 0; it < kScItems; ++it) {
        s_rec[rnk[it]] = rec[it];
        if (WITH_TAG) s_dig[rnk[it]] = (uint16_t)dig[it];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < tile_n; e += kScThreads) {
        const uint64_t r = s_rec[e];
        const unsigned d = WITH_TAG ? (unsigned)s_dig[e] : digit_of<false>(r, a, p, ft);
        dst[s_delta[d] + (unsigned)e] = r;     // < n < 2^31
    }
}

// ---------------------------------------------------------------------------- heads -> unique
// head(j) = the record's (identifier, ID) differs from its predecessor's in sorted order.  Records of
// one identifier are a contiguous range of the sorted order starting at tag_start[t].

// bit e of s_bits = sorted position tile_base + e starts the range of an identifier
__device__ inline void mark_tag_starts(const PkArgs& a, int64_t tile_base, unsigned* s_bits, const unsigned* s_tag_start) {
    for (int i = threadIdx.x; i < kTile / 32; i += kThreads) s_bits[i] = 0u;
    __syncthreads();
    for (int t = threadIdx.x; t < 256; t += kThreads) {
        const int64_t s = s_tag_start[t];
        if (s_tag_start[t + 1] > s_tag_start[t] && s >= tile_base && s < tile_base + kTile)
            atomicOr(&s_bits[(s - tile_base) >> 5], 1u << ((s - tile_base) & 31));
    }
    __syncthreads();
}

// The record before a lane's item `it` in sorted order (items are laid out it * 64 + lane within a wave's 1024):
// the neighbouring lane's item, lane 63's previous item for lane 0, and one load per wave for its very first item.
__device__ inline uint64_t prev_record(const uint64_t* r, int it, int lane, uint64_t before_wave) {
    const uint64_t left = shfl64(r[it], lane == 0 ? 0 : lane - 1);
    if (lane != 0) return left;
    return it == 0 ? before_wave : shfl64(r[it - 1], kWave - 1);
}

__global__ __launch_bounds__(kThreads) void k_pk_heads_count(PkArgs a, const uint64_t* __restrict__ rec) {
    __shared__ unsigned s_w[kWaves];
    __shared__ unsigned s_bits[kTile / 32];
    __shared__ unsigned s_tag_start[257];
    for (int t = threadIdx.x; t < 257; t += kThreads) s_tag_start[t] = a.tag_start[t];
    __syncthreads();
    const int64_t tile_base = (int64_t)blockIdx.x * kTile;
    mark_tag_starts(a, tile_base, s_bits, s_tag_start);
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int e0 = wave * (kWave * kItems) + lane;
    unsigned cnt = 0;
    uint64_t r[kItems];
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t j = tile_base + e0 + it * kWave;
        r[it] = j < a.n ? rec[j] : 0ull;
    }
    const int64_t wave_first = tile_base + wave * (kWave * kItems);
    const uint64_t before_wave = (wave_first > 0 && wave_first < a.n) ? rec[wave_first - 1] : 0ull;
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int e = e0 + it * kWave;
        const int64_t j = tile_base + e;
        const uint64_t prev = prev_record(r, it, lane, before_wave);
        if (j < a.n) {
            const bool start = (s_bits[e >> 5] >> (e & 31)) & 1u;
            cnt += (j == 0 || start || (r[it] >> a.pos_bits) != (prev >> a.pos_bits)) ? 1u : 0u;
        }
    }
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, kWave);
    if (lane == 0) s_w[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) a.tile_heads[blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

// single block: exclusive scan of the per-tile head counts; total = number of distinct keys
__global__ __launch_bounds__(1024) void k_pk_heads_scan(unsigned* __restrict__ tile_heads, unsigned n_tiles,
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
    if (threadIdx.x == 0) *n_unique_out = (int64_t)s_carry;
}

// own_prefix: tile_heads holds the tiles' raw head counts and every block sums the counts of the tiles before its own
// (a few KB from L2 per block, which saves the launch of a single-block scan between two dependent kernels; used up to
// kOwnPrefixTiles tiles); otherwise tile_heads holds their exclusive prefix sums (k_pk_heads_scan).  The last tile
// writes the number of distinct keys in the first case.
constexpr unsigned kOwnPrefixTiles = 8192;
// the last t < 256 with tag_start[t] <= j
__device__ inline int tag_of_sorted(const unsigned* s_tag_start, int64_t j) {
    int lo = 0, hi = 256;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)s_tag_start[mid] <= j) lo = mid; else hi = mid;
    }
    return lo;
}
__global__ __launch_bounds__(kThreads) void k_pk_emit(PkArgs a, const uint64_t* __restrict__ rec,
                                                     uint64_t* __restrict__ uniq, int32_t* __restrict__ inverse,
                                                     int32_t* __restrict__ perm, int32_t* __restrict__ seg_off,
                                                     int32_t* __restrict__ seg_of, int own_prefix,
                                                     int64_t* __restrict__ n_unique_out) {
    __shared__ unsigned s_w[kWaves];
    __shared__ unsigned s_pre[kWaves];
    __shared__ unsigned s_bits[kTile / 32];
    __shared__ unsigned s_tag_start[257];
    unsigned before = 0;       // heads in the tiles before this one: this thread's share (own_prefix) or all (thread 0)
    if (own_prefix) {
        for (unsigned t = threadIdx.x; t < blockIdx.x; t += kThreads) before += a.tile_heads[t];
    } else if (threadIdx.x == 0) {
        before = a.tile_heads[blockIdx.x];
    }
    for (int t = threadIdx.x; t < 257; t += kThreads) s_tag_start[t] = a.tag_start[t];
    __syncthreads();
    const int64_t tile_base = (int64_t)blockIdx.x * kTile;
    mark_tag_starts(a, tile_base, s_bits, s_tag_start);
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int e0 = wave * (kWave * kItems) + lane;
    const uint64_t pos_mask = (1ull << a.pos_bits) - 1ull;
    // pass 1: heads per wave
    uint64_t r[kItems];
    unsigned headbits = 0; // bit it = element is a head
    unsigned cnt = 0;
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t j = tile_base + e0 + it * kWave;
        r[it] = j < a.n ? rec[j] : 0ull;
    }
    const int64_t wave_first = tile_base + wave * (kWave * kItems);
    const uint64_t before_wave = (wave_first > 0 && wave_first < a.n) ? rec[wave_first - 1] : 0ull;
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int e = e0 + it * kWave;
        const int64_t j = tile_base + e;
        const uint64_t prev = prev_record(r, it, lane, before_wave);
        const bool start = (s_bits[e >> 5] >> (e & 31)) & 1u;
        const bool head = j < a.n && (j == 0 || start || (r[it] >> a.pos_bits) != (prev >> a.pos_bits));
        headbits |= head ? (1u << it) : 0u;
        cnt += head ? 1u : 0u;
    }
    unsigned wave_total = cnt;
    for (int o = 32; o > 0; o >>= 1) {
        wave_total += __shfl_xor(wave_total, o, kWave);
        before += __shfl_xor(before, o, kWave);
    }
    if (lane == 0) {
        s_w[wave] = wave_total;
        s_pre[wave] = before;
    }
    __syncthreads();
    unsigned running = s_pre[0] + s_pre[1] + s_pre[2] + s_pre[3];
    if (own_prefix && blockIdx.x == a.n_tiles - 1 && threadIdx.x == 0)
        *n_unique_out = (int64_t)(running + s_w[0] + s_w[1] + s_w[2] + s_w[3]);
    for (int w = 0; w < wave; ++w) running += s_w[w];
    const int64_t wave_last = wave_first + kWave * kItems - 1 < a.n ? wave_first + kWave * kItems - 1 : a.n - 1;
    const int tag_lo = wave_first < a.n ? tag_of_sorted(s_tag_start, wave_first) : 0;
    const int tag_hi = wave_first < a.n ? tag_of_sorted(s_tag_start, wave_last) : 0;
    // pass 2: element order inside the wave is (it, lane)
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        const int64_t j = tile_base + e0 + it * kWave;
        const bool head = (headbits >> it) & 1u;
        const uint64_t m = __ballot(head);
        const unsigned seg = running + (unsigned)rank_in(m, lane) + (head ? 1u : 0u) - 1u; // heads up to and incl. j, minus 1
        running += (unsigned)__popcll(m);
        if (j < a.n) {
            const uint32_t p = (uint32_t)(r[it] & pos_mask);
            if (inverse) inverse[p] = (int32_t)seg;
            // the mapping is read again a gigabyte of traffic later (expand, reduce): no cache allocation
            if (perm) __builtin_nontemporal_store((int32_t)p, &perm[j]);
            if (seg_of) __builtin_nontemporal_store((int32_t)seg, &seg_of[j]);
            if (head) {
                // identifier of sorted position j: the last t with tag_start[t] <= j (one search per wave when its
                // 1024 positions carry one identifier, which is the rule: there are at most 256 boundaries)
                int lo = tag_lo;
                if (tag_lo != tag_hi) lo = tag_of_sorted(s_tag_start, j);
                uniq[seg] = ((uint64_t)lo << a.tag_shift) | (r[it] >> a.pos_bits);
                if (seg_off) seg_off[seg] = (int32_t)j;
            }
            if (j == a.n - 1 && seg_off) seg_off[seg + 1] = (int32_t)a.n;
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_pk_counts(const int32_t* __restrict__ seg_off, const int64_t* __restrict__ n_unique,
                                                       int32_t* __restrict__ counts) {
    const int64_t u = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (u < *n_unique) counts[u] = seg_off[u + 1] - seg_off[u];
}

__global__ void k_pk_empty(int64_t* n_unique, int32_t* seg_off, unsigned long long* err_count) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *n_unique = 0;
        *err_count = 0ull;
        if (seg_off) seg_off[0] = 0;
    }
}

constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct PkLayout {
    size_t rec_a, rec_b, tile_hist, digit_total, tile_heads, tag_start, seg_off, total;
    unsigned n_tiles;
};
PkLayout pk_layout(int64_t n) {
    PkLayout L{};
    L.n_tiles = (unsigned)((n + kTile - 1) / kTile);
    size_t o = 0;
    L.rec_a = o; o = align_up(o + (size_t)n * 8, 256);
    L.rec_b = o; o = align_up(o + (size_t)n * 8, 256);
    L.tile_hist = o; o = align_up(o + (size_t)kMaxRadix * L.n_tiles * 4, 256);
    L.digit_total = o; o = align_up(o + kMaxRadix * 4, 256);
    L.tile_heads = o; o = align_up(o + (size_t)L.n_tiles * 4, 256);
    L.tag_start = o; o = align_up(o + 257 * 4, 256);
    L.seg_off = o; o = align_up(o + (size_t)(n + 1) * 4, 256);
    L.total = o;
    return L;
}

int bits_for(int64_t n) { // positions 0 .. n-1
    int b = 1;
    while ((1ll << b) < n) ++b;
    return b;
}

// can the call take the packed path?
bool packed_fits(int64_t n, int n_fields, int id_bits) { return n_fields <= kMaxFields && id_bits + bits_for(n) <= 64; }

} // namespace

extern "C" {

size_t emb_tag_dedup_workspace_bytes(int64_t n, int n_fields, int tag_bits, int id_bits) {
    if (n < 0) return 0;
    const int64_t m = n < 1 ? 1 : n;
    (void)tag_bits;
    if (packed_fits(m, n_fields, id_bits)) return pk_layout(m).total;
    // two-call form: the tagged keys, then the general deduplication
    return align_up((size_t)m * 8, 256) + emb_dedup_workspace_bytes(m);
}

int emb_tag_dedup(const uint64_t* x, const int64_t* field_off, const uint8_t* field_tag, int n_fields, int64_t n,
                  int tag_bits, int id_bits, uint64_t* key_out, uint64_t* uniq, int32_t* inverse, int32_t* counts,
                  int32_t* perm, int32_t* seg_off, int32_t* seg_of, int64_t* n_unique, int64_t* err_count,
                  void* workspace, size_t workspace_bytes, void* stream) {
    if (n < 0 || n > 0x7FFFFFFFll || n_fields < 0 || n_fields > 4096 || tag_bits < 0 || tag_bits > 16) return EMB_ERR_INVALID_ARG;
    if (id_bits < 1 || id_bits > 63 - tag_bits || !n_unique || !err_count) return EMB_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned long long* errs = reinterpret_cast<unsigned long long*>(err_count);
    if (n == 0) {
        hipLaunchKernelGGL(k_pk_empty, dim3(1), dim3(64), 0, s, n_unique, seg_off, errs);
        MTGR_LAUNCH_CHECK();
        return EMB_OK;
    }
    if (!x || !field_off || !field_tag || n_fields == 0 || !uniq) return EMB_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < emb_tag_dedup_workspace_bytes(n, n_fields, tag_bits, id_bits) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255))
        return EMB_ERR_WORKSPACE;
    char* w = static_cast<char*>(workspace);
    if (!packed_fits(n, n_fields, id_bits)) {
        // records of ID and position do not fit 64 bits (or too many fields for the LDS table): tag, then deduplicate
        uint64_t* keys = key_out ? key_out : reinterpret_cast<uint64_t*>(w);
        const size_t off = align_up((size_t)n * 8, 256);
        int rc = tag_keys_limited(x, field_off, field_tag, n_fields, n, tag_bits, id_bits, keys, err_count, stream);
        if (rc != EMB_OK) return rc;
        return emb_dedup(keys, n, uniq, inverse, counts, perm, seg_off, seg_of, n_unique, w + off, workspace_bytes - off, stream);
    }
    const PkLayout L = pk_layout(n);
    PkArgs a{};
    a.x = x;
    a.field_off = field_off;
    a.field_tag = field_tag;
    a.n_fields = n_fields;
    a.n = n;
    a.n_tiles = L.n_tiles;
    a.id_bits = id_bits;
    a.tag_shift = 63 - tag_bits;
    a.pos_bits = bits_for(n);
    a.rec_a = reinterpret_cast<uint64_t*>(w + L.rec_a);
    a.rec_b = reinterpret_cast<uint64_t*>(w + L.rec_b);
    a.tile_hist = reinterpret_cast<unsigned*>(w + L.tile_hist);
    a.digit_total = reinterpret_cast<unsigned*>(w + L.digit_total);
    a.tile_heads = reinterpret_cast<unsigned*>(w + L.tile_heads);
    a.tag_start = reinterpret_cast<unsigned*>(w + L.tag_start);
    int32_t* seg = seg_off ? seg_off : reinterpret_cast<int32_t*>(w + L.seg_off);

    // digits: the virtual key (identifier << id_bits | id) has id_bits + tag_bits bits, split evenly into
    // the fewest passes of at most 9 bits
    const int total_bits = id_bits + tag_bits;
    const int n_pass = (total_bits + kMaxBits - 1) / kMaxBits;
    PassPlan plan[kMaxPasses];
    {
        const int base = total_bits / n_pass, extra = total_bits % n_pass;
        int sh = 0;
        for (int p = 0; p < n_pass; ++p) {
            plan[p].shift = sh;
            plan[p].bits = base + (p < extra ? 1 : 0);
            sh += plan[p].bits;
        }
    }
    const size_t ft_bytes = field_table_bytes(n_fields);
    const size_t sc_tag_bytes = ((ft_bytes + 15) & ~(size_t)15) + (size_t)kTile * 2;   // field table + digits of the tile
    hipLaunchKernelGGL(k_pk_plan, dim3(1), dim3(256), 0, s, a, errs);
    MTGR_LAUNCH_CHECK();
    const uint64_t* src = nullptr;
    uint64_t* dst = a.rec_a;
    for (int p = 0; p < n_pass; ++p) {
        const bool with_tag = plan[p].shift + plan[p].bits > id_bits;
        if (p == 0) {
            if (with_tag) hipLaunchKernelGGL(k_pk_hist0<true>, dim3(xcd_grid(L.n_tiles)), dim3(kThreads), ft_bytes, s, a, plan[p], key_out, errs);
            else hipLaunchKernelGGL(k_pk_hist0<false>, dim3(xcd_grid(L.n_tiles)), dim3(kThreads), ft_bytes, s, a, plan[p], key_out, errs);
        } else {
            if (with_tag) hipLaunchKernelGGL(k_pk_hist<true>, dim3(xcd_grid(L.n_tiles)), dim3(kThreads), ft_bytes, s, a, plan[p], src);
            else hipLaunchKernelGGL(k_pk_hist<false>, dim3(xcd_grid(L.n_tiles)), dim3(kThreads), 0, s, a, plan[p], src);
        }
        hipLaunchKernelGGL(k_pk_scan, dim3(1u << plan[p].bits), dim3(kThreads), 0, s, a);
        MTGR_LAUNCH_CHECK();
        const uint64_t* in = p == 0 ? x : src;
#define MTGR_SC(B_, F_, T_) \
    hipLaunchKernelGGL((k_pk_scatter<B_, F_, T_>), dim3(xcd_grid(L.n_tiles)), dim3(kScThreads), (T_) ? sc_tag_bytes : 0, s, a, plan[p], in, dst)
        const bool nine = plan[p].bits > 8;
        if (p == 0) {
            if (nine) { if (with_tag) MTGR_SC(9, true, true); else MTGR_SC(9, true, false); }
            else { if (with_tag) MTGR_SC(8, true, true); else MTGR_SC(8, true, false); }
        } else {
            if (nine) { if (with_tag) MTGR_SC(9, false, true); else MTGR_SC(9, false, false); }
            else { if (with_tag) MTGR_SC(8, false, true); else MTGR_SC(8, false, false); }
        }
#undef MTGR_SC
        MTGR_LAUNCH_CHECK();
        src = dst;
        dst = (dst == a.rec_a) ? a.rec_b : a.rec_a;
    }
    hipLaunchKernelGGL(k_pk_heads_count, dim3(L.n_tiles), dim3(kThreads), 0, s, a, src);
    const int own_prefix = L.n_tiles <= kOwnPrefixTiles ? 1 : 0;
    if (!own_prefix) hipLaunchKernelGGL(k_pk_heads_scan, dim3(1), dim3(1024), 0, s, a.tile_heads, L.n_tiles, n_unique);
    hipLaunchKernelGGL(k_pk_emit, dim3(L.n_tiles), dim3(kThreads), 0, s, a, src, uniq, inverse, perm, seg, seg_of, own_prefix,
                       n_unique);
    MTGR_LAUNCH_CHECK();
    if (counts) {
        hipLaunchKernelGGL(k_pk_counts, dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, seg, n_unique, counts);
        MTGR_LAUNCH_CHECK();
    }
    return EMB_OK;
}

} // extern "C"
