// Row movement and row arithmetic of the embedding path for gfx950: gather of table rows,
// expand by inverse index, deterministic gradient segment-reduce, row-wise Adagrad.
//
// All of it is HBM-bound.  A row is moved as 16-byte vectors by a sub-wave of LPR lanes
// (LPR = row bytes / 16 rounded up to a power of two), so one wave instruction covers 64/LPR
// whole rows with fully used 64..128-byte segments, and several rows are in flight per lane
// group before the first is consumed.
#include <cmath>

#include "common.hpp"

using namespace mtgr;

namespace {

constexpr int kBlock = 256;
constexpr int kUnroll = 8;            // segment reduce: rows a lane group fetches per batch at the first level
constexpr int kUnrollUpper = 8;       // ... and at the upper levels
constexpr int kUnrollFused = 8;       // fused backward, first level: each item also carries a table row and a record
constexpr int kPipeMax = 8;           // batches up to this size are double-buffered

__device__ inline const char* chunk_row_cptr(const HtView& v, uint32_t row) {
    const char* base = static_cast<const char*>(v.st->values[row >> v.chunk_log2]);
    return base + (size_t)(row & ((1u << v.chunk_log2) - 1u)) * (size_t)v.row_bytes;
}

// Base pointers of the value chunks and their row records, copied to LDS once per block: a row's address then
// depends on its index only, not on a load from the chunk directory in HBM (which would put a second memory
// round trip in front of every batch of row loads).
__device__ inline void stage_chunks(const HtView& v, char** s_values, RowMeta** s_meta) {
    const int nc = (int)(v.rows_capacity >> v.chunk_log2);
    for (int c = threadIdx.x; c < nc; c += kBlock) {
        s_values[c] = static_cast<char*>(v.st->values[c]);
        if (s_meta) s_meta[c] = v.st->meta[c];
    }
    __syncthreads();
}
__device__ inline char* staged_row(const HtView& v, char* const* s_values, uint32_t row) {
    return s_values[row >> v.chunk_log2] + (size_t)(row & ((1u << v.chunk_log2) - 1u)) * (size_t)v.row_bytes;
}
__device__ inline RowMeta* staged_meta(const HtView& v, RowMeta* const* s_meta, uint32_t row) {
    return s_meta[row >> v.chunk_log2] + (row & ((1u << v.chunk_log2) - 1u));
}

// Block order of a kernel whose main input is a matrix the previous kernel of the stream has just written
// front to back (the distinct rows for the expand, the reduced gradients for the update): the blocks walk it back
// to front.  The matrix is larger than the 256 MB memory-side cache, which at that moment holds its most recently
// written part - the end; read first, that part is served from the cache instead of HBM (expand of 9 M positions
// over 2.1 M rows of 256 bytes: 600 -> 575 us).  Returns -1 for a block beyond the count.
__device__ inline int64_t block_from_the_end(int64_t n, int per_block) {
    return (n + per_block - 1) / per_block - 1 - (int64_t)blockIdx.x;
}

// Cache hints.  Rows and indices that a kernel reads once (table rows in the gather and the update, gradient
// rows in the reduce, the sorted-order mapping) are loaded non-temporally, and rows nobody reads again soon (the
// expanded embeddings, the updated table rows) are stored non-temporally: they then do not displace what the next
// kernel of the step will read - the distinct rows between gather and expand, the reduced gradients between reduce
// and update - from the L2 and the memory-side cache.  Measured on the long-sequence step, all hints together:
// 2.38 -> 2.25 ms.  Two that were tried cost time: a non-temporal load of a row record that the same lane rewrites
// (update +65 us), and non-temporal loads of the distinct rows in the expand, where a row is read by about four
// neighbouring positions (+65 us).
//
// ---------------------------------------------------------------------------- gather / expand
// One wave owns 64 consecutive output rows; lane l reads index l once, the LPR-lane groups then
// take the rows in turn, kCopyUnroll rows in flight per group.  SRC_TABLE: source row = chunked
// table row (index -1 -> zeros); otherwise source row = base + index * row_bytes.
// FULL = all 64 rows present and every lane of a group carries a vector: no per-row branches,
// so the loads of one batch and the stores of the previous one stay in flight together.
constexpr int kCopyUnroll = 16;      // 256-byte rows: all 64 rows of a wave in one batch (8: expand 8 us slower; 4: 3 us slower)

template <int LPR, bool SRC_TABLE, bool NT_STORE, bool FULL, bool DST_IDX>
__device__ inline void copy_rows_body(const HtView& v, char* const* s_values, const char* __restrict__ src_base, int my_index,
                                      int my_dst, int rows_here, int vecs, int row_bytes, char* __restrict__ out_wave, int lane) {
    constexpr int kGroups = kWave / LPR;          // rows per wave instruction
    constexpr int kU = (kGroups * kCopyUnroll > kWave) ? (kWave / kGroups) : kCopyUnroll;
    const int sub = lane % LPR, grp = lane / LPR;
    const bool lane_on = FULL || sub < vecs;
#pragma unroll 1
    for (int r0 = 0; r0 < kWave; r0 += kGroups * kU) {
        if (!FULL && r0 >= rows_here) break;
        V16 val[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int r = r0 + u * kGroups + grp;
            const int idx = __shfl(my_index, r, kWave);
            const bool ok = lane_on && (FULL || r < rows_here);
            const int safe = idx < 0 ? 0 : idx;
            const char* p = SRC_TABLE ? staged_row(v, s_values, (uint32_t)safe) : src_base + (size_t)safe * (size_t)row_bytes;
            if (FULL) {
                val[u] = (SRC_TABLE && !DST_IDX) ? ld16_nt(p + sub * 16) : ld16(p + sub * 16);   // gather: a table row is read once
            } else {
                val[u] = V16{0u, 0u, 0u, 0u};
                if (ok) val[u] = ld16(p + sub * 16);
            }
            if (SRC_TABLE && idx < 0) val[u] = V16{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int r = r0 + u * kGroups + grp;
            // DST_IDX: out_wave is the matrix base and the row position comes from the second index
            const int64_t drow = DST_IDX ? (int64_t)__shfl(my_dst, r, kWave) : (int64_t)r;
            char* q = out_wave + (size_t)drow * (size_t)row_bytes + sub * 16;
            if (FULL) {
                if (NT_STORE) st16_nt(q, val[u]); else st16(q, val[u]);
            } else if (lane_on && r < rows_here) {
                if (NT_STORE) st16_nt(q, val[u]); else st16(q, val[u]);
            }
        }
    }
}

template <int LPR, bool SRC_TABLE, bool NT_STORE, bool DST_IDX>
__global__ __launch_bounds__(kBlock) void k_copy_rows(HtView v, const char* __restrict__ src_base,
                                                      const int32_t* __restrict__ index,
                                                      const int32_t* __restrict__ via,
                                                      const int32_t* __restrict__ dst_index, const int64_t* n_dev,
                                                      int64_t n_max, int row_bytes, char* __restrict__ out) {
    __shared__ char* s_values[SRC_TABLE ? kMaxChunks : 1];
    if (SRC_TABLE) stage_chunks(v, s_values, nullptr);
    const int64_t n = read_count(n_dev, n_max);
    const int lane = lane_id();
    // sorted expand: the source is the matrix of distinct rows the gather has just written
    const int64_t blk = DST_IDX ? block_from_the_end(n, kBlock) : (int64_t)blockIdx.x;
    if (blk < 0) return;
    const int64_t wave_base = blk * kBlock + (threadIdx.x & ~(kWave - 1));
    if (wave_base >= n) return;
    const int vecs = row_bytes / 16;
    int my_index = (wave_base + lane < n) ? (DST_IDX ? __builtin_nontemporal_load(&index[wave_base + lane]) : index[wave_base + lane]) : -1;
    if (via && my_index >= 0) my_index = via[my_index]; // source row = via[index[j]] (fused gather + expand)
    const int my_dst = (DST_IDX && wave_base + lane < n) ? __builtin_nontemporal_load(&dst_index[wave_base + lane]) : 0;
    const int rows_here = (int)((n - wave_base) < kWave ? (n - wave_base) : kWave);
    char* out_wave = DST_IDX ? out : out + (size_t)wave_base * (size_t)row_bytes;
    if (rows_here == kWave && vecs == LPR)
        copy_rows_body<LPR, SRC_TABLE, NT_STORE, true, DST_IDX>(v, s_values, src_base, my_index, my_dst, rows_here, vecs,
                                                                row_bytes, out_wave, lane);
    else
        copy_rows_body<LPR, SRC_TABLE, NT_STORE, false, DST_IDX>(v, s_values, src_base, my_index, my_dst, rows_here, vecs,
                                                                 row_bytes, out_wave, lane);
}

template <bool SRC_TABLE, bool NT, bool DST_IDX>
int launch_copy_rows(const HtView& v, const char* src, const int32_t* index, const int32_t* via, const int32_t* dst_index,
                     const int64_t* n_dev, int64_t n_max, int row_bytes, char* out, hipStream_t s) {
    const int vecs = row_bytes / 16;
    const unsigned grid = (unsigned)((n_max + kBlock - 1) / kBlock);
#define MTGR_CASE(L)                                                                                              \
    hipLaunchKernelGGL((k_copy_rows<L, SRC_TABLE, NT, DST_IDX>), dim3(grid), dim3(kBlock), 0, s, v, src, index, via,      \
                       dst_index, n_dev, n_max, row_bytes, out)
    if (vecs <= 1) MTGR_CASE(1);
    else if (vecs <= 2) MTGR_CASE(2);
    else if (vecs <= 4) MTGR_CASE(4);
    else if (vecs <= 8) MTGR_CASE(8);
    else if (vecs <= 16) MTGR_CASE(16);
    else if (vecs <= 32) MTGR_CASE(32);
    else MTGR_CASE(64);
#undef MTGR_CASE
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

// ---------------------------------------------------------------------------- segment reduce
// Items are reduced in a fixed order, level by level.  Level 1 items are the positions in sorted
// order (row = grad[perm[j]], segment = seg_of[j]); a group of LPR lanes folds kSpan
// consecutive items.  Runs of one segment that lie strictly inside the span are complete and
// stored to reduced[]; the first and the last run of the span may continue in a neighbour span,
// so they are handed to the next level as two fp32 partial rows (segment -1 = no item).  The next
// level folds kSpan of those, and so on until one span holds everything.  Every sum is a fixed
// tree, so results are reproducible run to run.  Span length trades partial-row traffic (two
// fp32 rows per span) against parallelism; 64 measured best on the long-sequence workload
// (0.67 ms against 0.72 ms at 128 and 0.84 ms at 256 for 8.7 M rows of 256 bytes).
constexpr int kSpan = 64;

// FPL = floats accumulated per lane (4 for fp32 rows of 16 bytes per lane, 8 for bf16)
template <int FPL>
struct Acc {
    float f[FPL];
    __device__ inline void zero() {
#pragma unroll
        for (int i = 0; i < FPL; ++i) f[i] = 0.0f;
    }
};
__device__ inline void acc_add(Acc<4>& a, const V16& v, bool /*bf16*/) {
    a.f[0] += __uint_as_float(v.x);
    a.f[1] += __uint_as_float(v.y);
    a.f[2] += __uint_as_float(v.z);
    a.f[3] += __uint_as_float(v.w);
}
__device__ inline void acc_add(Acc<8>& a, const V16& v, bool) {
    a.f[0] += bf16lo(v.x); a.f[1] += bf16hi(v.x);
    a.f[2] += bf16lo(v.y); a.f[3] += bf16hi(v.y);
    a.f[4] += bf16lo(v.z); a.f[5] += bf16hi(v.z);
    a.f[6] += bf16lo(v.w); a.f[7] += bf16hi(v.w);
}
template <int FPL>
__device__ inline void acc_store(float* row, int sub, const Acc<FPL>& a) {
    // lane `sub` owns floats [sub*FPL, sub*FPL+FPL) of the row
#pragma unroll
    for (int q = 0; q < FPL / 4; ++q) {
        V16 o{__float_as_uint(a.f[4 * q]), __float_as_uint(a.f[4 * q + 1]), __float_as_uint(a.f[4 * q + 2]),
              __float_as_uint(a.f[4 * q + 3])};
        st16(row + sub * FPL + 4 * q, o);
    }
}

// Row-wise Adagrad arithmetic, spelled with explicit roundings so that every kernel that applies
// it produces the same bits: acc' = fma(ss, 1/D, acc); scale = lr / (sqrt(acc') + eps);
// w' = fma(-scale, g, w).
__device__ inline float adagrad_acc(float acc_old, float ss, float inv_d) { return __fmaf_rn(ss, inv_d, acc_old); }
__device__ inline float adagrad_scale(float acc_new, float lr, float eps) {
    return __fdiv_rn(lr, __fadd_rn(__fsqrt_rn(acc_new), eps));
}
__device__ inline float adagrad_w(float w, float g, float scale) { return __fmaf_rn(-scale, g, w); }
// Sum of squares of a row in a fixed tree that does not depend on how many elements a lane holds:
// fma chains over aligned quads of elements, then pairwise sums of neighbouring quads, octets, ...
// (in-lane first, then xor-shuffles with growing distance).
template <int N>
__device__ inline float sumsq_lane(const float* g) {
    float q[N / 4];
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
        float s = 0.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) s = __fmaf_rn(g[4 * i + e], g[4 * i + e], s);
        q[i] = s;
    }
#pragma unroll
    for (int w = 1; w < N / 4; w <<= 1)
#pragma unroll
        for (int i = 0; i + w < N / 4; i += 2 * w) q[i] = __fadd_rn(q[i], q[i + w]);
    return q[0];
}
template <int LPR>
__device__ inline float sumsq_group(float ss) {
#pragma unroll
    for (int o = 1; o < LPR; o <<= 1) ss = __fadd_rn(ss, __shfl_xor(ss, o, kWave));
    return ss;
}

struct LevelIn {
    const char* rows;        // level 1: grad matrix; level >= 2: fp32 partial rows
    const int32_t* perm;     // level 1 only: source row of item j is perm[j] ...
    const int32_t* via;      // ... or via[perm[j]] when given (pooled gradients: position -> bag)
    const int32_t* seg;      // segment of each item in order (-1 = no item)
    int64_t n_items;
    int in_row_bytes;
};

// UNR = rows a group fetches per batch, the next batch being fetched while the current one is
// folded: 4 at the large first level, 8 at the small upper levels, which are chains of dependent
// round trips (their stores would otherwise sit between a batch's loads and their use).
template <int LPR, int FPL, bool LEVEL1, int UNR>
__global__ __launch_bounds__(kBlock) void k_seg_reduce(LevelIn in, int dim, float* __restrict__ reduced,
                                                       float* __restrict__ part_rows, int32_t* __restrict__ part_seg,
                                                       int last_level) {
    constexpr int kGroups = kWave / LPR;
    // fp32 gradient rows are loaded non-temporally (long-sequence step: reduce -36 us, whole step -17 us); for bf16
    // gradients, whose fp32 sums are twice the size of the rows read, the hint showed no gain (large configuration,
    // whose step times spread by 0.1 ms from run to run) and is left off
    constexpr bool kNtGrad = LEVEL1 && FPL == 4;
    const int lane = lane_id();
    const int sub = lane % LPR, grp = lane / LPR;
    const int gbase = lane - sub;
    const int64_t span = ((int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave) * kGroups + grp;
    const int64_t first = span * kSpan;
    const bool group_on = first < in.n_items;
    const int vecs = in.in_row_bytes / 16;
    const bool lane_on = group_on && sub < vecs;
    const int items = group_on ? (int)((in.n_items - first) < kSpan ? (in.n_items - first) : kSpan) : 0;

    Acc<FPL> acc;
    acc.zero();
    int cur_seg = -1;
    int runs_closed = 0;     // runs already flushed in this span
    bool have = false;

    // flush the current run: first run of the span -> partial slot 0, otherwise complete -> reduced[]
    auto flush_mid = [&](void) {
        if (!have) return;
        if (runs_closed == 0 && !last_level) {
            if (lane_on) acc_store<FPL>(part_rows + (size_t)(2 * span) * dim, sub, acc);
            if (sub == 0) part_seg[2 * span] = cur_seg;
        } else {
            if (lane_on) acc_store<FPL>(reduced + (size_t)cur_seg * dim, sub, acc);
        }
        runs_closed++;
        acc.zero();
        have = false;
    };

    // each lane of the group preloads the source row index / segment of items sub, sub+LPR, ...
    constexpr int kPre = (kSpan / LPR) < 1 ? 1 : ((kSpan / LPR) > 4 ? 4 : (kSpan / LPR)); // items a lane holds per chunk
    constexpr int kChunk = LPR * kPre;                        // items per chunk (flat index f = u*LPR + lane-in-group)
    constexpr int kBatches = (kChunk + UNR - 1) / UNR;
    for (int c = 0; c < kSpan; c += kChunk) {
        int my_src[kPre];          // source row of the item (< 2^31)
        int my_seg[kPre];
#pragma unroll
        for (int u = 0; u < kPre; ++u) {
            const int it = c + u * LPR + sub;
            my_src[u] = -1;
            my_seg[u] = -1;
            if (group_on && it < items) {
                const int64_t j = first + it;
                if (LEVEL1) {
                    const int32_t p = __builtin_nontemporal_load(&in.perm[j]);
                    my_src[u] = in.via ? in.via[p] : p;
                } else {
                    my_src[u] = (int)j;
                }
                my_seg[u] = (LEVEL1 ? __builtin_nontemporal_load(&in.seg[j]) : in.seg[j]);
            }
        }
        // batch b fetches the rows of flat items b*UNR .. b*UNR+UNR-1 of the chunk
        auto issue = [&](int b, V16* v_, int* sg_) {
#pragma unroll
            for (int k = 0; k < UNR; ++k) {
                const int f = b * UNR + k;
                sg_[k] = -1;
                v_[k] = V16{0u, 0u, 0u, 0u};
                if (f < kChunk) {
                    const int sl = gbase + f % LPR;
                    const int src = __shfl(my_src[f / LPR], sl, kWave);
                    sg_[k] = __shfl(my_seg[f / LPR], sl, kWave);
                    // The load must not sit behind a branch: with a data-dependent number of loads in flight the wait
                    // before a fold is for all of them, the next batch's included, and the double buffer is void.  A lane
                    // without a row reads the first 16 bytes of the matrix instead and masks them out; the mask is made
                    // opaque to the compiler, which otherwise puts the branch back.
                    const bool on = lane_on && sg_[k] >= 0;
                    uint32_t keep = on ? 0xFFFFFFFFu : 0u;
                    asm("" : "+v"(keep));
                    const V16 t = (kNtGrad ? ld16_nt : ld16)(in.rows + (on ? (size_t)src * (size_t)in.in_row_bytes + sub * 16 : (size_t)0));
                    v_[k] = V16{t.x & keep, t.y & keep, t.z & keep, t.w & keep};
                }
            }
        };
        auto fold = [&](const V16* v_, const int* sg_) {
#pragma unroll
            for (int k = 0; k < UNR; ++k) {
                if (sg_[k] < 0) continue;
                if (have && sg_[k] != cur_seg) flush_mid();
                cur_seg = sg_[k];
                have = true;
                acc_add(acc, v_[k], false);
            }
        };
        if constexpr (UNR <= kPipeMax) {
            // the loads of batch b+1 are issued before batch b is folded, so that a wave always has loads in flight
            V16 val[2][UNR];
            int seg[2][UNR];
            issue(0, val[0], seg[0]);
#pragma unroll
            for (int b = 0; b < kBatches; ++b) {
                if (b + 1 < kBatches) issue(b + 1, val[(b + 1) & 1], seg[(b + 1) & 1]);
                fold(val[b & 1], seg[b & 1]);
            }
        } else {
            V16 val[UNR];
            int seg[UNR];
#pragma unroll
            for (int b = 0; b < kBatches; ++b) {
                issue(b, val, seg);
                fold(val, seg);
            }
        }
    }
    // last run of the span
    if (group_on) {
        if (last_level) {
            if (have && lane_on) acc_store<FPL>(reduced + (size_t)cur_seg * dim, sub, acc);
        } else {
            // a span with a single run has already nothing in slot 0: put the run there, slot 1 empty
            const int slot = (runs_closed == 0) ? 0 : 1;
            if (have && lane_on) acc_store<FPL>(part_rows + (size_t)(2 * span + slot) * dim, sub, acc);
            if (sub == 0) {
                part_seg[2 * span + slot] = have ? cur_seg : -1;
                if (slot == 0) part_seg[2 * span + 1] = -1;
            }
        }
    }
}

// ---------------------------------------------------------------------------- segment reduce + update in one pass
// Same spans, same order of additions and the same partial rows as k_seg_reduce, but a run that
// completes inside a span goes straight into the row-wise Adagrad update of row row_idx[segment]
// instead of the reduced matrix.  Which items end such a run is known as soon as the span's segment
// numbers are (they are loaded first), so the table row and the row record a completed sum will need
// are fetched together with the gradient rows of its batch, one batch ahead of their use: the update
// never waits on a load of its own.  The base pointers of the value chunks are staged in LDS, so no
// address depends on a load from the chunk directory in HBM.
struct FuseArgs {
    HtView v;
    const int32_t* row_idx;   // row of every segment (-1 = none)
    float lr, eps;
    uint32_t step;
    int touch;                // also set last_seen = step and count one touch
    int n_chunks;
};

template <int LPR, int FPL, bool LEVEL1, int UNR, bool TBL_BF16>
__global__ __launch_bounds__(kBlock) void k_seg_reduce_apply(LevelIn in, int dim, float* __restrict__ part_rows,
                                                             int32_t* __restrict__ part_seg, int last_level, FuseArgs fz) {
    __shared__ char* s_values[kMaxChunks];
    __shared__ RowMeta* s_meta[kMaxChunks];
    for (int c = threadIdx.x; c < fz.n_chunks; c += kBlock) {
        s_values[c] = static_cast<char*>(fz.v.st->values[c]);
        s_meta[c] = fz.v.st->meta[c];
    }
    __syncthreads();
    constexpr int kGroups = kWave / LPR;
    constexpr bool kNtGrad = LEVEL1 && FPL == 4;    // as in k_seg_reduce
    constexpr int kWB = FPL * (TBL_BF16 ? 2 : 4);   // bytes of the table row a lane owns (16, or 8 for bf16 rows at upper levels)
    const int lane = lane_id();
    const int sub = lane % LPR, grp = lane / LPR;
    const int gbase = lane - sub;
    const int64_t span = ((int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave) * kGroups + grp;
    const int64_t first = span * kSpan;
    const bool group_on = first < in.n_items;
    const int vecs = in.in_row_bytes / 16;
    const bool lane_on = group_on && sub < vecs;
    const int items = group_on ? (int)((in.n_items - first) < kSpan ? (in.n_items - first) : kSpan) : 0;
    const uint32_t chunk_mask = (1u << fz.v.chunk_log2) - 1u;
    const float inv_d = __fdiv_rn(1.0f, (float)dim);

    Acc<FPL> acc;
    acc.zero();
    int cur_seg = -1;
    int runs_closed = 0;
    bool have = false;

    // the run in `acc` is complete and its row (w_) and record (rec_) are here: update the row
    auto apply = [&](int row, const V16& w_, const V16& rec_) {
        const float ss = sumsq_group<LPR>(sumsq_lane<FPL>(acc.f));
        const uint32_t rec_acc = __shfl(rec_.x, gbase, kWave), rec_freq = __shfl(rec_.z, gbase, kWave),
                       rec_hot = __shfl(rec_.w, gbase, kWave);
        if (row >= 0) {
            const float acc_new = adagrad_acc(__uint_as_float(rec_acc), ss, inv_d);
            const float scale = adagrad_scale(acc_new, fz.lr, fz.eps);
            const uint32_t r = (uint32_t)row;
            if (lane_on) {
                char* wp = s_values[r >> fz.v.chunk_log2] + (size_t)(r & chunk_mask) * (size_t)fz.v.row_bytes + sub * kWB;
                if (!TBL_BF16) {
                    stg16_nt(wp, V16{__float_as_uint(adagrad_w(__uint_as_float(w_.x), acc.f[0], scale)),
                                 __float_as_uint(adagrad_w(__uint_as_float(w_.y), acc.f[1], scale)),
                                 __float_as_uint(adagrad_w(__uint_as_float(w_.z), acc.f[2], scale)),
                                 __float_as_uint(adagrad_w(__uint_as_float(w_.w), acc.f[3], scale))});
                } else {
                    const uint32_t o0 = pack_bf16(adagrad_w(bf16lo(w_.x), acc.f[0], scale), adagrad_w(bf16hi(w_.x), acc.f[1], scale));
                    const uint32_t o1 = pack_bf16(adagrad_w(bf16lo(w_.y), acc.f[2], scale), adagrad_w(bf16hi(w_.y), acc.f[3], scale));
                    if constexpr (FPL == 8) {
                        const uint32_t o2 = pack_bf16(adagrad_w(bf16lo(w_.z), acc.f[4], scale), adagrad_w(bf16hi(w_.z), acc.f[5], scale));
                        const uint32_t o3 = pack_bf16(adagrad_w(bf16lo(w_.w), acc.f[6], scale), adagrad_w(bf16hi(w_.w), acc.f[7], scale));
                        stg16_nt(wp, V16{o0, o1, o2, o3});
                    } else {
                        MTGR_AS_GLOBAL uint32_t* q = (MTGR_AS_GLOBAL uint32_t*)wp;
                        q[0] = o0;
                        q[1] = o1;
                    }
                }
            }
            if (sub == 0) {
                RowMeta* m = s_meta[r >> fz.v.chunk_log2] + (r & chunk_mask);
                if (fz.touch) stg16(m, V16{__float_as_uint(acc_new), fz.step, rec_freq + 1u, rec_hot});
                else ((MTGR_AS_GLOBAL RowMeta*)m)->acc = acc_new;
            }
        }
        runs_closed++;
        acc.zero();
        have = false;
    };

    constexpr int kPre = (kSpan / LPR) < 1 ? 1 : ((kSpan / LPR) > 4 ? 4 : (kSpan / LPR));
    constexpr int kChunk = LPR * kPre;
    constexpr int kBatches = (kChunk + UNR - 1) / UNR;
    // segment of the first item of the span: its run continues from the span before (unless this is the last level)
    int seg_first = -1;
    if (group_on) seg_first = in.seg[first];
    for (int c = 0; c < kSpan; c += kChunk) {
        int my_src[kPre], my_seg[kPre], my_row[kPre], my_next[kPre];
#pragma unroll
        for (int u = 0; u < kPre; ++u) {
            const int it = c + u * LPR + sub;
            my_src[u] = -1;
            my_seg[u] = -1;
            my_row[u] = -1;
            my_next[u] = -2;       // segment of the item after this one (-2: there is none in this span)
            if (group_on && it < items) {
                const int64_t j = first + it;
                if (LEVEL1) {
                    const int32_t p = __builtin_nontemporal_load(&in.perm[j]);
                    my_src[u] = in.via ? in.via[p] : p;
                } else {
                    my_src[u] = (int)j;
                }
                my_seg[u] = in.seg[j];
                // segment of the next item; at the upper levels the second slot of a span may be empty (-1) and
                // the run goes on with the first slot of the span after it, which never is
                if (it + 1 < items) {
                    int nx = in.seg[j + 1];
                    if (!LEVEL1 && nx < 0) nx = it + 2 < items ? in.seg[j + 2] : -2;
                    my_next[u] = nx;
                }
            }
        }
        // does item (u, lane) end a run that is applied here?  Not the run that came in from the span before,
        // not the run that goes on into the next span (both travel to the next level as partial rows), unless
        // this is the last level, where every run ends here.  Segment -1 = no item (upper levels).
#pragma unroll
        for (int u = 0; u < kPre; ++u) {
            const bool ends = my_seg[u] >= 0 && my_next[u] != my_seg[u];
            const bool applied = last_level ? ends : (ends && my_next[u] != -2 && my_seg[u] != seg_first);
            my_row[u] = applied ? fz.row_idx[my_seg[u]] : -2;     // -2: nothing to apply at this item; -1: segment without a row
        }
        // element `idx` of a small per-lane array without dynamic register indexing
        auto pick = [&](const int* arr, int idx) {
            int r = arr[0];
#pragma unroll
            for (int u = 1; u < kPre; ++u) r = idx == u ? arr[u] : r;
            return r;
        };
        auto issue = [&](int b, V16* v_, int* sg_, int* rw_, V16* w_, V16* rec_) {
#pragma unroll
            for (int k = 0; k < UNR; ++k) {
                const int f = b * UNR + k;
                sg_[k] = -1;
                rw_[k] = -2;
                v_[k] = V16{0u, 0u, 0u, 0u};
                w_[k] = V16{0u, 0u, 0u, 0u};
                rec_[k] = V16{0u, 0u, 0u, 0u};
                if (f < kChunk) {
                    const int sl = gbase + f % LPR;
                    const int u = f / LPR;
                    const int src = __shfl(pick(my_src, u), sl, kWave);
                    sg_[k] = __shfl(pick(my_seg, u), sl, kWave);
                    rw_[k] = __shfl(pick(my_row, u), sl, kWave);
                    // every load unconditional and a plain global load, as in k_seg_reduce and k_adagrad: an item
                    // without a gradient row reads the matrix's first bytes, one that ends no run here reads row 0 and
                    // its record (cache hits), and opaque masks drop what was read
                    const bool on = lane_on && sg_[k] >= 0;
                    const bool ron = rw_[k] >= 0;
                    uint32_t keep = on ? 0xFFFFFFFFu : 0u, keep_r = ron ? 0xFFFFFFFFu : 0u;
                    asm("" : "+v"(keep), "+v"(keep_r));
                    const V16 t = (kNtGrad ? ld16_nt : ld16)(in.rows + (on ? (size_t)src * (size_t)in.in_row_bytes + sub * 16 : (size_t)0));
                    v_[k] = V16{t.x & keep, t.y & keep, t.z & keep, t.w & keep};
                    const uint32_t r = ron ? (uint32_t)rw_[k] : 0u;
                    const char* wp = s_values[r >> fz.v.chunk_log2] + (size_t)(r & chunk_mask) * (size_t)fz.v.row_bytes + (lane_on ? sub * kWB : 0);
                    V16 wt{0u, 0u, 0u, 0u};
                    if (kWB == 16) wt = ldg16_nt(wp);
                    else {
                        const MTGR_AS_GLOBAL uint32_t* q = (const MTGR_AS_GLOBAL uint32_t*)wp;
                        wt.x = q[0];
                        wt.y = q[1];
                    }
                    w_[k] = V16{wt.x & keep_r, wt.y & keep_r, wt.z & keep_r, wt.w & keep_r};
                    const V16 rt = ldg16(s_meta[r >> fz.v.chunk_log2] + (r & chunk_mask));
                    rec_[k] = V16{rt.x & keep_r, rt.y & keep_r, rt.z & keep_r, rt.w & keep_r};
                }
            }
        };
        auto fold = [&](const V16* v_, const int* sg_, const int* rw_, const V16* w_, const V16* rec_) {
#pragma unroll
            for (int k = 0; k < UNR; ++k) {
                if (sg_[k] < 0) continue;
                if (have && sg_[k] != cur_seg) {
                    // the run that came in from the span before ends here: partial slot 0
                    if (lane_on) acc_store<FPL>(part_rows + (size_t)(2 * span) * dim, sub, acc);
                    if (sub == 0) part_seg[2 * span] = cur_seg;
                    runs_closed++;
                    acc.zero();
                }
                cur_seg = sg_[k];
                have = true;
                acc_add(acc, v_[k], false);
                if (rw_[k] != -2) apply(rw_[k], w_[k], rec_[k]);
            }
        };
        if constexpr (UNR <= 4 && FPL == 4) {
            // two named buffers, two batches per trip: the loads of the next batch are issued before the current
            // one is folded, and no buffer is ever indexed by a run-time value
            V16 val_a[UNR], wv_a[UNR], rec_a[UNR], val_b[UNR], wv_b[UNR], rec_b[UNR];
            int seg_a[UNR], rw_a[UNR], seg_b[UNR], rw_b[UNR];
            issue(0, val_a, seg_a, rw_a, wv_a, rec_a);
#pragma unroll 1
            for (int b = 0; b < kBatches; b += 2) {
                if (b + 1 < kBatches) issue(b + 1, val_b, seg_b, rw_b, wv_b, rec_b);
                fold(val_a, seg_a, rw_a, wv_a, rec_a);
                if (b + 2 < kBatches) issue(b + 2, val_a, seg_a, rw_a, wv_a, rec_a);
                if (b + 1 < kBatches) fold(val_b, seg_b, rw_b, wv_b, rec_b);
            }
        } else {
            V16 val[UNR], wv[UNR], rec[UNR];
            int seg[UNR], rw[UNR];
#pragma unroll 1
            for (int b = 0; b < kBatches; ++b) {
                issue(b, val, seg, rw, wv, rec);
                fold(val, seg, rw, wv, rec);
            }
        }
    }
    // the run that goes on into the next span (at the last level every run has been applied above)
    if (group_on && !last_level) {
        const int slot = (runs_closed == 0) ? 0 : 1;
        if (have && lane_on) acc_store<FPL>(part_rows + (size_t)(2 * span + slot) * dim, sub, acc);
        if (sub == 0) {
            part_seg[2 * span + slot] = have ? cur_seg : -1;
            if (slot == 0) part_seg[2 * span + 1] = -1;
        }
    }
}

struct ReduceLayout {
    int levels;
    int64_t items[8];       // items entering level l (l = 0 is level 1)
    int64_t spans[8];
    size_t rows_off[8];     // partial rows written by level l
    size_t seg_off[8];
    size_t total;
};
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
ReduceLayout reduce_layout(int64_t n, int dim) {
    ReduceLayout L;
    size_t o = 0;
    int64_t items = n;
    int l = 0;
    for (;; ++l) {
        const int64_t spans = (items + kSpan - 1) / kSpan;
        L.items[l] = items;
        L.spans[l] = spans;
        L.rows_off[l] = o; o = align256(o + (size_t)(2 * spans) * dim * 4);
        L.seg_off[l] = o; o = align256(o + (size_t)(2 * spans) * 4);
        if (spans <= 1 || l == 7) { ++l; break; }
        items = 2 * spans;
    }
    L.levels = l;
    L.total = o;
    return L;
}

template <int LPR, int FPL>
int launch_reduce(const char* grad, int in_row_bytes, const int32_t* seg_of, const int32_t* perm, const int32_t* via,
                  int64_t n, int dim, float* reduced, char* ws, const ReduceLayout& L, hipStream_t s) {
    constexpr int kGroups = kWave / LPR;
    constexpr int kSpansPerBlock = (kBlock / kWave) * kGroups;
    for (int l = 0; l < L.levels; ++l) {
        const int last = (l == L.levels - 1) ? 1 : 0;
        const unsigned grid = (unsigned)((L.spans[l] + kSpansPerBlock - 1) / kSpansPerBlock);
        float* prow = reinterpret_cast<float*>(ws + L.rows_off[l]);
        int32_t* pseg = reinterpret_cast<int32_t*>(ws + L.seg_off[l]);
        if (l == 0) {
            LevelIn in{grad, perm, via, seg_of, n, in_row_bytes};
            hipLaunchKernelGGL((k_seg_reduce<LPR, FPL, true, kUnroll>), dim3(grid), dim3(kBlock), 0, s, in, dim, reduced, prow, pseg, last);
        } else {
            LevelIn in{ws + L.rows_off[l - 1], nullptr, nullptr, reinterpret_cast<const int32_t*>(ws + L.seg_off[l - 1]),
                       L.items[l], dim * 4};
            // partial rows are fp32: dim*4 bytes, dim/4 vectors per row
            constexpr int LPR2 = (FPL == 8) ? (LPR * 2 > 64 ? 64 : LPR * 2) : LPR;
            constexpr int kGroups2 = kWave / LPR2;
            constexpr int kSpb2 = (kBlock / kWave) * kGroups2;
            const unsigned grid2 = (unsigned)((L.spans[l] + kSpb2 - 1) / kSpb2);
            hipLaunchKernelGGL((k_seg_reduce<LPR2, 4, false, kUnrollUpper>), dim3(grid2), dim3(kBlock), 0, s, in, dim, reduced, prow, pseg, last);
        }
        MTGR_LAUNCH_CHECK();
    }
    return EMB_OK;
}

// the same levels with k_seg_reduce_apply; gradients come in the table dtype (FPL = 8: bf16 table)
template <int LPR, int FPL>
int launch_reduce_apply(const char* grad, int in_row_bytes, const int32_t* seg_of, const int32_t* perm, int64_t n, int dim,
                        char* ws, const ReduceLayout& L, hipStream_t s, const FuseArgs& fz) {
    constexpr bool kTblBf16 = FPL == 8;
    constexpr int kGroups = kWave / LPR;
    constexpr int kSpansPerBlock = (kBlock / kWave) * kGroups;
    for (int l = 0; l < L.levels; ++l) {
        const int last = (l == L.levels - 1) ? 1 : 0;
        const unsigned grid = (unsigned)((L.spans[l] + kSpansPerBlock - 1) / kSpansPerBlock);
        float* prow = reinterpret_cast<float*>(ws + L.rows_off[l]);
        int32_t* pseg = reinterpret_cast<int32_t*>(ws + L.seg_off[l]);
        if (l == 0) {
            LevelIn in{grad, perm, nullptr, seg_of, n, in_row_bytes};
            hipLaunchKernelGGL((k_seg_reduce_apply<LPR, FPL, true, kUnrollFused, kTblBf16>), dim3(grid), dim3(kBlock), 0, s, in, dim, prow, pseg, last, fz);
        } else {
            LevelIn in{ws + L.rows_off[l - 1], nullptr, nullptr, reinterpret_cast<const int32_t*>(ws + L.seg_off[l - 1]),
                       L.items[l], dim * 4};
            constexpr int LPR2 = (FPL == 8) ? (LPR * 2 > 64 ? 64 : LPR * 2) : LPR;
            constexpr int kGroups2 = kWave / LPR2;
            constexpr int kSpb2 = (kBlock / kWave) * kGroups2;
            const unsigned grid2 = (unsigned)((L.spans[l] + kSpb2 - 1) / kSpb2);
            hipLaunchKernelGGL((k_seg_reduce_apply<LPR2, 4, false, kUnrollUpper, kTblBf16>), dim3(grid2), dim3(kBlock), 0, s, in, dim, prow, pseg, last, fz);
        }
        MTGR_LAUNCH_CHECK();
    }
    return EMB_OK;
}

// ---------------------------------------------------------------------------- row-wise Adagrad
// One wave owns 64 consecutive entries of row_idx; an LPR-lane group updates one row:
// sum of squares by xor-shuffles inside the group, then w -= lr * g / (sqrt(acc) + eps).
// TOUCH: the row record is rewritten whole - new accumulator, last_seen = step, touch count + 1 -
// so that a training step updates the record once instead of once per lookup and once per update
// (a random 16-byte record costs a read-modify-write in memory either way).
template <int LPR, bool BF16, bool TOUCH>
__global__ __launch_bounds__(kBlock) void k_adagrad(HtView v, const int32_t* __restrict__ row_idx,
                                                    const float* __restrict__ g, const int64_t* n_dev, int64_t n_max,
                                                    float lr, float eps, uint32_t step) {
    __shared__ char* s_values[kMaxChunks];
    __shared__ RowMeta* s_meta[kMaxChunks];
    stage_chunks(v, s_values, s_meta);
    const int64_t n = read_count(n_dev, n_max);
    const int lane = lane_id();
    const int64_t blk = block_from_the_end(n, kBlock);     // the reduced gradients have just been written
    if (blk < 0) return;
    const int64_t wave_base = blk * kBlock + (threadIdx.x & ~(kWave - 1));
    if (wave_base >= n) return;
    constexpr int kGroups = kWave / LPR;
    constexpr int kF = BF16 ? 8 : 4;              // elements per lane
    const int sub = lane % LPR, grp = lane / LPR;
    const bool lane_on = sub * kF < v.dim;
    const int my_index = (wave_base + lane < n) ? row_idx[wave_base + lane] : -1;
    const int rows_here = (int)((n - wave_base) < kWave ? (n - wave_base) : kWave);
    const float inv_d = __fdiv_rn(1.0f, (float)v.dim);
    constexpr int kRows = 4;                      // rows in flight per group (2: 4 us slower; 1: 10 us slower)
#pragma unroll 1
    for (int r0 = 0; r0 < kWave; r0 += kGroups * kRows) {
        if (r0 >= rows_here) break;
        float gv[kRows][kF];
        V16 wv[kRows];
        int idx[kRows];
        bool on[kRows];
        float acc_old[kRows];
        uint32_t freq_old[kRows], hot_old[kRows];
        // all loads of the batch go out before anything waits: gradient row, weight row and the row's record (its
        // own cache line) are independent.  None sits behind a branch and all are plain global loads, or the
        // compiler waits after each: an entry without a row reads row 0 and the wave's first gradient row instead and
        // masks them out (the mask is opaque to the compiler, which would otherwise put the branch back).
        V16 gq[kRows][kF / 4], rec[kRows];
        uint32_t keep[kRows];
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
            const int r = r0 + u * kGroups + grp;
            idx[u] = __shfl(my_index, r & (kWave - 1), kWave);
            on[u] = r < rows_here && idx[u] >= 0;
            keep[u] = on[u] ? 0xFFFFFFFFu : 0u;
            asm("" : "+v"(keep[u]));
            const uint32_t row = on[u] ? (uint32_t)idx[u] : 0u;
            const RowMeta* m = staged_meta(v, s_meta, row);
            rec[u] = TOUCH ? ldg16(m) : V16{__float_as_uint(((const MTGR_AS_GLOBAL RowMeta*)m)->acc), 0u, 0u, 0u};
            const float* gp = g + (size_t)(wave_base + (on[u] ? r : 0)) * v.dim + (lane_on ? sub * kF : 0);
#pragma unroll
            for (int q = 0; q < kF / 4; ++q) gq[u][q] = ld16_nt(gp + 4 * q);
            wv[u] = ldg16_nt(staged_row(v, s_values, row) + (lane_on ? sub * 16 : 0));
        }
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
            const uint32_t k = lane_on ? keep[u] : 0u;
#pragma unroll
            for (int q = 0; q < kF / 4; ++q) {
                gv[u][4 * q] = __uint_as_float(gq[u][q].x & k);
                gv[u][4 * q + 1] = __uint_as_float(gq[u][q].y & k);
                gv[u][4 * q + 2] = __uint_as_float(gq[u][q].z & k);
                gv[u][4 * q + 3] = __uint_as_float(gq[u][q].w & k);
            }
            wv[u] = V16{wv[u].x & k, wv[u].y & k, wv[u].z & k, wv[u].w & k};
            acc_old[u] = __uint_as_float(rec[u].x & keep[u]);
            freq_old[u] = rec[u].z & keep[u];
            hot_old[u] = rec[u].w & keep[u];
        }
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
            const float ss = sumsq_group<LPR>(sumsq_lane<kF>(gv[u]));
            if (!on[u]) continue;
            const uint32_t row = (uint32_t)idx[u];
            const float acc = adagrad_acc(acc_old[u], ss, inv_d);
            const float scale = adagrad_scale(acc, lr, eps);
            if (lane_on) {
                char* wp = staged_row(v, s_values, row) + sub * 16;
                V16 o;
                if (BF16) {
                    o.x = pack_bf16(adagrad_w(bf16lo(wv[u].x), gv[u][0], scale), adagrad_w(bf16hi(wv[u].x), gv[u][1], scale));
                    o.y = pack_bf16(adagrad_w(bf16lo(wv[u].y), gv[u][2], scale), adagrad_w(bf16hi(wv[u].y), gv[u][3], scale));
                    o.z = pack_bf16(adagrad_w(bf16lo(wv[u].z), gv[u][4], scale), adagrad_w(bf16hi(wv[u].z), gv[u][5], scale));
                    o.w = pack_bf16(adagrad_w(bf16lo(wv[u].w), gv[u][6], scale), adagrad_w(bf16hi(wv[u].w), gv[u][7], scale));
                } else {
                    o.x = __float_as_uint(adagrad_w(__uint_as_float(wv[u].x), gv[u][0], scale));
                    o.y = __float_as_uint(adagrad_w(__uint_as_float(wv[u].y), gv[u][1], scale));
                    o.z = __float_as_uint(adagrad_w(__uint_as_float(wv[u].z), gv[u][2], scale));
                    o.w = __float_as_uint(adagrad_w(__uint_as_float(wv[u].w), gv[u][3], scale));
                }
                stg16_nt(wp, o);
            }
            if (sub == 0) {
                RowMeta* m = staged_meta(v, s_meta, row);
                if (TOUCH) stg16(m, V16{__float_as_uint(acc), step, freq_old[u] + 1u, hot_old[u]});
                else ((MTGR_AS_GLOBAL RowMeta*)m)->acc = acc;
            }
        }
    }
}

// ---------------------------------------------------------------------------- hot / cold rows (App. C "Mixed Precision Training")
// A 16-bit table may keep an fp32 master copy of its frequently used rows in a separate hot
// store (RowMeta::hot = index + 1).  Lookups deliver every row in the table dtype (hot rows
// rounded on the way out); the optimizer updates a hot row's master in fp32, so that many small
// updates are not lost to 16-bit rounding, and a cold row in place as before.  These kernels
// use one group of LPR lanes per row, 8 elements per lane.

// row -> pointer to its 16-byte record
__device__ inline RowMeta* meta_ptr(const HtView& v, uint32_t row) {
    return &v.st->meta[row >> v.chunk_log2][row & ((1u << v.chunk_log2) - 1u)];
}
__device__ inline void hot_load8(const float* hp, float* w) {
    const V16 a = ld16(hp), b = ld16(hp + 4);
    w[0] = __uint_as_float(a.x); w[1] = __uint_as_float(a.y); w[2] = __uint_as_float(a.z); w[3] = __uint_as_float(a.w);
    w[4] = __uint_as_float(b.x); w[5] = __uint_as_float(b.y); w[6] = __uint_as_float(b.z); w[7] = __uint_as_float(b.w);
}
__device__ inline void hot_store8(float* hp, const float* w) {
    st16(hp, V16{__float_as_uint(w[0]), __float_as_uint(w[1]), __float_as_uint(w[2]), __float_as_uint(w[3])});
    st16(hp + 4, V16{__float_as_uint(w[4]), __float_as_uint(w[5]), __float_as_uint(w[6]), __float_as_uint(w[7])});
}
__device__ inline void unpack8(const V16& c, float* w) {
    w[0] = bf16lo(c.x); w[1] = bf16hi(c.x); w[2] = bf16lo(c.y); w[3] = bf16hi(c.y);
    w[4] = bf16lo(c.z); w[5] = bf16hi(c.z); w[6] = bf16lo(c.w); w[7] = bf16hi(c.w);
}
__device__ inline V16 pack8(const float* w) {
    return V16{pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3]), pack_bf16(w[4], w[5]), pack_bf16(w[6], w[7])};
}
__global__ void k_zero_words(uint32_t* p, int n) {
    if ((int)threadIdx.x < n) p[threadIdx.x] = 0u;
}
template <int LPR>
__device__ inline int64_t group_item() {
    constexpr int kGroups = kWave / LPR;
    return ((int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave) * kGroups + lane_id() / LPR;
}
template <int LPR>
constexpr int rows_per_block() { return (kBlock / kWave) * (kWave / LPR); }

// Give the rows of row_idx that were touched at least min_freq times and have no master yet one
// from the hot store (free stack first, then the bump pointer); rows stay cold when it is full.
template <int LPR>
__global__ __launch_bounds__(kBlock) void k_promote(HtView v, const int32_t* __restrict__ row_idx, const int64_t* n_dev,
                                                    int64_t n_max, uint32_t min_freq, unsigned long long* n_promoted) {
    const int64_t n = read_count(n_dev, n_max);
    const int lane = lane_id(), sub = lane % LPR;
    const int64_t u = group_item<LPR>();
    const int idx = u < n ? row_idx[u] : -1;
    int h = -1;
    if (sub == 0 && idx >= 0) {
        const RowMeta* m = meta_ptr(v, (uint32_t)idx);
        if (m->freq >= min_freq && m->hot == 0) {
            HtHead* hd = &v.st->head;
            const int f = atomicSub(&hd->hot_free_count, 1); // an entry is taken only by who sees a positive count
            if (f > 0) {
                h = (int)v.hot_free[f - 1];
            } else {
                atomicAdd(&hd->hot_free_count, 1);
                const unsigned b = atomicAdd(&hd->hot_bump, 1u);
                if (b < v.hot_capacity) h = (int)b;
                else atomicSub(&hd->hot_bump, 1u);
            }
        }
    }
    h = __shfl(h, lane - sub, kWave);
    if (h < 0) return;
    if (sub * 8 < v.dim) {
        float w[8];
        unpack8(ld16(chunk_row_cptr(v, (uint32_t)idx) + sub * 16), w);
        hot_store8(v.hot_values + (size_t)h * v.dim + sub * 8, w);
    }
    if (sub == 0) {
        meta_ptr(v, (uint32_t)idx)->hot = (uint32_t)h + 1u;
        if (n_promoted) atomicAdd(n_promoted, 1ull);
    }
}

// Demotion: one lane per slot decides (a live key whose row has a master and has not been looked up for `idle`
// steps); the slot of the master goes back on the hot store's free stack and the record's hot field is cleared;
// the wave then takes its demoting rows in turn and writes the master, rounded to nearest even, into the 16-bit
// row - the values lookups delivered for the row anyway.
__global__ __launch_bounds__(kBlock) void k_demote(HtView v, uint64_t n_slots, uint32_t now, uint32_t idle,
                                                   unsigned long long* n_demoted) {
    const int lane = lane_id();
    const uint64_t slot = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    uint32_t row = kRowInvalid, hot = 0;
    if (slot < n_slots) {
        const V16 e = ld16(v.slots + slot);
        const uint64_t k = ((uint64_t)e.y << 32) | e.x;
        if (k != kEmptyKey && k != kTombKey && e.z != kRowInvalid) {
            const RowMeta m = *meta_ptr(v, e.z);
            if (m.hot != 0 && now - m.last_seen >= idle) {
                row = e.z;
                hot = m.hot;
            }
        }
    }
    uint64_t m = __ballot(hot != 0);
    if (!m) return;
    if (n_demoted && lane == __ffsll((unsigned long long)m) - 1) atomicAdd(n_demoted, (unsigned long long)__popcll(m));
    if (hot != 0) { // hot rows are few: one atomic each
        v.hot_free[atomicAdd(&v.st->head.hot_free_count, 1)] = hot - 1u;
        meta_ptr(v, row)->hot = 0u;
    }
    while (m) {
        const int src = __ffsll((unsigned long long)m) - 1;
        m &= m - 1;
        const uint32_t r = __shfl(row, src, kWave);
        const float* hp = v.hot_values + (size_t)(__shfl(hot, src, kWave) - 1u) * v.dim;
        uint32_t* d32 = reinterpret_cast<uint32_t*>(const_cast<char*>(chunk_row_cptr(v, r)));
        for (int w = lane; w < v.dim / 2; w += kWave) d32[w] = pack_bf16(hp[2 * w], hp[2 * w + 1]);
    }
}

// out[dst,:] = row (source index = via ? via[index[j]] : index[j]; dst = dst_index ? dst_index[j] : j);
// index -1 gives a zero row.
template <int LPR>
__global__ __launch_bounds__(kBlock) void k_gather_mixed(HtView v, const int32_t* __restrict__ index,
                                                         const int32_t* __restrict__ via,
                                                         const int32_t* __restrict__ dst_index, const int64_t* n_dev,
                                                         int64_t n_max, char* __restrict__ out) {
    const int64_t n = read_count(n_dev, n_max);
    const int sub = lane_id() % LPR;
    const int64_t j = group_item<LPR>();
    if (j >= n || sub * 8 >= v.dim) return;
    int idx = index[j];
    if (via && idx >= 0) idx = via[idx];
    const int64_t dst = dst_index ? (int64_t)dst_index[j] : j;
    char* o = out + (size_t)dst * v.row_bytes + sub * 16;
    if (idx < 0) {
        st16(o, V16{0u, 0u, 0u, 0u});
        return;
    }
    const uint32_t hot = meta_ptr(v, (uint32_t)idx)->hot;
    if (hot != 0) {
        float w[8];
        hot_load8(v.hot_values + (size_t)(hot - 1u) * v.dim + sub * 8, w);
        st16(o, pack8(w));
    } else {
        st16(o, ld16(chunk_row_cptr(v, (uint32_t)idx) + sub * 16));
    }
}

// Row-wise Adagrad with the arithmetic of k_adagrad; a hot row's master stays in fp32.
template <int LPR>
__global__ __launch_bounds__(kBlock) void k_adagrad_mixed(HtView v, const int32_t* __restrict__ row_idx,
                                                          const float* __restrict__ g, const int64_t* n_dev,
                                                          int64_t n_max, float lr, float eps, int touch, uint32_t step) {
    const int64_t n = read_count(n_dev, n_max);
    const int sub = lane_id() % LPR;
    const int64_t u = group_item<LPR>();
    const bool lane_on = sub * 8 < v.dim;
    const int idx = u < n ? row_idx[u] : -1;
    float gv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) gv[e] = 0.0f;
    if (idx >= 0 && lane_on) hot_load8(g + (size_t)u * v.dim + sub * 8, gv);
    const float ss = sumsq_group<LPR>(sumsq_lane<8>(gv));
    if (idx < 0) return;
    RowMeta* m = meta_ptr(v, (uint32_t)idx);
    const uint32_t hot = m->hot;
    const float acc = adagrad_acc(m->acc, ss, __fdiv_rn(1.0f, (float)v.dim));
    const float scale = adagrad_scale(acc, lr, eps);
    if (lane_on) {
        float w[8];
        if (hot != 0) {
            float* hp = v.hot_values + (size_t)(hot - 1u) * v.dim + sub * 8;
            hot_load8(hp, w);
#pragma unroll
            for (int e = 0; e < 8; ++e) w[e] = adagrad_w(w[e], gv[e], scale);
            hot_store8(hp, w);
        } else {
            char* wp = const_cast<char*>(chunk_row_cptr(v, (uint32_t)idx)) + sub * 16;
            unpack8(ld16(wp), w);
#pragma unroll
            for (int e = 0; e < 8; ++e) w[e] = adagrad_w(w[e], gv[e], scale);
            st16(wp, pack8(w));
        }
    }
    if (sub == 0) {
        m->acc = acc;
        if (touch) {
            m->last_seen = step;
            m->freq += 1u;
        }
    }
}

// ---------------------------------------------------------------------------- put rows (checkpoint import)
// values[row_idx[u],:] = src[u,:] and the row record = (acc[u], last_seen[u], freq[u]): the inverse of
// gather + export, used to restore a dump into a table.  16-byte vectors, one lane per vector.
__global__ __launch_bounds__(kBlock) void k_put_rows(HtView v, const int32_t* __restrict__ row_idx,
                                                     const char* __restrict__ src, const float* __restrict__ acc,
                                                     const uint32_t* __restrict__ last_seen,
                                                     const uint32_t* __restrict__ freq, int64_t n) {
    const int vecs = v.row_bytes / 16;
    const int64_t item = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t u = item / vecs;
    const int sub = (int)(item % vecs);
    if (u >= n) return;
    const int ri = row_idx[u];
    if (ri < 0) return;
    const uint32_t row = (uint32_t)ri;
    char* dst = const_cast<char*>(chunk_row_cptr(v, row));
    RowMeta* m = &v.st->meta[row >> v.chunk_log2][row & ((1u << v.chunk_log2) - 1u)];
    if (src) {
        const V16 x = ld16(src + (size_t)u * v.row_bytes + sub * 16);
        st16(dst + sub * 16, x);
        const uint32_t hot = v.hot_values ? m->hot : 0u;
        if (hot != 0) { // a row with an fp32 master: the master follows
            float w[8];
            unpack8(x, w);
            hot_store8(v.hot_values + (size_t)(hot - 1u) * v.dim + sub * 8, w);
        }
    }
    if (sub == 0) {
        if (acc) m->acc = acc[u];
        if (last_seen) m->last_seen = last_seen[u];
        if (freq) m->freq = freq[u];
    }
}

// masters[hot(row_idx[u]) - 1, :] = src[u,:] for the rows that have a master (checkpoint import of the fp32 copies
// ht_export_hot dumped); one lane per 16-byte vector of four floats.
__global__ __launch_bounds__(kBlock) void k_put_hot(HtView v, const int32_t* __restrict__ row_idx,
                                                    const float* __restrict__ src, int64_t n,
                                                    unsigned long long* n_written) {
    const int vecs = v.dim / 4;
    const int64_t item = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t u = item / vecs;
    const int sub = (int)(item % vecs);
    if (u >= n) return;
    const int ri = row_idx[u];
    if (ri < 0) return;
    const uint32_t hot = meta_ptr(v, (uint32_t)ri)->hot;
    if (hot == 0) return;
    st16(v.hot_values + (size_t)(hot - 1u) * v.dim + sub * 4, ld16(src + (size_t)u * v.dim + sub * 4));
    if (sub == 0 && n_written) atomicAdd(n_written, 1ull);
}

// ---------------------------------------------------------------------------- sparse Adam
// The optimizer the paper trains with (Sec. 4.1), in its lazy / sparse form: only the listed rows
// move.  m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;  w -= step_size * m / (sqrt(v) + eps) with
// step_size = lr * sqrt(1 - b2^t) / (1 - b1^t) computed on the host.  One lane handles 4 (fp32
// table) or 8 (bf16 table) elements; the moment rows are fp32.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void k_adam(HtView v, const int32_t* __restrict__ row_idx, const float* __restrict__ g,
                                                 const int64_t* n_dev, int64_t n_max, float step_size, float b1,
                                                 float b2, float eps) {
    const int64_t n = read_count(n_dev, n_max);
    constexpr int kF = BF16 ? 8 : 4;
    const int per_row = v.dim / kF;                      // lanes' worth of work per row
    const int64_t item = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t u = item / per_row;
    const int sub = (int)(item % per_row);
    if (u >= n) return;
    const int ri = row_idx[u];
    if (ri < 0) return;
    const uint32_t row = (uint32_t)ri;
    const size_t o = (size_t)(row & ((1u << v.chunk_log2) - 1u)) * (size_t)v.dim + (size_t)sub * kF;
    float* pm = v.st->adam_m[row >> v.chunk_log2] + o;
    float* pv = v.st->adam_v[row >> v.chunk_log2] + o;
    const float* pg = g + (size_t)u * v.dim + (size_t)sub * kF;
    char* pw = const_cast<char*>(chunk_row_cptr(v, row)) + sub * 16;
    float w[kF];
    // a row of a 16-bit table that has an fp32 master: the master is what moves (and is not rounded)
    float* master = nullptr;
    if constexpr (BF16) {
        if (v.hot_values) {
            const uint32_t hot = meta_ptr(v, row)->hot;
            if (hot != 0) master = v.hot_values + (size_t)(hot - 1u) * v.dim + (size_t)sub * kF;
        }
    }
    const V16 wv = master ? V16{0u, 0u, 0u, 0u} : ld16(pw);
    if constexpr (BF16) {
        if (master) hot_load8(master, w);
    }
    if (master) {
    } else if (BF16) {
        w[0] = bf16lo(wv.x); w[1] = bf16hi(wv.x); w[2] = bf16lo(wv.y); w[3] = bf16hi(wv.y);
        w[4 % kF] = bf16lo(wv.z); w[5 % kF] = bf16hi(wv.z); w[6 % kF] = bf16lo(wv.w); w[7 % kF] = bf16hi(wv.w);
    } else {
        w[0] = __uint_as_float(wv.x); w[1] = __uint_as_float(wv.y); w[2] = __uint_as_float(wv.z); w[3] = __uint_as_float(wv.w);
    }
    const float c1 = __fsub_rn(1.0f, b1), c2 = __fsub_rn(1.0f, b2);
#pragma unroll
    for (int q = 0; q < kF / 4; ++q) {
        V16 gm = ld16(pg + 4 * q), mm = ld16(pm + 4 * q), vv = ld16(pv + 4 * q);
        uint32_t* gp = &gm.x; uint32_t* mp = &mm.x; uint32_t* vp = &vv.x;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float gg = __uint_as_float(gp[e]);
            const float m1 = __fmaf_rn(c1, gg, __fmul_rn(b1, __uint_as_float(mp[e])));
            const float v1 = __fmaf_rn(c2, __fmul_rn(gg, gg), __fmul_rn(b2, __uint_as_float(vp[e])));
            mp[e] = __float_as_uint(m1);
            vp[e] = __float_as_uint(v1);
            w[4 * q + e] = __fmaf_rn(-step_size, __fdiv_rn(m1, __fadd_rn(__fsqrt_rn(v1), eps)), w[4 * q + e]);
        }
        st16(pm + 4 * q, mm);
        st16(pv + 4 * q, vv);
    }
    if constexpr (BF16) {
        if (master) {
            hot_store8(master, w);
            return;
        }
    }
    V16 o16;
    if (BF16) {
        o16.x = pack_bf16(w[0], w[1]); o16.y = pack_bf16(w[2], w[3]);
        o16.z = pack_bf16(w[4 % kF], w[5 % kF]); o16.w = pack_bf16(w[6 % kF], w[7 % kF]);
    } else {
        o16.x = __float_as_uint(w[0]); o16.y = __float_as_uint(w[1]); o16.z = __float_as_uint(w[2]); o16.w = __float_as_uint(w[3]);
    }
    st16(pw, o16);
}

} // namespace

extern "C" {

// launch K<LPR> for the smallest power-of-two group that covers `vecs` 16-byte vectors of a 16-bit row
#define MTGR_MIXED_LAUNCH(K, vecs, n_rows, s, ...)                                                                     \
    do {                                                                                                               \
        if ((vecs) <= 1) hipLaunchKernelGGL((K<1>), dim3((unsigned)(((n_rows) + rows_per_block<1>() - 1) / rows_per_block<1>())), dim3(kBlock), 0, s, __VA_ARGS__);       \
        else if ((vecs) <= 2) hipLaunchKernelGGL((K<2>), dim3((unsigned)(((n_rows) + rows_per_block<2>() - 1) / rows_per_block<2>())), dim3(kBlock), 0, s, __VA_ARGS__);  \
        else if ((vecs) <= 4) hipLaunchKernelGGL((K<4>), dim3((unsigned)(((n_rows) + rows_per_block<4>() - 1) / rows_per_block<4>())), dim3(kBlock), 0, s, __VA_ARGS__);  \
        else if ((vecs) <= 8) hipLaunchKernelGGL((K<8>), dim3((unsigned)(((n_rows) + rows_per_block<8>() - 1) / rows_per_block<8>())), dim3(kBlock), 0, s, __VA_ARGS__);  \
        else if ((vecs) <= 16) hipLaunchKernelGGL((K<16>), dim3((unsigned)(((n_rows) + rows_per_block<16>() - 1) / rows_per_block<16>())), dim3(kBlock), 0, s, __VA_ARGS__); \
        else hipLaunchKernelGGL((K<32>), dim3((unsigned)(((n_rows) + rows_per_block<32>() - 1) / rows_per_block<32>())), dim3(kBlock), 0, s, __VA_ARGS__);                \
    } while (0)

int ht_promote(emb_table_t* t, const int32_t* row_idx, const int64_t* n_dev, int64_t n_max, uint32_t min_freq,
               int64_t* n_promoted, void* stream) {
    if (!t || n_max < 0 || n_max > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (!t->hot_values) return EMB_ERR_NO_STORAGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n_promoted) {
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(n_promoted), 2);
        MTGR_LAUNCH_CHECK();
    }
    if (n_max == 0) return EMB_OK;
    if (!row_idx) return EMB_ERR_INVALID_ARG;
    HtView v = t->view();
    MTGR_MIXED_LAUNCH(k_promote, t->row_bytes / 16, n_max, s, v, row_idx, n_dev, n_max, min_freq,
                      reinterpret_cast<unsigned long long*>(n_promoted));
    MTGR_LAUNCH_CHECK();
    return t->snapshot(s);
}

int ht_demote(emb_table_t* t, uint32_t now, uint32_t idle, int64_t* n_demoted, void* stream) {
    if (!t) return EMB_ERR_INVALID_ARG;
    if (!t->hot_values || !t->slots) return EMB_ERR_NO_STORAGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n_demoted) {
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(n_demoted), 2);
        MTGR_LAUNCH_CHECK();
    }
    const uint64_t n_slots = 1ull << t->cap_log2;
    hipLaunchKernelGGL(k_demote, dim3((unsigned)((n_slots + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, t->view(), n_slots, now,
                       idle, reinterpret_cast<unsigned long long*>(n_demoted));
    MTGR_LAUNCH_CHECK();
    return t->snapshot(s);
}

int ht_gather(emb_table_t* t, const int32_t* row_idx, const int64_t* n_dev, int64_t n_max, void* out, void* stream) {
    if (!t || n_max < 0 || n_max > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (n_max == 0) return EMB_OK;
    if (!row_idx || !out || (reinterpret_cast<uintptr_t>(out) & 15)) return EMB_ERR_INVALID_ARG;
    if (t->n_chunks == 0) return EMB_ERR_NO_STORAGE;
    if (t->hot_values) {
        HtView v = t->view();
        MTGR_MIXED_LAUNCH(k_gather_mixed, t->row_bytes / 16, n_max, static_cast<hipStream_t>(stream), v, row_idx,
                          (const int32_t*)nullptr, (const int32_t*)nullptr, n_dev, n_max, static_cast<char*>(out));
        MTGR_LAUNCH_CHECK();
        return EMB_OK;
    }
    return launch_copy_rows<true, false, false>(t->view(), nullptr, row_idx, nullptr, nullptr, n_dev, n_max, t->row_bytes,
                                                static_cast<char*>(out), static_cast<hipStream_t>(stream));
}

int emb_expand(const void* uniq_rows, const int32_t* inverse, int64_t n, int dim, int dtype, void* out, void* stream) {
    if (n < 0 || n > 0x7FFFFFFFll || dim <= 0 || (dtype != EMB_F32 && dtype != EMB_BF16)) return EMB_ERR_INVALID_ARG;
    if (n == 0) return EMB_OK;
    const int row_bytes = dim * (dtype == EMB_F32 ? 4 : 2);
    if (row_bytes % 16 != 0 || row_bytes > 1024) return EMB_ERR_INVALID_ARG;
    if (!uniq_rows || !inverse || !out) return EMB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(uniq_rows) & 15) || (reinterpret_cast<uintptr_t>(out) & 15)) return EMB_ERR_INVALID_ARG;
    HtView none{};
    return launch_copy_rows<false, true, false>(none, static_cast<const char*>(uniq_rows), inverse, nullptr, nullptr, nullptr, n,
                                                row_bytes, static_cast<char*>(out), static_cast<hipStream_t>(stream));
}

int emb_expand_sorted(const void* uniq_rows, const int32_t* seg_of, const int32_t* perm, int64_t n, int dim, int dtype,
                      void* out, void* stream) {
    if (n < 0 || n > 0x7FFFFFFFll || dim <= 0 || (dtype != EMB_F32 && dtype != EMB_BF16)) return EMB_ERR_INVALID_ARG;
    if (n == 0) return EMB_OK;
    const int row_bytes = dim * (dtype == EMB_F32 ? 4 : 2);
    if (row_bytes % 16 != 0 || row_bytes > 1024) return EMB_ERR_INVALID_ARG;
    if (!uniq_rows || !seg_of || !perm || !out) return EMB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(uniq_rows) & 15) || (reinterpret_cast<uintptr_t>(out) & 15)) return EMB_ERR_INVALID_ARG;
    HtView none{};
    return launch_copy_rows<false, true, true>(none, static_cast<const char*>(uniq_rows), seg_of, nullptr, perm, nullptr, n,
                                               row_bytes, static_cast<char*>(out), static_cast<hipStream_t>(stream));
}

int ht_gather_expand_sorted(emb_table_t* t, const int32_t* row_idx, const int32_t* seg_of, const int32_t* perm, int64_t n,
                            void* out, void* stream) {
    if (!t || n < 0 || n > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (n == 0) return EMB_OK;
    if (!row_idx || !seg_of || !perm || !out || (reinterpret_cast<uintptr_t>(out) & 15)) return EMB_ERR_INVALID_ARG;
    if (t->n_chunks == 0) return EMB_ERR_NO_STORAGE;
    if (t->hot_values) {
        HtView v = t->view();
        MTGR_MIXED_LAUNCH(k_gather_mixed, t->row_bytes / 16, n, static_cast<hipStream_t>(stream), v, seg_of, row_idx, perm,
                          (const int64_t*)nullptr, n, static_cast<char*>(out));
        MTGR_LAUNCH_CHECK();
        return EMB_OK;
    }
    return launch_copy_rows<true, true, true>(t->view(), nullptr, seg_of, row_idx, perm, nullptr, n, t->row_bytes,
                                              static_cast<char*>(out), static_cast<hipStream_t>(stream));
}

size_t grad_segment_reduce_workspace_bytes(int64_t n, int dim) {
    if (n <= 0 || dim <= 0) return 256;
    return reduce_layout(n, dim).total;
}

static int reduce_dispatch(const void* grad, int grad_dtype, const int32_t* seg_of, const int32_t* perm, const int32_t* via,
                           int64_t n, int dim, float* reduced, void* workspace, size_t workspace_bytes, hipStream_t s,
                           const FuseArgs* fz = nullptr) {
    const int in_row_bytes = dim * (grad_dtype == EMB_F32 ? 4 : 2);
    if (in_row_bytes % 16 != 0 || dim > 256) return EMB_ERR_INVALID_ARG;
    if (!grad || !seg_of || !perm || (!reduced && !fz)) return EMB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(grad) & 15) || (reinterpret_cast<uintptr_t>(reduced) & 15)) return EMB_ERR_INVALID_ARG;
    const ReduceLayout L = reduce_layout(n, dim);
    if (!workspace || workspace_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return EMB_ERR_WORKSPACE;
    const char* g = static_cast<const char*>(grad);
    char* ws = static_cast<char*>(workspace);
    const int vecs = in_row_bytes / 16;
#define MTGR_RED(L_)                                                                                                      \
    (fz ? (grad_dtype == EMB_F32 ? launch_reduce_apply<L_, 4>(g, in_row_bytes, seg_of, perm, n, dim, ws, L, s, *fz)       \
                                 : launch_reduce_apply<L_, 8>(g, in_row_bytes, seg_of, perm, n, dim, ws, L, s, *fz))      \
        : (grad_dtype == EMB_F32 ? launch_reduce<L_, 4>(g, in_row_bytes, seg_of, perm, via, n, dim, reduced, ws, L, s)    \
                                 : launch_reduce<L_, 8>(g, in_row_bytes, seg_of, perm, via, n, dim, reduced, ws, L, s)))
    if (vecs <= 1) return MTGR_RED(1);
    if (vecs <= 2) return MTGR_RED(2);
    if (vecs <= 4) return MTGR_RED(4);
    if (vecs <= 8) return MTGR_RED(8);
    if (vecs <= 16) return MTGR_RED(16);
    if (vecs <= 32) return MTGR_RED(32);
    return MTGR_RED(64);
#undef MTGR_RED
}

int grad_segment_reduce(const void* grad, int grad_dtype, const int32_t* seg_of, const int32_t* perm, int64_t n,
                        int dim, float* reduced, void* workspace, size_t workspace_bytes, void* stream) {
    if (n < 0 || n > 0x7FFFFFFFll || dim <= 0 || (grad_dtype != EMB_F32 && grad_dtype != EMB_BF16)) return EMB_ERR_INVALID_ARG;
    if (n == 0) return EMB_OK;
    return reduce_dispatch(grad, grad_dtype, seg_of, perm, nullptr, n, dim, reduced, workspace, workspace_bytes,
                           static_cast<hipStream_t>(stream));
}

int grad_reduce_apply_adagrad(emb_table_t* t, const void* grad, const int32_t* seg_of, const int32_t* perm, int64_t n,
                              const int32_t* row_idx, float lr, float eps, int touch, uint32_t step, void* workspace,
                              size_t workspace_bytes, void* stream) {
    if (!t || n < 0 || n > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (n == 0) return EMB_OK;
    if (!row_idx) return EMB_ERR_INVALID_ARG;
    if (t->n_chunks == 0) return EMB_ERR_NO_STORAGE;
    if (t->hot_values) return EMB_ERR_INVALID_ARG; // rows with fp32 masters take the two-call form
    FuseArgs fz{t->view(), row_idx, lr, eps, step, touch ? 1 : 0, t->n_chunks};
    return reduce_dispatch(grad, t->desc.dtype, seg_of, perm, nullptr, n, t->desc.dim, nullptr, workspace, workspace_bytes,
                           static_cast<hipStream_t>(stream), &fz);
}

// ---------------------------------------------------------------------------- pooling (Sec. 3.2, HashTableCollection)
// Bags are runs of consecutive positions (one bag per sample and field).  Pooling the rows of a bag
// is the same fixed-tree segmented sum as the gradient reduction, with the bag as the segment and
// uniq_rows[inverse[i]] as the row of position i; its backward pass is the gradient reduction with
// row dY[bag_of[i]] (scaled by 1/len for the mean) as the gradient of position i.
namespace {
__global__ __launch_bounds__(kBlock) void k_bag_of(const int64_t* __restrict__ bag_off, int n_bags, int64_t n,
                                                   int32_t* __restrict__ bag_of) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    int lo = 0, hi = n_bags; // invariant: bag_off[lo] <= i < bag_off[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (bag_off[mid] <= i) lo = mid; else hi = mid;
    }
    bag_of[i] = lo;
}
// out[b,:] = in[b,:] / len(b) for the mean (empty bags give zeros), or a plain copy / zero fill
__global__ __launch_bounds__(kBlock) void k_bag_rows(const float* __restrict__ in, const int64_t* __restrict__ bag_off,
                                                     int n_bags, int dim, int mean, int zero_empty_only,
                                                     float* __restrict__ out) {
    const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= (int64_t)n_bags * dim) return;
    const int b = (int)(e / dim);
    const int64_t len = bag_off[b + 1] - bag_off[b];
    if (zero_empty_only) {
        if (len == 0) out[e] = 0.0f;
        return;
    }
    float v = in[e];
    if (len == 0) v = 0.0f;
    else if (mean) v = __fdiv_rn(v, (float)len);
    out[e] = v;
}
struct PoolLayout {
    size_t bag_of, scaled, reduce, total;
};
PoolLayout pool_layout(int64_t n, int n_bags, int dim) {
    PoolLayout L;
    size_t o = 0;
    L.bag_of = o; o = align256(o + (size_t)(n > 0 ? n : 1) * 4);
    L.scaled = o; o = align256(o + (size_t)(n_bags > 0 ? n_bags : 1) * dim * 4);
    L.reduce = o; o += reduce_layout(n > 0 ? n : 1, dim).total;
    L.total = o;
    return L;
}
} // namespace

size_t emb_pool_workspace_bytes(int64_t n, int n_bags, int dim) {
    if (n < 0 || n_bags < 0 || dim <= 0) return 0;
    return pool_layout(n, n_bags, dim).total;
}

int emb_pool_bags(const void* uniq_rows, int dtype, const int32_t* inverse, const int64_t* bag_off, int n_bags, int64_t n,
                  int dim, int mean, float* pooled, void* workspace, size_t workspace_bytes, void* stream) {
    if (n < 0 || n > 0x7FFFFFFFll || n_bags < 0 || dim <= 0 || (dtype != EMB_F32 && dtype != EMB_BF16)) return EMB_ERR_INVALID_ARG;
    if (n_bags == 0) return n == 0 ? EMB_OK : EMB_ERR_INVALID_ARG;
    if (!bag_off || !pooled || (n > 0 && (!uniq_rows || !inverse))) return EMB_ERR_INVALID_ARG;
    const PoolLayout L = pool_layout(n, n_bags, dim);
    if (!workspace || workspace_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return EMB_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    int32_t* bag_of = reinterpret_cast<int32_t*>(ws + L.bag_of);
    const unsigned bgrid = (unsigned)(((int64_t)n_bags * dim + kBlock - 1) / kBlock);
    if (n > 0) {
        hipLaunchKernelGGL(k_bag_of, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, bag_off, n_bags, n, bag_of);
        MTGR_LAUNCH_CHECK();
        // segmented sum: segment = bag, source row of position i = uniq_rows[inverse[i]]
        int rc = reduce_dispatch(uniq_rows, dtype, bag_of, inverse, nullptr, n, dim, pooled, ws + L.reduce,
                                 workspace_bytes - L.reduce, s);
        if (rc != EMB_OK) return rc;
    }
    // bags without positions were not written by the sum; the mean divides by the bag length
    if (mean)
        hipLaunchKernelGGL(k_bag_rows, dim3(bgrid), dim3(kBlock), 0, s, pooled, bag_off, n_bags, dim, 1, 0, pooled);
    else
        hipLaunchKernelGGL(k_bag_rows, dim3(bgrid), dim3(kBlock), 0, s, pooled, bag_off, n_bags, dim, 0, 1, pooled);
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

int grad_segment_reduce_pooled(const float* d_pooled, const int64_t* bag_off, int n_bags, const int32_t* seg_of,
                               const int32_t* perm, int64_t n, int dim, int mean, float* reduced, void* workspace,
                               size_t workspace_bytes, void* stream) {
    if (n < 0 || n > 0x7FFFFFFFll || n_bags < 0 || dim <= 0) return EMB_ERR_INVALID_ARG;
    if (n == 0) return EMB_OK;
    if (!d_pooled || !bag_off || n_bags == 0) return EMB_ERR_INVALID_ARG;
    const PoolLayout L = pool_layout(n, n_bags, dim);
    if (!workspace || workspace_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return EMB_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    int32_t* bag_of = reinterpret_cast<int32_t*>(ws + L.bag_of);
    float* scaled = reinterpret_cast<float*>(ws + L.scaled);
    hipLaunchKernelGGL(k_bag_of, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, bag_off, n_bags, n, bag_of);
    const unsigned bgrid = (unsigned)(((int64_t)n_bags * dim + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(k_bag_rows, dim3(bgrid), dim3(kBlock), 0, s, d_pooled, bag_off, n_bags, dim, mean ? 1 : 0, 0, scaled);
    MTGR_LAUNCH_CHECK();
    // gradient of position i = scaled[bag_of[i]]; summed per distinct key in the usual fixed order
    return reduce_dispatch(scaled, EMB_F32, seg_of, perm, bag_of, n, dim, reduced, ws + L.reduce, workspace_bytes - L.reduce, s);
}

int ht_put(emb_table_t* t, const int32_t* row_idx, const void* values, const float* acc, const uint32_t* last_seen,
           const uint32_t* freq, int64_t n, void* stream) {
    if (!t || n < 0 || n > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (n == 0) return EMB_OK;
    if (!row_idx || (values && (reinterpret_cast<uintptr_t>(values) & 15))) return EMB_ERR_INVALID_ARG;
    if (t->n_chunks == 0) return EMB_ERR_NO_STORAGE;
    HtView v = t->view();
    const int vecs = t->row_bytes / 16;
    const unsigned grid = (unsigned)((n * vecs + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(k_put_rows, dim3(grid), dim3(kBlock), 0, static_cast<hipStream_t>(stream), v, row_idx,
                       static_cast<const char*>(values), acc, last_seen, freq, n);
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

int ht_put_hot(emb_table_t* t, const int32_t* row_idx, const float* masters, int64_t n, int64_t* n_written, void* stream) {
    if (!t || n < 0 || n > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (!t->hot_values) return EMB_ERR_NO_STORAGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n_written) {
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(n_written), 2);
        MTGR_LAUNCH_CHECK();
    }
    if (n == 0) return EMB_OK;
    if (!row_idx || !masters || (reinterpret_cast<uintptr_t>(masters) & 15)) return EMB_ERR_INVALID_ARG;
    HtView v = t->view();
    const int vecs = v.dim / 4;
    hipLaunchKernelGGL(k_put_hot, dim3((unsigned)((n * vecs + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, v, row_idx, masters, n,
                       reinterpret_cast<unsigned long long*>(n_written));
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

int ht_apply_adam(emb_table_t* t, const int32_t* row_idx, const float* reduced, const int64_t* n_dev, int64_t n_max,
                  float lr, float beta1, float beta2, float eps, int64_t step, void* stream) {
    if (!t || n_max < 0 || n_max > 0x7FFFFFFFll || step < 1) return EMB_ERR_INVALID_ARG;
    if (!(beta1 >= 0.0f && beta1 < 1.0f && beta2 >= 0.0f && beta2 < 1.0f)) return EMB_ERR_INVALID_ARG;
    if (n_max == 0) return EMB_OK;
    if (!row_idx || !reduced || (reinterpret_cast<uintptr_t>(reduced) & 15)) return EMB_ERR_INVALID_ARG;
    HtView v = t->view();
    if (!v.has_adam) return EMB_ERR_NO_STORAGE; // moment rows must be registered for every chunk
    const double bc1 = 1.0 - std::pow((double)beta1, (double)step), bc2 = 1.0 - std::pow((double)beta2, (double)step);
    const float step_size = (float)((double)lr * std::sqrt(bc2) / bc1);
    const bool bf = t->desc.dtype == EMB_BF16;
    const int per_row = t->desc.dim / (bf ? 8 : 4);
    const unsigned grid = (unsigned)((n_max * per_row + kBlock - 1) / kBlock);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (bf) hipLaunchKernelGGL(k_adam<true>, dim3(grid), dim3(kBlock), 0, s, v, row_idx, reduced, n_dev, n_max, step_size, beta1, beta2, eps);
    else hipLaunchKernelGGL(k_adam<false>, dim3(grid), dim3(kBlock), 0, s, v, row_idx, reduced, n_dev, n_max, step_size, beta1, beta2, eps);
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

static int adagrad_impl(emb_table_t* t, const int32_t* row_idx, const float* reduced, const int64_t* n_dev,
                        int64_t n_max, float lr, float eps, bool touch, uint32_t step, void* stream) {
    if (!t || n_max < 0 || n_max > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (n_max == 0) return EMB_OK;
    if (!row_idx || !reduced || (reinterpret_cast<uintptr_t>(reduced) & 15)) return EMB_ERR_INVALID_ARG;
    if (t->n_chunks == 0) return EMB_ERR_NO_STORAGE;
    HtView v = t->view();
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((n_max + kBlock - 1) / kBlock);
    const int vecs = t->row_bytes / 16;
    const bool bf = t->desc.dtype == EMB_BF16;
    if (t->hot_values) {
        MTGR_MIXED_LAUNCH(k_adagrad_mixed, vecs, n_max, s, v, row_idx, reduced, n_dev, n_max, lr, eps, touch ? 1 : 0, step);
        MTGR_LAUNCH_CHECK();
        return EMB_OK;
    }
#define MTGR_ADA2(L_, B_, T_) \
    hipLaunchKernelGGL((k_adagrad<L_, B_, T_>), dim3(grid), dim3(kBlock), 0, s, v, row_idx, reduced, n_dev, n_max, lr, eps, step)
#define MTGR_ADA(L_)                                                    \
    do {                                                                \
        if (bf) { if (touch) MTGR_ADA2(L_, true, true); else MTGR_ADA2(L_, true, false); }   \
        else { if (touch) MTGR_ADA2(L_, false, true); else MTGR_ADA2(L_, false, false); }    \
    } while (0)
    if (vecs <= 1) MTGR_ADA(1);
    else if (vecs <= 2) MTGR_ADA(2);
    else if (vecs <= 4) MTGR_ADA(4);
    else if (vecs <= 8) MTGR_ADA(8);
    else if (vecs <= 16) MTGR_ADA(16);
    else if (vecs <= 32) MTGR_ADA(32);
    else MTGR_ADA(64);
#undef MTGR_ADA
#undef MTGR_ADA2
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

int ht_apply_adagrad(emb_table_t* t, const int32_t* row_idx, const float* reduced, const int64_t* n_dev,
                     int64_t n_max, float lr, float eps, void* stream) {
    return adagrad_impl(t, row_idx, reduced, n_dev, n_max, lr, eps, false, 0u, stream);
}

int ht_apply_adagrad_touch(emb_table_t* t, const int32_t* row_idx, const float* reduced, const int64_t* n_dev,
                           int64_t n_max, float lr, float eps, uint32_t step, void* stream) {
    return adagrad_impl(t, row_idx, reduced, n_dev, n_max, lr, eps, true, step, stream);
}

} // extern "C"
