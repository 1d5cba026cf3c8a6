// Shared device/host helpers of the gfx950 sparse-embedding kernels (wave64 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <cstddef>

#include "mtgr_emb.h"

namespace mtgr {

constexpr int kWave = 64;
constexpr uint64_t kEmptyKey = 0xFFFFFFFFFFFFFFFFull; // never-used slot
constexpr uint64_t kTombKey = 0xFFFFFFFFFFFFFFFEull;  // deleted slot, reclaimed by rehash only
constexpr uint32_t kRowInvalid = 0xFFFFFFFFu;
constexpr int kLineSlots = 8;                         // one probe = one aligned 128-byte line of 8 slots
constexpr int kMaxChunks = 256;
constexpr int kStatStripes = 64;

// One slot of the key structure: the key and the index of its embedding row (Sec. 3.1: the key
// structure maps keys to pointers into the embedding structure).
struct __attribute__((aligned(16))) Slot {
    unsigned long long key;
    uint32_t row;
    uint32_t pad;
};

// Per-row auxiliary data of the embedding structure, one 16-byte record per row so that the
// touch of find-or-insert and the accumulator update of the optimizer hit the same line.
struct __attribute__((aligned(16))) RowMeta {
    float acc;           // row-wise Adagrad accumulator
    uint32_t last_seen;  // step of the last find-or-insert touch
    uint32_t freq;       // number of touches
    uint32_t hot;        // 0 = the row lives in its chunk only; h+1 = fp32 master copy in row h of the hot store
};

// Device-resident table state: counters + chunk directory.  Lives in caller memory.
// Counters that are only ever added to (no return value needed) are striped over 64 cache lines:
// atomics of concurrently running blocks on one address queue up behind each other (about 25 ns
// apiece on this part), atomics on different lines do not.
enum StatSlot { kStatLookups = 0, kStatProbes, kStatCas, kStatCasFail, kStatAlloc, kStatLive, kStatTomb, kStatUnused,
                kStatHist0 /* .. kStatHist0 + 7: keys that inspected 1, 2, .. 7, 8 or more slot lines */ };
constexpr int kStatSlots = 16;
struct HtHead {
    // line 0: the row allocator
    unsigned int bump;       // rows handed out by the bump allocator
    int free_count;          // entries on the free-row stack (may dip below 0 inside an insert kernel)
    unsigned int status;     // EMB_DEV_* bits
    unsigned int hot_bump;   // rows handed out from the hot store
    int hot_free_count;      // entries on the hot store's free stack
    unsigned int pad0;
    unsigned long long pad1[13];
    // line 1: admission.  Every block that brings new keys does one returning atomic here and one on `bump`;
    // atomics on one 128-byte line queue up behind each other (about 25 ns apiece), so the two counters
    // live on lines of their own.
    unsigned int occupied;   // slots that are not never-used (live + deleted): inserts are admitted against the load-factor limit here
    unsigned int pad2;
    unsigned long long refused; // new keys turned away so far (limit reached, out of rows, probe sequence exhausted)
    unsigned long long pad3[14];
    unsigned long long stat[kStatStripes][kStatSlots]; // [stripe][StatSlot]; live / deleted counts are the sums over stripes
};
static_assert(offsetof(HtHead, occupied) == 128 && offsetof(HtHead, stat) == 256, "counter lines");
struct HtState {
    HtHead head;
    void* values[kMaxChunks];
    RowMeta* meta[kMaxChunks];
    uint32_t* free_list[kMaxChunks];
    float* adam_m[kMaxChunks];   // optional per-chunk first/second moment rows (fp32 [rows, dim]); null = none
    float* adam_v[kMaxChunks];
};

// Host view of the counters.
struct HtCounts {
    unsigned long long live, tombstones;
    unsigned int bump;
    int free_count;
    unsigned int status;
    unsigned int hot_bump;
    int hot_free_count;
    unsigned long long refused;
    unsigned long long stat[5];
    unsigned long long probe_hist[8];
    static HtCounts from(const HtHead& h) {
        HtCounts c{};
        c.refused = h.refused;
        c.hot_bump = h.hot_bump;
        c.hot_free_count = h.hot_free_count;
        c.bump = h.bump;
        c.free_count = h.free_count;
        c.status = h.status;
        for (int i = 0; i < kStatStripes; ++i) {
            c.live += h.stat[i][kStatLive];            // wraps: stripes hold signed deltas
            c.tombstones += h.stat[i][kStatTomb];
            for (int k = 0; k < 5; ++k) c.stat[k] += h.stat[i][k];
            for (int k = 0; k < 8; ++k) c.probe_hist[k] += h.stat[i][kStatHist0 + k];
        }
        return c;
    }
};

// What a table kernel needs, passed by value.
struct HtView {
    Slot* slots;
    HtState* st;
    uint64_t line_mask;      // (capacity / kLineSlots) - 1
    uint32_t slot_limit;     // floor(max_load_factor * capacity): live + deleted slots never exceed it
    uint32_t rows_capacity;  // rows in registered chunks
    int chunk_log2;
    int dim;
    int dtype;
    int row_bytes;
    float init_c;            // init_scale * 2^-23
    int count;               // maintain probe counters
    int has_adam;            // moment rows are registered for every chunk
    float* hot_values;       // optional fp32 master rows of frequently used keys [hot_capacity, dim]; null = none
    uint32_t* hot_free;      // free stack of the hot store [hot_capacity]
    uint32_t hot_capacity;
};

// ---- slot hash: the 64-bit finalizer of MurmurHash3 (Sec. 3.1 names MurmurHash3) ----------
__host__ __device__ inline uint64_t slot_hash(uint64_t k) {
    k ^= k >> 33;
    k *= 0xff51afd7ed558ccdull;
    k ^= k >> 33;
    k *= 0xc4ceb9fe1a85ec53ull;
    k ^= k >> 33;
    return k;
}
// Probe sequence over 8-slot lines: line_t = (h0 + t * S) mod L with S odd and key dependent,
// so that by Theorem 1 every line of a power-of-two table is visited exactly once in L steps.
__host__ __device__ inline uint64_t probe_start(uint64_t h, uint64_t line_mask) { return h & line_mask; }
__host__ __device__ inline uint64_t probe_stride(uint64_t h, uint64_t line_mask) { return ((h >> 32) | 1ull) & (line_mask | 1ull); }

// ---- row initialisation: element j of the row of `key` = output j+1 of the splitmix64 stream
// seeded with the key, top 24 bits centred, times init_scale * 2^-23 (one exact int->float
// conversion and one fp32 multiply, so host and device agree bit for bit).
__device__ inline float init_value(uint64_t key, int j, float init_c) {
    uint64_t z = key + (uint64_t)(j + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    int q = (int)(z >> 40) - (1 << 23);
    return __fmul_rn((float)q, init_c);
}

// ---- bf16 (round to nearest even) -----------------------------------------------------------
__device__ inline uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ inline float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ inline float bf16lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ inline float bf16hi(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }
__device__ inline uint32_t pack_bf16(float lo, float hi) { return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16); }

// ---- wave64 primitives ------------------------------------------------------------------------
__device__ inline int lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }
// members of `mask` among the lanes below the calling lane (`lane` must be the caller's own lane: the count is two
// mbcnt instructions instead of a 64-bit shift, two ands and two population counts)
__device__ inline int rank_in(uint64_t mask, int /*lane*/) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}
// The lanes of the wave whose BITS-wide digit equals this lane's, as the two halves of a 64-lane mask, and from
// them the lane's rank among those peers and their number.  One ballot per digit bit; the mask is kept in 32-bit
// halves and narrowed with (mask xnor bit) so that a bit costs four vector instructions (bit extract, compare,
// two three-input logic ops) - a 64-bit select between the ballot and its complement costs nine.
struct Peers {
    uint32_t lo, hi;
    __device__ inline unsigned rank() const { return __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u)); }
    __device__ inline unsigned count() const { return (unsigned)(__popc(lo) + __popc(hi)); }
};
template <int BITS>
__device__ inline Peers match_digit(unsigned d) {
    Peers p{~0u, ~0u};
#pragma unroll
    for (int bit = 0; bit < BITS; ++bit) {
        uint32_t sel = (uint32_t)__builtin_amdgcn_sbfe((int)d, bit, 1);   // all ones when the bit is set
        asm("" : "+v"(sel));     // keeps the compare on `sel` itself (otherwise it is re-derived from d with a shift)
        const uint64_t m = __ballot((int)sel);
        // p &= ~(m ^ sel): one three-input logic instruction per half (truth table 0x90 = a & (b xnor c))
        p.lo = __builtin_amdgcn_bitop3_b32(p.lo, (uint32_t)m, sel, 0x90);
        p.hi = __builtin_amdgcn_bitop3_b32(p.hi, (uint32_t)(m >> 32), sel, 0x90);
    }
    return p;
}
template <typename T>
__device__ inline T wave_bcast(T v, int src) { return __shfl(v, src, kWave); }
__device__ inline uint64_t shfl64(uint64_t v, int src) {
    uint32_t lo = __shfl((uint32_t)v, src, kWave), hi = __shfl((uint32_t)(v >> 32), src, kWave);
    return ((uint64_t)hi << 32) | lo;
}
// loads that bypass the per-CU vector cache (see find-or-insert): agent-scope atomic loads
__device__ inline uint64_t load_fresh(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline unsigned long long load_fresh(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline uint32_t load_fresh(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline int64_t read_count(const int64_t* n_dev, int64_t n_max) {
    if (!n_dev) return n_max;
    int64_t n = *n_dev;
    return n < 0 ? 0 : (n > n_max ? n_max : n);
}

// 16-byte vector moves
struct __attribute__((aligned(16))) V16 { uint32_t x, y, z, w; };
__device__ inline V16 ld16(const void* p) { return *reinterpret_cast<const V16*>(p); }
__device__ inline V16 ld16_nt(const void* p) {
    const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
    return V16{__builtin_nontemporal_load(q), __builtin_nontemporal_load(q + 1), __builtin_nontemporal_load(q + 2),
               __builtin_nontemporal_load(q + 3)};
}
__device__ inline void st16(void* p, V16 v) { *reinterpret_cast<V16*>(p) = v; }
__device__ inline void st16_nt(void* p, V16 v) {
    __builtin_nontemporal_store(v.x, reinterpret_cast<uint32_t*>(p) + 0);
    __builtin_nontemporal_store(v.y, reinterpret_cast<uint32_t*>(p) + 1);
    __builtin_nontemporal_store(v.z, reinterpret_cast<uint32_t*>(p) + 2);
    __builtin_nontemporal_store(v.w, reinterpret_cast<uint32_t*>(p) + 3);
}

// The same through a pointer that the compiler cannot prove to be global memory because it was itself loaded
// from memory (the chunk directory).  Left generic, such an access becomes a "flat" instruction, which counts on
// the LDS wait counter as well as on the memory one; the compiler then waits for it on the spot, and the loads of
// a batch go out one round trip after the other.  The address-space cast makes it a plain global access.
#define MTGR_AS_GLOBAL __attribute__((address_space(1)))
__device__ inline V16 ldg16(const void* p) {
    const MTGR_AS_GLOBAL uint32_t* q = (const MTGR_AS_GLOBAL uint32_t*)p;
    return V16{q[0], q[1], q[2], q[3]};
}
__device__ inline V16 ldg16_nt(const void* p) {
    const MTGR_AS_GLOBAL uint32_t* q = (const MTGR_AS_GLOBAL uint32_t*)p;
    return V16{__builtin_nontemporal_load(q), __builtin_nontemporal_load(q + 1), __builtin_nontemporal_load(q + 2),
               __builtin_nontemporal_load(q + 3)};
}
__device__ inline void stg16(void* p, V16 v) {
    MTGR_AS_GLOBAL uint32_t* q = (MTGR_AS_GLOBAL uint32_t*)p;
    q[0] = v.x;
    q[1] = v.y;
    q[2] = v.z;
    q[3] = v.w;
}
__device__ inline void stg16_nt(void* p, V16 v) {
    MTGR_AS_GLOBAL uint32_t* q = (MTGR_AS_GLOBAL uint32_t*)p;
    __builtin_nontemporal_store(v.x, q + 0);
    __builtin_nontemporal_store(v.y, q + 1);
    __builtin_nontemporal_store(v.z, q + 2);
    __builtin_nontemporal_store(v.w, q + 3);
}

inline int check_hip(hipError_t e) { return e == hipSuccess ? EMB_OK : EMB_ERR_HIP; }
#define MTGR_LAUNCH_CHECK()                         \
    do {                                            \
        if (hipGetLastError() != hipSuccess) return EMB_ERR_HIP; \
    } while (0)

// emb_tag_keys with a declared ID width: raw IDs that need more than min(id_bits, 63 - tag_bits) bits are
// counted and wrapped (dedup.hip; also the first half of emb_tag_dedup's two-call form).
int tag_keys_limited(const uint64_t* x, const int64_t* field_off, const uint8_t* field_tag, int n_fields, int64_t n,
                     int tag_bits, int id_bits, uint64_t* key_out, int64_t* err_count, void* stream);

} // namespace mtgr

// The host object behind emb_table_t.
struct emb_table {
    static constexpr int kSnaps = 4;
    emb_table_desc_t desc;
    mtgr::HtState* st;          // device
    mtgr::Slot* slots;          // device
    int cap_log2;
    int n_chunks;
    int n_adam_chunks;          // chunks that have moment rows registered (in order)
    float* hot_values;          // device, optional hot store
    uint32_t* hot_free;
    uint32_t hot_capacity;
    int row_bytes;
    uint64_t n_rehash;
    // Host-side upper bounds of the device counters: exact values as of some point of the
    // stream (`base_*`) plus the n_max of every find-or-insert issued after that point.  The
    // base advances without blocking: each state-changing call queues a copy of the counters to
    // pinned host memory followed by an event, and the newest completed copy is adopted.
    uint64_t base_live, base_tomb, base_rows;
    uint64_t pending;
    mtgr::HtHead* snap_host;               // pinned, kSnaps entries
    hipEvent_t snap_ev[kSnaps];
    uint64_t snap_seq[kSnaps];             // 0 = never recorded
    uint64_t snap_pending_after[kSnaps];   // n_max issued after the snapshot was queued
    uint64_t seq, min_valid_seq, base_seq;
    int snap_next;

    // live + deleted slots the key structure may hold: floor(max_load_factor * capacity)
    uint32_t slot_limit() const { return (uint32_t)((double)desc.max_load_factor * (double)(1ull << cap_log2)); }
    uint64_t live_bound() const { return base_live + pending; }
    uint64_t occupied_bound() const { return base_live + base_tomb + pending; }
    uint64_t rows_used_bound() const { return base_rows + pending; }

    void adopt(const mtgr::HtCounts& c, uint64_t pending_after, uint64_t s) {
        base_live = c.live;
        base_tomb = c.tombstones;
        const uint64_t freec = c.free_count > 0 ? (uint64_t)c.free_count : 0ull;
        base_rows = (uint64_t)c.bump > freec ? (uint64_t)c.bump - freec : 0ull;
        pending = pending_after;
        base_seq = s;
    }
    // adopt the newest completed snapshot, if any is newer than the current base
    void refresh() {
        int best = -1;
        for (int i = 0; i < kSnaps; ++i) {
            if (snap_seq[i] == 0 || snap_seq[i] < min_valid_seq || snap_seq[i] <= base_seq) continue;
            if (best >= 0 && snap_seq[i] < snap_seq[best]) continue;
            if (hipEventQuery(snap_ev[i]) == hipSuccess) best = i;
        }
        if (best >= 0) adopt(mtgr::HtCounts::from(snap_host[best]), snap_pending_after[best], snap_seq[best]);
    }
    void issued(uint64_t n_max) {
        pending += n_max;
        for (int i = 0; i < kSnaps; ++i) snap_pending_after[i] += n_max;
    }
    int snapshot(hipStream_t s) {
        const int i = snap_next;
        snap_next = (snap_next + 1) % kSnaps;
        if (hipMemcpyAsync(&snap_host[i], st, sizeof(mtgr::HtHead), hipMemcpyDeviceToHost, s) != hipSuccess) return EMB_ERR_HIP;
        if (hipEventRecord(snap_ev[i], s) != hipSuccess) return EMB_ERR_HIP;
        snap_seq[i] = ++seq;
        snap_pending_after[i] = 0;
        return EMB_OK;
    }

    mtgr::HtView view() const {
        mtgr::HtView v;
        v.slots = slots;
        v.st = st;
        v.line_mask = slots ? ((1ull << cap_log2) / mtgr::kLineSlots - 1ull) : 0ull;
        v.slot_limit = slots ? slot_limit() : 0u;
        v.rows_capacity = (uint32_t)((uint64_t)n_chunks << desc.chunk_rows_log2);
        v.chunk_log2 = desc.chunk_rows_log2;
        v.dim = desc.dim;
        v.dtype = desc.dtype;
        v.row_bytes = row_bytes;
        v.init_c = desc.init_scale * (1.0f / 8388608.0f);
        v.count = desc.count_probes;
        v.has_adam = (n_chunks > 0 && n_adam_chunks == n_chunks) ? 1 : 0;
        v.hot_values = hot_values;
        v.hot_free = hot_free;
        v.hot_capacity = hot_capacity;
        return v;
    }
};
