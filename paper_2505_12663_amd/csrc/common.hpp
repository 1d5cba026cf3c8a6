// Shared device/host helpers of the gfx950 sparse-embedding kernels (wave64 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mtgr_emb.h"

namespace mtgr {

constexpr int kWave = 64;
constexpr uint64_t kEmptyKey = 0xFFFFFFFFFFFFFFFFull; // never-used slot
constexpr uint64_t kTombKey = 0xFFFFFFFFFFFFFFFEull;  // deleted slot, reclaimed by rehash only
constexpr uint32_t kRowInvalid = 0xFFFFFFFFu;
constexpr int kLineSlots = 8;                         // one probe = one aligned 64-byte line of keys
constexpr int kMaxChunks = 256;

// Device-resident table state: counters + chunk directory.  Lives in caller memory.
struct HtState {
    unsigned long long live;
    unsigned long long tombstones;
    unsigned int bump;       // rows handed out by the bump allocator
    int free_count;          // entries on the free-row stack (may dip below 0 inside an insert kernel)
    unsigned int status;     // EMB_DEV_* bits
    unsigned int pad0;
    unsigned long long lookups, probes, cas_attempts, cas_failures, alloc_atomics;
    unsigned long long pad1[7];
    void* values[kMaxChunks];
    float* acc[kMaxChunks];
    uint32_t* last_seen[kMaxChunks];
    uint32_t* freq[kMaxChunks];
    uint32_t* free_list[kMaxChunks];
};

// What a table kernel needs, passed by value.
struct HtView {
    uint64_t* keys;
    uint32_t* rows;
    HtState* st;
    uint64_t line_mask;      // (capacity / kLineSlots) - 1
    uint32_t rows_capacity;  // rows in registered chunks
    int chunk_log2;
    int dim;
    int dtype;
    int row_bytes;
    float init_c;            // init_scale * 2^-23
    int count;               // maintain probe counters
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
__device__ inline uint64_t lanes_below(int lane) { return (1ull << lane) - 1ull; }
__device__ inline int rank_in(uint64_t mask, int lane) { return __popcll(mask & lanes_below(lane)); }
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
__device__ inline void st16(void* p, V16 v) { *reinterpret_cast<V16*>(p) = v; }
__device__ inline void st16_nt(void* p, V16 v) {
    __builtin_nontemporal_store(v.x, reinterpret_cast<uint32_t*>(p) + 0);
    __builtin_nontemporal_store(v.y, reinterpret_cast<uint32_t*>(p) + 1);
    __builtin_nontemporal_store(v.z, reinterpret_cast<uint32_t*>(p) + 2);
    __builtin_nontemporal_store(v.w, reinterpret_cast<uint32_t*>(p) + 3);
}

inline int check_hip(hipError_t e) { return e == hipSuccess ? EMB_OK : EMB_ERR_HIP; }
#define MTGR_LAUNCH_CHECK()                         \
    do {                                            \
        if (hipGetLastError() != hipSuccess) return EMB_ERR_HIP; \
    } while (0)

} // namespace mtgr

// The host object behind emb_table_t.
struct emb_table {
    emb_table_desc_t desc;
    mtgr::HtState* st;          // device
    uint64_t* keys;             // device
    uint32_t* rows;             // device
    int cap_log2;
    int n_chunks;
    int row_bytes;
    uint64_t n_rehash;
    // host-side upper bounds between two ht_stats calls
    uint64_t occupied_bound;    // live + tombstones
    uint64_t live_bound;
    uint64_t rows_used_bound;   // bump + never below what is on the free list

    mtgr::HtView view() const {
        mtgr::HtView v;
        v.keys = keys;
        v.rows = rows;
        v.st = st;
        v.line_mask = keys ? ((1ull << cap_log2) / mtgr::kLineSlots - 1ull) : 0ull;
        v.rows_capacity = (uint32_t)((uint64_t)n_chunks << desc.chunk_rows_log2);
        v.chunk_log2 = desc.chunk_rows_log2;
        v.dim = desc.dim;
        v.dtype = desc.dtype;
        v.row_bytes = row_bytes;
        v.init_c = desc.init_scale * (1.0f / 8388608.0f);
        v.count = desc.count_probes;
        return v;
    }
};
