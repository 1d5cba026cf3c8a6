// Dynamic embedding hash table for gfx950 (Sec. 3.1): key structure of 16-byte slots
// (key, row index) decoupled from the chunked embedding structure, open addressing over
// 128-byte lines of 8 slots with a key-dependent odd line stride (Theorem 1 gives full
// coverage), sub-wave cooperative probing (8 lanes inspect one line with one coalesced
// 128-byte load), CAS insertion into never-used slots only, deleted markers,
// block-aggregated row allocation, key-only rehash.
#include <cstddef>

#include "common.hpp"

using namespace mtgr;

namespace {

constexpr int kBlock = 256;
constexpr int kBigBlock = 1024;            // eviction: aggregates its pushes per block
constexpr int kBigWaves = kBigBlock / kWave;
// find-or-insert aggregates admission and row allocation per block and has block-wide barriers between its
// rounds, so every wave waits for the block's slowest key.  512 keys per block measured best: against 1024,
// a lookup of 5.7 M present keys at load 0.73 takes 188 us instead of 250, the same with 5 % new keys 260 us
// instead of 360, a 4 M-key bulk insert 735 us instead of 860; 256 helps the sparse case a little more
// (243 us) but costs the bulk insert its aggregation (1150 us).
constexpr int kFoiBlock = 512;
constexpr int kFoiWaves = kFoiBlock / kWave;
constexpr unsigned kTouchMaxGrid = 2048;   // the pass that resolves deferred elements: 256 CUs x 8 blocks of 256 threads

__device__ inline void* chunk_row_ptr(const HtView& v, uint32_t row) {
    char* base = static_cast<char*>(v.st->values[row >> v.chunk_log2]);
    return base + (size_t)(row & ((1u << v.chunk_log2) - 1u)) * (size_t)v.row_bytes;
}
#define CHUNK_META(v, row) ((v).st->meta[(row) >> (v).chunk_log2][(row) & ((1u << (v).chunk_log2) - 1u)])
#define CHUNK_FREE(v, pos) ((v).st->free_list[(pos) >> (v).chunk_log2][(pos) & ((1u << (v).chunk_log2) - 1u)])

// --------------------------------------------------------------------------------------------
__global__ void k_fill_slots(Slot* slots, uint64_t n) {
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const V16 e{0xFFFFFFFFu, 0xFFFFFFFFu, kRowInvalid, 0u};
    for (; i < n; i += stride) st16(slots + i, e);
}

__global__ void k_zero_bytes(uint32_t* p, size_t n_words) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) p[i] = 0u;
}

__global__ void k_set_adam(HtState* st, int c, float* m, float* v) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        st->adam_m[c] = m;
        st->adam_v[c] = v;
    }
}

__global__ void k_set_chunk(HtState* st, int c, void* values, RowMeta* meta, uint32_t* free_list, uint64_t rows) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        st->values[c] = values;
        st->meta[c] = meta;
        st->free_list[c] = free_list;
        st->adam_m[c] = nullptr;
        st->adam_v[c] = nullptr;
    }
    // unused rows keep freq == 0 (see k_find_or_insert)
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < rows; i += stride)
        st16(meta + i, V16{0u, 0u, 0u, 0u});
}

struct ProbeCounters {
    unsigned probes, cas, cas_fail;
    unsigned my_lines;   // slot lines inspected for this lane's own key (probe histogram)
};

// --------------------------------------------------------------------------------------------
// Probe for `key` with the 8 lanes of a group, line after line.  All 64 lanes of the wave call
// this together; `active` says whether this lane's group has work.  Returns (group-uniform) the
// slot of the key, -1 when absent, -2 when every line was visited without room.  With INSERT, an
// absent key is claimed in the first never-used slot of the first line on its probe sequence that
// has one; *created tells whether this call claimed it.
// Concurrent inserts: a key is only ever stored by a successful CAS on an EMPTY slot, EMPTY slots
// of a line are claimed in ascending order, and a line is re-read with loads that bypass the
// non-coherent caches after every failed CAS, so two groups inserting the same key meet in the
// same slot.  The loop ends: a retry only follows a CAS that lost to a different key, which takes
// one of the line's at most 8 EMPTY slots away for good; every other iteration finishes the
// group or moves on to one of the finitely many unvisited lines.
constexpr long long kSlotAbsent = -3;    // read-only lookup, settled: the key is not in the table

template <bool INSERT>
__device__ inline long long probe_group(const HtView& v, uint64_t key, bool active, int lane, bool* created,
                                        ProbeCounters* pc, uint32_t* row_out = nullptr) {
    const int sub = lane & (kLineSlots - 1);
    const int gbase = lane & ~(kLineSlots - 1);
    const uint64_t h = slot_hash(key);
    uint64_t line = probe_start(h, v.line_mask);
    const uint64_t stride = probe_stride(h, v.line_mask);
    uint64_t remaining = v.line_mask + 1; // lines not yet visited: bounds the loop
    long long result = -1;
    bool done = !active;
    *created = false;
    unsigned lines = 0;
    while (__any(!done)) {
        Slot* sp = v.slots + line * kLineSlots + sub;
        uint64_t k = kEmptyKey;
        uint32_t slot_row = kRowInvalid;
        if (!done) {
            if (INSERT) {
                k = load_fresh(&sp->key);
            } else {       // read-only: the whole slot in one load, so that a hit brings its row index along
                const V16 e = ld16(sp);
                k = ((uint64_t)e.y << 32) | e.x;
                slot_row = e.z;
            }
        }
        const uint64_t m_hit = __ballot(!done && k == key);
        const uint64_t m_empty = __ballot(!done && k == kEmptyKey);
        const unsigned hit8 = (unsigned)(m_hit >> gbase) & 0xFFu;
        const unsigned empty8 = (unsigned)(m_empty >> gbase) & 0xFFu;
        bool retry_line = false;
        if (!done) {
            pc->probes += (sub == 0);
            ++lines;
            if (hit8) {
                result = (long long)(line * kLineSlots + (__ffs(hit8) - 1));
                if (!INSERT && row_out) *row_out = __shfl(slot_row, gbase + (__ffs(hit8) - 1), kWave);
                done = true;
            } else if (empty8 && !INSERT) {
                done = true; // absent
            }
        }
        if (INSERT) {
            // groups that saw no hit but an EMPTY slot try to claim the first one
            const bool want = !done && !hit8 && empty8;
            const int e = want ? (__ffs(empty8) - 1) : 0;
            uint64_t old = 0;
            if (want && sub == e) {
                old = atomicCAS(&sp->key, (unsigned long long)kEmptyKey, (unsigned long long)key);
                pc->cas += 1;
                if (old != kEmptyKey) pc->cas_fail += 1;
            }
            old = shfl64(old, gbase + e);
            if (want) {
                if (old == kEmptyKey) {
                    result = (long long)(line * kLineSlots + e);
                    *created = true;
                    done = true;
                } else if (old == key) {
                    result = (long long)(line * kLineSlots + e); // another group inserted the same key first
                    done = true;
                } else {
                    retry_line = true; // slot went to a different key: look at the line again
                }
            }
        }
        if (!done && !retry_line) {
            line = (line + stride) & v.line_mask;
            if (--remaining == 0) {
                done = true;
                result = -2;
            }
        }
    }
    pc->my_lines = lines;   // group-uniform; the caller credits it to the lane that owns the key
    return result;
}

// First lines of the 8 keys of every group, all loads in flight at once, read-only: a key found there is
// settled without entering the line-by-line loop (at the load factors in use that is nearly all
// present keys).  A first line that shows no match but a never-used slot settles the key as absent;
// *empty_slot then names the first such slot, which is where an insert will try its claim.  The line
// is read with ordinary loads and may be out of date, which is harmless: occupied slots never change,
// so "no match among the occupied slots before the first empty one" stays true, and the claim itself
// (a compare-and-swap) decides whether that slot was still empty.  found_slot stays -1 for unsettled
// elements (first line full without a match).
__device__ inline void first_line_pass(const HtView& v, uint64_t my_key, bool my_ok, int lane, long long* found_slot,
                                       uint32_t* found_row, long long* empty_slot, ProbeCounters* pc) {
    const int sub = lane & (kLineSlots - 1);
    const int gbase = lane & ~(kLineSlots - 1);
    uint64_t kr[kLineSlots];
    uint64_t line[kLineSlots];
    V16 ent[kLineSlots];
#pragma unroll
    for (int r = 0; r < kLineSlots; ++r) {
        kr[r] = shfl64(my_key, gbase + r);
        line[r] = probe_start(slot_hash(kr[r]), v.line_mask);
        ent[r] = ld16(v.slots + line[r] * kLineSlots + sub);
    }
    *found_slot = -1;
    *found_row = kRowInvalid;
    *empty_slot = -1;
#pragma unroll
    for (int r = 0; r < kLineSlots; ++r) {
        const bool ok = __shfl((int)my_ok, gbase + r, kWave) != 0;
        const uint64_t k = ((uint64_t)ent[r].y << 32) | ent[r].x;
        const uint64_t m = __ballot(ok && k == kr[r]);
        const unsigned hit8 = (unsigned)(m >> gbase) & 0xFFu;
        const int hl = hit8 ? (__ffs(hit8) - 1) : 0;
        const uint32_t row = __shfl(ent[r].z, gbase + hl, kWave);
        if (sub == r && hit8) {
            *found_slot = (long long)(line[r] * kLineSlots + hl);
            *found_row = row;
        }
        pc->probes += (sub == r && ok) ? 1u : 0u;
        // a never-used slot in the first line and no match means the key is absent
        const uint64_t me = __ballot(ok && k == kEmptyKey);
        const unsigned empty8 = (unsigned)(me >> gbase) & 0xFFu;
        if (sub == r && !hit8 && empty8) {
            *found_slot = kSlotAbsent;
            *empty_slot = (long long)(line[r] * kLineSlots + (__ffs(empty8) - 1));
        }
    }
}

__device__ inline unsigned long long* stat_stripe(const HtView& v, unsigned id) {
    return v.st->head.stat[id & (kStatStripes - 1)];
}

// key_lines: slot lines inspected for this lane's key (0 = the lane had no key)
__device__ inline void flush_counters(const HtView& v, int lane, unsigned wave_no, int64_t cnt, ProbeCounters pc,
                                      unsigned key_lines) {
    unsigned tot_p = pc.probes, tot_c = pc.cas, tot_f = pc.cas_fail;
    unsigned long long* hc = stat_stripe(v, wave_no);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint64_t m = __ballot(b < 7 ? key_lines == (unsigned)(b + 1) : key_lines >= 8u);
        if (lane == 0 && m) atomicAdd(&hc[kStatHist0 + b], (unsigned long long)__popcll(m));
    }
    for (int o = 32; o > 0; o >>= 1) {
        tot_p += __shfl_xor(tot_p, o, kWave);
        tot_c += __shfl_xor(tot_c, o, kWave);
        tot_f += __shfl_xor(tot_f, o, kWave);
    }
    if (lane == 0 && cnt > 0) { // one atomic per counter per wave, on the wave's own stripe
        unsigned long long* c = stat_stripe(v, wave_no);
        atomicAdd(&c[kStatLookups], (unsigned long long)cnt);
        atomicAdd(&c[kStatProbes], (unsigned long long)tot_p);
        if (tot_c) atomicAdd(&c[kStatCas], (unsigned long long)tot_c);
        if (tot_f) atomicAdd(&c[kStatCasFail], (unsigned long long)tot_f);
    }
}

__device__ inline void touch_row(const HtView& v, uint32_t row, uint32_t step) {
    RowMeta* m = &CHUNK_META(v, row);
    atomicAdd(&m->freq, 1u);
    m->last_seen = step;
}

// One wave handles 64 keys: each lane owns one key; the 8 groups of 8 lanes first look at the first
// line of each of their 8 keys, then work through the unsettled keys one after the other.
//
// The call runs in two rounds so that the load-factor limit holds exactly (Sec. 3.1 "Capacity
// Expansion": the key structure is expanded when the load factor passes the limit).
//   Round 1 looks every key up without writing.  Keys that are present are settled here - the whole
//   call, when the batch brings no new keys.
//   Admission: the block adds the number of its absent keys to the count of occupied slots; what would
//   exceed floor(max_load_factor * capacity) is given back, and those elements are turned away
//   (row -1, counted in head.refused, status bit) without having claimed anything.  Live + deleted
//   slots therefore never exceed the limit.
//   Round 2 claims a never-used slot for every admitted key by compare-and-swap.  A key that a
//   duplicate in another wave has inserted meanwhile is simply found; its reservation is returned.
// Rows for the new keys of all waves of a block are taken from the allocator with one atomic per
// block (a 4 M-key bulk insert otherwise queues 130 k atomics on the bump pointer): free stack first,
// then the bump pointer, which never passes the registered rows; a claim that gets no row leaves a
// deleted marker in its slot and its element is turned away too.
// TOUCH = false: existing keys are found without counting a touch and a created row starts
// with touch count 0 (the update call of the step counts it, in the write it does anyway).
// retry: only the elements an earlier call left at -1 are processed, the others keep their results.
// admit = 0: the host has shown that every element of the call fits below the limit even if all are
// new keys; the block then skips the admission (an atomic whose result it would have to wait for) and
// just adds the slots it claimed to the count.
template <bool COUNT, bool TOUCH>
__global__ __launch_bounds__(kFoiBlock) void k_find_or_insert(HtView v, const uint64_t* __restrict__ key,
                                                              const int64_t* n_dev, int64_t n_max, uint32_t step,
                                                              int32_t* __restrict__ row_idx,
                                                              uint8_t* __restrict__ inserted, int retry, int admit) {
    __shared__ int s_absent[kFoiWaves], s_new[kFoiWaves], s_surplus[kFoiWaves];
    __shared__ unsigned s_bits[kFoiWaves];
    __shared__ int s_admitted, s_old_free, s_take, s_got;
    __shared__ unsigned s_bump;
    const int64_t n = read_count(n_dev, n_max);
    if ((int64_t)blockIdx.x * kFoiBlock >= n) return; // whole block beyond the count
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    // whether the free stack holds rows, read long before the allocation needs it (only eviction pushes
    // rows, and never while this kernel runs, so a zero stays a zero)
    const uint32_t free_hint =
        threadIdx.x == 0 ? load_fresh(reinterpret_cast<const uint32_t*>(&v.st->head.free_count)) : 0u;
    const int64_t wave_base = (int64_t)blockIdx.x * kFoiBlock + wave * kWave;
    const bool wave_on = wave_base < n;
    const int64_t i = wave_base + lane;
    const bool valid = i < n && !(retry && row_idx[i] >= 0);
    const uint64_t my_key = valid ? key[i] : 0ull;
    const bool bad = valid && (my_key >> 63);
    const bool my_ok = valid && !bad;
    const int sub = lane & (kLineSlots - 1);
    const int gbase = lane & ~(kLineSlots - 1);

    ProbeCounters pc{0u, 0u, 0u, 0u};
    unsigned key_lines = my_ok ? 1u : 0u;   // distinct slot lines of its probe sequence inspected for this lane's key
    long long my_slot = -1, my_empty = -1;
    uint32_t my_row = kRowInvalid;
    bool my_created = false;
    // ---- round 1: read-only lookup
    if (wave_on) {
        bool unused;
        first_line_pass(v, my_key, my_ok, lane, &my_slot, &my_row, &my_empty, &pc);
        const bool need_slow = my_ok && my_slot == -1;   // first line full without a match
        if (__any(need_slow)) {
            for (int r = 0; r < kLineSlots; ++r) {
                const bool act = __shfl((int)need_slow, gbase + r, kWave) != 0;
                if (!__any(act)) continue;
                const uint64_t k = shfl64(my_key, gbase + r);
                uint32_t row = kRowInvalid;
                const long long s = probe_group<false>(v, k, act, lane, &unused, &pc, &row);
                if (sub == r && act) {
                    my_slot = s == -1 ? kSlotAbsent : s;   // -2: every line visited, no match, no room
                    my_row = row;
                    key_lines = pc.my_lines;        // the line-by-line walk starts over at the first line
                }
            }
        }
    }
    // ---- admission of the absent keys against the load-factor limit
    const bool absent = my_ok && my_slot == kSlotAbsent;
    const uint64_t m_absent = __ballot(absent);
    unsigned wave_bits = 0;   // status bits raised by this wave: one atomic per block, not one per element
    if (__any(bad)) wave_bits |= EMB_DEV_BAD_KEY;
    const uint64_t m_full = __ballot(my_ok && my_slot == -2);   // no match and not one never-used slot in the table
    if (m_full) wave_bits |= EMB_DEV_PROBE_EXHAUSTED;
    if (lane == 0) {
        s_absent[wave] = __popcll(m_absent);
        s_surplus[wave] = __popcll(m_full);
        s_bits[wave] = wave_bits;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0, no_room = 0;
        unsigned bits = 0;
        for (int w = 0; w < kFoiWaves; ++w) {
            total += s_absent[w];
            no_room += s_surplus[w];
            bits |= s_bits[w];
        }
        if (no_room > 0) atomicAdd(&v.st->head.refused, (unsigned long long)no_room);
        int admitted = 0;
        if (total > 0 && !admit) {
            admitted = total;
        } else if (total > 0) {
            const unsigned old_occ = atomicAdd(&v.st->head.occupied, (unsigned)total);
            admitted = old_occ >= v.slot_limit ? 0 : (int)(v.slot_limit - old_occ);
            if (admitted > total) admitted = total;
            if (admitted < total) {
                atomicSub(&v.st->head.occupied, (unsigned)(total - admitted));
                atomicAdd(&v.st->head.refused, (unsigned long long)(total - admitted));
                bits |= EMB_DEV_NEED_REHASH;
            }
            if (COUNT) atomicAdd(&stat_stripe(v, blockIdx.x)[kStatAlloc], 1ull);
        }
        if (bits) atomicOr(&v.st->head.status, bits);
        s_admitted = admitted;
    }
    __syncthreads();
    int absent_rank = rank_in(m_absent, lane);
    for (int w = 0; w < wave; ++w) absent_rank += s_absent[w];
    const bool claim = absent && absent_rank < s_admitted;
    // ---- round 2: the admitted keys claim a slot (block-uniform branch: most blocks of a step bring no new key)
    if (s_admitted > 0) {
        if (wave_on && __any(claim)) {
            // a key whose first line showed a never-used slot tries that slot at once, every lane for itself: the
            // compare-and-swap tells whether it was still free (claimed), holds the key by now (a duplicate in
            // another wave was faster: found) or went to another key (then, as for keys whose first line was full,
            // the line-by-line walk with fresh loads takes over)
            bool need_slow = claim;
            if (claim && my_empty >= 0) {
                const uint64_t old = atomicCAS(&v.slots[my_empty].key, (unsigned long long)kEmptyKey, (unsigned long long)my_key);
                pc.cas += 1;
                if (old == kEmptyKey) {
                    my_slot = my_empty;
                    my_created = true;
                    need_slow = false;
                } else {
                    pc.cas_fail += 1;
                    if (old == my_key) {
                        my_slot = my_empty;
                        my_row = kRowInvalid;      // resolved below, or by k_touch if the creator has not published it yet
                        need_slow = false;
                    }
                }
            }
            if (__any(need_slow)) {
                for (int r = 0; r < kLineSlots; ++r) {
                    const bool act = __shfl((int)need_slow, gbase + r, kWave) != 0;
                    if (!__any(act)) continue;
                    const uint64_t k = shfl64(my_key, gbase + r);
                    bool created;
                    const long long s = probe_group<true>(v, k, act, lane, &created, &pc);
                    if (sub == r && act) {
                        my_slot = s;
                        my_created = created;
                        my_row = kRowInvalid;
                        key_lines = key_lines > pc.my_lines ? key_lines : pc.my_lines;   // distinct lines of the key's sequence
                    }
                }
            }
        }
        // ---- block-aggregated row allocation for the lanes that claimed a slot; reservations of admitted
        // keys that turned out to be present (or found no slot) are returned
        const uint64_t m_new = __ballot(my_created);
        const uint64_t m_surplus = __ballot(claim && !my_created);
        const uint64_t m_lost = __ballot(claim && my_slot == -2);   // cannot happen while reservations hold; counted all the same
        if (lane == 0) {
            s_new[wave] = __popcll(m_new);
            s_surplus[wave] = __popcll(m_surplus);
            s_bits[wave] = (unsigned)__popcll(m_lost);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int total = 0, surplus = 0;
            unsigned lost = 0;
            for (int w = 0; w < kFoiWaves; ++w) {
                total += s_new[w];
                surplus += s_surplus[w];
                lost += s_bits[w];
            }
            if (admit) {
                if (surplus > 0) atomicSub(&v.st->head.occupied, (unsigned)surplus);
            } else if (total > 0) {
                atomicAdd(&v.st->head.occupied, (unsigned)total);   // the slots claimed; nothing waits for the result
            }
            if (lost > 0) {
                atomicAdd(&v.st->head.refused, (unsigned long long)lost);
                atomicOr(&v.st->head.status, EMB_DEV_PROBE_EXHAUSTED);
            }
            int old_free = 0, take = 0, got = 0;
            unsigned bump_base = 0;
            if (total > 0) {
                unsigned n_atomics = 0;
                if (free_hint != 0u) {
                    old_free = atomicSub(&v.st->head.free_count, total);
                    ++n_atomics;
                }
                take = old_free < 0 ? 0 : (old_free > total ? total : old_free);
                got = take;
                const int need = total - take;
                if (need > 0) {
                    bump_base = atomicAdd(&v.st->head.bump, (unsigned)need);
                    ++n_atomics;
                    int avail = bump_base >= v.rows_capacity ? 0 : (int)(v.rows_capacity - bump_base);
                    if (avail > need) avail = need;
                    if (avail < need)   // give the overshoot back: the pointer ends at the registered rows
                        atomicSub(&v.st->head.bump, (unsigned)(need - avail));
                    got += avail;
                }
                unsigned long long* c = stat_stripe(v, blockIdx.x);
                if (got > 0) atomicAdd(&c[kStatLive], (unsigned long long)got);
                if (got < total) {
                    atomicAdd(&c[kStatTomb], (unsigned long long)(total - got));
                    atomicAdd(&v.st->head.refused, (unsigned long long)(total - got));
                    atomicOr(&v.st->head.status, EMB_DEV_OUT_OF_ROWS);
                }
                if (COUNT) atomicAdd(&c[kStatAlloc], (unsigned long long)n_atomics);
            }
            s_old_free = old_free;
            s_take = take;
            s_got = got;
            s_bump = bump_base;
        }
        __syncthreads();
        if (my_created) {
            int r = rank_in(m_new, lane);
            for (int w = 0; w < wave; ++w) r += s_new[w];
            const int take = s_take;
            if (r < take) {
                my_row = CHUNK_FREE(v, (unsigned)(s_old_free - 1 - r));
            } else if (r < s_got) {
                my_row = s_bump + (unsigned)(r - take);
            } else {
                // no row left: give the slot up again (as a deleted marker); the element reports -1
                v.slots[my_slot].key = kTombKey;
                my_row = kRowInvalid;
                my_created = false;
                my_slot = -1;
            }
        }
        // ---- initialise the new rows, the whole wave writing one row at a time (coalesced).  Every
        // creating lane resolves its own row address first, so the loop has no dependent loads.
        const uint64_t my_dst = my_created ? reinterpret_cast<uint64_t>(chunk_row_ptr(v, my_row)) : 0ull;
        uint64_t my_m = 0ull, my_v = 0ull; // moment rows of the new row, when an Adam state is registered
        if (my_created && v.has_adam) {
            const size_t o = (size_t)(my_row & ((1u << v.chunk_log2) - 1u)) * (size_t)v.dim;
            my_m = reinterpret_cast<uint64_t>(v.st->adam_m[my_row >> v.chunk_log2] + o);
            my_v = reinterpret_cast<uint64_t>(v.st->adam_v[my_row >> v.chunk_log2] + o);
        }
        uint64_t m_init = __ballot(my_created);
        while (m_init) {
            const int src = __ffsll((unsigned long long)m_init) - 1;
            m_init &= m_init - 1;
            const uint64_t k = shfl64(my_key, src);
            char* dst = reinterpret_cast<char*>(shfl64(my_dst, src));
            if (v.has_adam) {
                float* pm = reinterpret_cast<float*>(shfl64(my_m, src));
                float* pv = reinterpret_cast<float*>(shfl64(my_v, src));
                for (int j = lane; j < v.dim; j += kWave) {
                    pm[j] = 0.0f;
                    pv[j] = 0.0f;
                }
            }
            if (v.dtype == EMB_F32) {
                for (int j = lane; j < v.dim; j += kWave) reinterpret_cast<float*>(dst)[j] = init_value(k, j, v.init_c);
            } else {
                for (int j = lane; j < v.dim; j += kWave)
                    reinterpret_cast<uint16_t*>(dst)[j] = f32_to_bf16(init_value(k, j, v.init_c));
            }
        }
        if (my_created) {
            // A row that is not in use always has freq == 0 (chunks are registered zeroed, eviction
            // resets it), so creator and duplicates alike count their touch with an atomic add and no
            // ordering between this record and the publication of the row index is needed - a release
            // fence here would write the whole L2 back per wave.
            RowMeta* m = &CHUNK_META(v, my_row);
            m->acc = 0.0f;
            m->last_seen = step;
            if (TOUCH) atomicAdd(&m->freq, 1u);
            __hip_atomic_store(&v.slots[my_slot].row, my_row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // ---- results.  A lane that found a key whose creator has not published the row yet records
    // the slot (as -(slot+2)); k_touch resolves it after this kernel.
    if (valid) {
        int32_t out;
        if (bad || my_slot < 0) {     // bad key, turned away, no row, probe sequence exhausted
            out = -1;
        } else if (my_created) {
            out = (int32_t)my_row;
        } else {
            if (my_row == kRowInvalid) my_row = load_fresh(&v.slots[my_slot].row);
            if (my_row == kRowInvalid) {
                out = (int32_t)(-(my_slot + 2));
            } else {
                out = (int32_t)my_row;
                if (TOUCH) touch_row(v, my_row, step);
            }
        }
        row_idx[i] = out;
        if (inserted) inserted[i] = my_created ? 1 : 0;
    }
    if (COUNT && wave_on)
        flush_counters(v, lane, blockIdx.x * kFoiWaves + wave, n - wave_base < kWave ? n - wave_base : kWave, pc, key_lines);
}

// Second half of find-or-insert: resolve the deferred elements and count their touch.
__global__ __launch_bounds__(kBlock) void k_touch(HtView v, const int64_t* n_dev, int64_t n_max, uint32_t step,
                                                  int32_t* __restrict__ row_idx, int touch) {
    const int64_t n = read_count(n_dev, n_max);
    if (blockIdx.x == 0 && threadIdx.x == 0 && v.st->head.free_count < 0)
        v.st->head.free_count = 0; // the free list ran dry during the insert
    // bounded grid, strided over the elements below the device-side count: the call is launched over the caller's
    // upper bound, which may be several times the count (35 k blocks that read the count and leave: 9 us; this: 4 us)
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock) {
        const int32_t r = row_idx[i];
        if (r > -2) continue;
        const uint32_t rr = v.slots[(uint64_t)(-(long long)r - 2)].row;
        if (rr == kRowInvalid) {
            row_idx[i] = -1; // the creator ran out of rows
        } else {
            row_idx[i] = (int32_t)rr;
            if (touch) touch_row(v, rr, step);
        }
    }
}

template <bool COUNT>
__global__ __launch_bounds__(kBlock) void k_find(HtView v, const uint64_t* __restrict__ key, const int64_t* n_dev,
                                                 int64_t n_max, int32_t* __restrict__ row_idx) {
    const int64_t n = read_count(n_dev, n_max);
    const int lane = lane_id();
    const int64_t wave_base = ((int64_t)blockIdx.x * kBlock + (threadIdx.x & ~(kWave - 1)));
    if (wave_base >= n) return;
    const int64_t i = wave_base + lane;
    const bool valid = i < n;
    const uint64_t my_key = valid ? key[i] : 0ull;
    const bool my_ok = valid && !(my_key >> 63);
    const int sub = lane & (kLineSlots - 1);
    const int gbase = lane & ~(kLineSlots - 1);
    ProbeCounters pc{0u, 0u, 0u, 0u};
    unsigned key_lines = my_ok ? 1u : 0u;
    long long my_slot;
    uint32_t my_row;
    bool unused_created;
    long long unused_empty;
    first_line_pass(v, my_key, my_ok, lane, &my_slot, &my_row, &unused_empty, &pc);
    const bool need_slow = my_ok && my_slot == -1;
    if (__any(need_slow)) {
        for (int r = 0; r < kLineSlots; ++r) {
            const bool act = __shfl((int)need_slow, gbase + r, kWave) != 0;
            if (!__any(act)) continue;
            const uint64_t k = shfl64(my_key, gbase + r);
            bool created;
            uint32_t row = kRowInvalid;
            const long long s = probe_group<false>(v, k, act, lane, &created, &pc, &row);
            if (sub == r && act) {
                my_slot = s;
                my_row = row;
                key_lines = pc.my_lines;
            }
        }
    }
    if (valid) row_idx[i] = (my_slot >= 0 && my_row != kRowInvalid) ? (int32_t)my_row : -1;
    if (COUNT) flush_counters(v, lane, blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave, n - wave_base < kWave ? n - wave_base : kWave, pc, key_lines);
}

// --------------------------------------------------------------------------------------------
// Eviction: one lane per slot.  Matching keys become deleted markers; their rows go to the free
// stack and their keys to the output list, with one atomic on each per block of 1024 slots.
__global__ __launch_bounds__(kBigBlock) void k_evict(HtView v, uint64_t n_slots, uint32_t now, uint32_t ttl,
                                                     uint32_t min_freq, uint32_t grace, uint64_t* evicted_keys,
                                                     int64_t evicted_cap, unsigned long long* n_evicted) {
    __shared__ int s_cnt[kBigWaves];
    __shared__ int s_free_base;
    __shared__ unsigned long long s_out_base;
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const uint64_t slot = (uint64_t)blockIdx.x * kBigBlock + threadIdx.x;
    bool go = false;
    uint64_t k = kEmptyKey;
    uint32_t row = kRowInvalid;
    uint32_t hot = 0;
    if (slot < n_slots) {
        const V16 e = ld16(v.slots + slot);
        k = ((uint64_t)e.y << 32) | e.x;
        row = e.z;
        if (k != kEmptyKey && k != kTombKey && row != kRowInvalid) {
            const RowMeta m = CHUNK_META(v, row);
            hot = m.hot;
            const uint32_t age = now - m.last_seen;
            const bool stale = ttl > 0 && age >= ttl;
            const bool rare = min_freq > 0 && m.freq < min_freq && age >= grace;
            go = stale || rare;
        }
    }
    const uint64_t m = __ballot(go);
    if (lane == 0) s_cnt[wave] = __popcll(m);
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
        for (int w = 0; w < kBigWaves; ++w) total += s_cnt[w];
        int free_base = 0;
        unsigned long long out_base = 0;
        if (total > 0) {
            free_base = atomicAdd(&v.st->head.free_count, total);
            out_base = atomicAdd(n_evicted, (unsigned long long)total);
            unsigned long long* c = stat_stripe(v, blockIdx.x);
            atomicAdd(&c[kStatLive], ~(unsigned long long)total + 1ull);
            atomicAdd(&c[kStatTomb], (unsigned long long)total);
        }
        s_free_base = free_base;
        s_out_base = out_base;
    }
    __syncthreads();
    if (go) {
        int r = rank_in(m, lane);
        for (int w = 0; w < wave; ++w) r += s_cnt[w];
        st16(v.slots + slot, V16{0xFFFFFFFEu, 0xFFFFFFFFu, kRowInvalid, 0u});
        CHUNK_FREE(v, (unsigned)(s_free_base + r)) = row;
        CHUNK_META(v, row) = RowMeta{0.0f, 0u, 0u, 0u}; // unused rows keep freq == 0
        if (hot != 0 && v.hot_free) // hot rows are few: one atomic each
            v.hot_free[atomicAdd(&v.st->head.hot_free_count, 1)] = hot - 1u;
        if (evicted_keys && (int64_t)(s_out_base + r) < evicted_cap) evicted_keys[s_out_base + r] = k;
    }
}

// Key-structure migration: one lane per old slot; a live pair is placed in the first never-used
// slot of the first line with one on its probe sequence in the new structure.  No key occurs
// twice, so no match test is needed.  Values are not touched (Sec. 3.1 "Capacity Expansion").
// DISPLACED_ONLY: second pass of the streaming migration - only keys that did not sit in their home line.
template <bool DISPLACED_ONLY>
__global__ __launch_bounds__(kBlock) void k_rehash(const Slot* __restrict__ old_slots, uint64_t n_old, Slot* new_slots,
                                                   uint64_t new_line_mask, HtState* st) {
    const uint64_t s = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (s >= n_old) return;
    const V16 e = ld16(old_slots + s);
    const uint64_t k = ((uint64_t)e.y << 32) | e.x;
    const uint32_t row = e.z;
    if (k == kEmptyKey || k == kTombKey || row == kRowInvalid) return;
    const uint64_t h = slot_hash(k);
    if (DISPLACED_ONLY && probe_start(h, n_old / kLineSlots - 1ull) == s / kLineSlots) return;   // placed by the first pass
    uint64_t line = probe_start(h, new_line_mask);
    const uint64_t stride = probe_stride(h, new_line_mask);
    for (uint64_t t = 0; t <= new_line_mask; ++t) {
        for (int j = 0; j < kLineSlots; ++j) {
            Slot* p = new_slots + line * kLineSlots + j;
            if (load_fresh(&p->key) != kEmptyKey) continue;
            const uint64_t old = atomicCAS(&p->key, (unsigned long long)kEmptyKey, (unsigned long long)k);
            if (old == kEmptyKey) {
                p->row = row;
                return;
            }
        }
        line = (line + stride) & new_line_mask;
    }
    atomicOr(&st->head.status, EMB_DEV_PROBE_EXHAUSTED);
}

// Migration into a structure of 2^k times the size (k >= 0), in two streaming passes instead of one
// random insert per key.  The home line of a key is the low bits of its hash, so the keys whose home
// is old line l have home l + j * L_old (j < 2^k) in the new structure, and nobody else has.
// Pass 1: the 8 lanes that hold old line l write those 2^k new lines completely - the keys that sat
// in their home line, packed to the front, then never-used slots.  Every new line is written exactly
// once, in whole 128-byte lines (no separate fill, no compare-and-swap, no reads of the new memory).
// Pass 2 (k_rehash with DISPLACED_ONLY): the keys that were not in their home line (it had been full
// when they arrived) are inserted by probing, as in the general migration.  A key in its home line is
// found by the first probe; the others are placed by the ordinary insert rule, so lookups see a table
// like any other.
__global__ __launch_bounds__(kBlock) void k_rehash_split(const Slot* __restrict__ old_slots, uint64_t n_old,
                                                         Slot* __restrict__ new_slots, int old_line_bits, int k) {
    const uint64_t slot = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (slot >= n_old) return;            // n_old is a multiple of the wave size: whole waves leave
    const int lane = lane_id();
    const int sub = lane & (kLineSlots - 1);
    const int gbase = lane & ~(kLineSlots - 1);
    const uint64_t line = slot / kLineSlots;
    const uint64_t old_lines = 1ull << old_line_bits;
    const V16 e = ld16(old_slots + slot);
    const uint64_t key = ((uint64_t)e.y << 32) | e.x;
    const uint32_t row = e.z;
    const bool live = key != kEmptyKey && key != kTombKey && row != kRowInvalid;
    const uint64_t h = slot_hash(key);
    const bool at_home = live && probe_start(h, old_lines - 1ull) == line;
    const unsigned target = (unsigned)((h >> old_line_bits) & ((1ull << k) - 1ull));   // which of the 2^k new lines
    const V16 never_used{0xFFFFFFFFu, 0xFFFFFFFFu, kRowInvalid, 0u};
    for (unsigned j = 0; j < (1u << k); ++j) {
        const uint64_t m = __ballot(at_home && target == j);
        unsigned m8 = (unsigned)(m >> gbase) & 0xFFu;
        for (int i = 0; i < sub; ++i) m8 &= m8 - 1u;          // drop the `sub` lowest members: the next one is this lane's
        const int src = m8 ? (__ffs(m8) - 1) : 0;
        const uint64_t kk = shfl64(key, gbase + src);
        const uint32_t rr = __shfl(row, gbase + src, kWave);
        const V16 out = m8 ? V16{(uint32_t)kk, (uint32_t)(kk >> 32), rr, 0u} : never_used;
        st16(new_slots + (line + (uint64_t)j * old_lines) * kLineSlots + sub, out);
    }
}

// After a rehash (or on fresh key storage) no deleted markers are left: occupied = live.  One wave.
__global__ void k_after_rehash(HtState* st) {
    static_assert(kStatStripes == kWave, "one lane per stripe");
    const int lane = lane_id();
    uint64_t live = st->head.stat[lane][kStatLive];   // stripes hold signed deltas: the sum wraps to the count
    st->head.stat[lane][kStatTomb] = 0ull;
    for (int o = 32; o > 0; o >>= 1) live += shfl64(live, lane ^ o);
    if (lane == 0) st->head.occupied = (unsigned)live;
}

__global__ void k_clear_status(HtState* st, unsigned bits) {
    if (blockIdx.x == 0 && threadIdx.x == 0) st->head.status &= ~bits;
}

// Unordered dump: one lane per slot decides, then the wave copies the rows of its live slots.
__global__ __launch_bounds__(kBlock) void k_export(HtView v, uint64_t n_slots, uint64_t* keys, char* values,
                                                   float* acc, uint32_t* last_seen, uint32_t* freq, int64_t cap,
                                                   unsigned long long* n_out) {
    const int lane = lane_id();
    const uint64_t slot = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    bool liveslot = false;
    uint64_t k = 0;
    uint32_t row = kRowInvalid;
    if (slot < n_slots) {
        const V16 e = ld16(v.slots + slot);
        k = ((uint64_t)e.y << 32) | e.x;
        row = e.z;
        liveslot = k != kEmptyKey && k != kTombKey && row != kRowInvalid;
    }
    uint64_t m = __ballot(liveslot);
    if (!m) return;
    const int leader = __ffsll((unsigned long long)m) - 1;
    unsigned long long base = 0;
    if (lane == leader) base = atomicAdd(n_out, (unsigned long long)__popcll(m));
    base = shfl64(base, leader);
    const unsigned long long pos = base + rank_in(m, lane);
    if (liveslot && (int64_t)pos < cap) {
        keys[pos] = k;
        const RowMeta rm = CHUNK_META(v, row);
        if (acc) acc[pos] = rm.acc;
        if (last_seen) last_seen[pos] = rm.last_seen;
        if (freq) freq[pos] = rm.freq;
    }
    if (!values) return;
    while (m) {
        const int src = __ffsll((unsigned long long)m) - 1;
        m &= m - 1;
        const uint32_t r = __shfl(row, src, kWave);
        const unsigned long long p = shfl64(pos, src);
        if ((int64_t)p >= cap) continue;
        const uint32_t* s32 = static_cast<const uint32_t*>(chunk_row_ptr(v, r));
        uint32_t* d32 = reinterpret_cast<uint32_t*>(values + (size_t)p * v.row_bytes);
        const uint32_t hot_r = v.hot_values ? CHUNK_META(v, r).hot : 0u;
        if (hot_r != 0) { // 16-bit table with an fp32 master for this row: dump the master, rounded
            const float* hp = v.hot_values + (size_t)(hot_r - 1u) * v.dim;
            for (int w = lane; w < v.dim / 2; w += kWave) d32[w] = pack_bf16(hp[2 * w], hp[2 * w + 1]);
        } else {
            for (int w = lane; w < v.row_bytes / 4; w += kWave) d32[w] = s32[w];
        }
    }
}

inline unsigned blocks_for(uint64_t n, int per_block) { return (unsigned)((n + per_block - 1) / per_block); }

// Dump of the fp32 master rows: one lane per slot decides, the wave copies.
__global__ __launch_bounds__(kBlock) void k_export_hot(HtView v, uint64_t n_slots, uint64_t* keys, float* values,
                                                       int64_t cap, unsigned long long* n_out) {
    const int lane = lane_id();
    const uint64_t slot = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    uint64_t k = 0;
    uint32_t hot = 0;
    if (slot < n_slots) {
        const V16 e = ld16(v.slots + slot);
        k = ((uint64_t)e.y << 32) | e.x;
        if (k != kEmptyKey && k != kTombKey && e.z != kRowInvalid) hot = CHUNK_META(v, e.z).hot;
    }
    uint64_t m = __ballot(hot != 0);
    if (!m) return;
    const int leader = __ffsll((unsigned long long)m) - 1;
    unsigned long long base = 0;
    if (lane == leader) base = atomicAdd(n_out, (unsigned long long)__popcll(m));
    base = shfl64(base, leader);
    const unsigned long long pos = base + rank_in(m, lane);
    if (hot != 0 && (int64_t)pos < cap) keys[pos] = k;
    if (!values) return;
    while (m) {
        const int src = __ffsll((unsigned long long)m) - 1;
        m &= m - 1;
        const uint32_t h = __shfl(hot, src, kWave) - 1u;
        const unsigned long long p = shfl64(pos, src);
        if ((int64_t)p >= cap) continue;
        const float* hp = v.hot_values + (size_t)h * v.dim;
        for (int w = lane; w < v.dim; w += kWave) values[(size_t)p * v.dim + w] = hp[w];
    }
}

} // namespace

// ================================================================================================
extern "C" {

int emb_tag_bits(int m) {
    if (m < 0) return EMB_ERR_INVALID_ARG;
    int k = 0;
    while ((1ll << k) <= (long long)m) ++k; // smallest k with 2^k >= m+1
    return k;
}

int emb_plan_merge(const int32_t* dims, const int32_t* dtypes, int m, int32_t* merged_of) {
    if (!dims || !dtypes || !merged_of || m < 0) return EMB_ERR_INVALID_ARG;
    int n_groups = 0;
    for (int t = 0; t < m; ++t) {
        int g = -1;
        for (int p = 0; p < t && g < 0; ++p)
            if (dims[p] == dims[t] && dtypes[p] == dtypes[t]) g = merged_of[p];
        merged_of[t] = g >= 0 ? g : n_groups++;
    }
    return n_groups;
}

uint64_t ht_probe_line(uint64_t key, int capacity_log2, uint64_t t) {
    if (capacity_log2 < 3 || capacity_log2 > 62) return ~0ull;
    const uint64_t line_mask = ((1ull << capacity_log2) / kLineSlots) - 1ull;
    const uint64_t h = slot_hash(key);
    return (probe_start(h, line_mask) + t * probe_stride(h, line_mask)) & line_mask;
}

const char* emb_status_string(int s) {
    switch (s) {
        case EMB_OK: return "ok";
        case EMB_ERR_INVALID_ARG: return "invalid argument";
        case EMB_ERR_KEY_RANGE: return "key out of range";
        case EMB_ERR_WORKSPACE: return "workspace too small or misaligned";
        case EMB_ERR_NO_STORAGE: return "no key storage or not enough row chunks";
        case EMB_ERR_HIP: return "HIP runtime error";
        case EMB_ERR_NEED_REHASH: return "load factor limit: rehash to a larger key structure";
        case EMB_ERR_TOO_LARGE: return "size beyond the fixed scratch of the allocation-free entry point";
        case EMB_CHECK_STATUS: return "launched; new keys may have been turned away: compare ht_stats().refused";
        default: return "unknown status";
    }
}

size_t emb_table_state_bytes(void) { return (sizeof(HtState) + 255) & ~(size_t)255; }

int emb_table_create(emb_table_t** out, const emb_table_desc_t* desc, void* state, size_t state_bytes,
                     void* stream) {
    if (!out || !desc || !state) return EMB_ERR_INVALID_ARG;
    if (state_bytes < emb_table_state_bytes() || (reinterpret_cast<uintptr_t>(state) & 255)) return EMB_ERR_INVALID_ARG;
    if (desc->dim <= 0 || (desc->dtype != EMB_F32 && desc->dtype != EMB_BF16)) return EMB_ERR_INVALID_ARG;
    const int row_bytes = desc->dim * (desc->dtype == EMB_F32 ? 4 : 2);
    if (row_bytes % 16 != 0 || desc->dim > 256) return EMB_ERR_INVALID_ARG;
    if (desc->chunk_rows_log2 < 4 || desc->chunk_rows_log2 > 30) return EMB_ERR_INVALID_ARG;
    if (desc->max_load_factor < 0.0f || desc->max_load_factor > 1.0f) return EMB_ERR_INVALID_ARG;
    emb_table* t = new emb_table();
    t->desc = *desc;
    if (t->desc.max_load_factor == 0.0f) t->desc.max_load_factor = 0.75f;
    if (t->desc.init_scale == 0.0f) t->desc.init_scale = 0.01f;
    t->st = static_cast<HtState*>(state);
    t->slots = nullptr;
    t->cap_log2 = 0;
    t->n_chunks = 0;
    t->n_adam_chunks = 0;
    t->row_bytes = row_bytes;
    t->n_rehash = 0;
    t->base_live = t->base_tomb = t->base_rows = t->pending = 0;
    t->seq = t->base_seq = 0;
    t->min_valid_seq = 1;
    t->snap_next = 0;
    t->snap_host = nullptr;
    if (hipHostMalloc(reinterpret_cast<void**>(&t->snap_host), sizeof(HtHead) * emb_table::kSnaps, hipHostMallocDefault) !=
        hipSuccess) {
        delete t;
        return EMB_ERR_HIP;
    }
    for (int i = 0; i < emb_table::kSnaps; ++i) {
        t->snap_seq[i] = 0;
        t->snap_pending_after[i] = 0;
        if (hipEventCreateWithFlags(&t->snap_ev[i], hipEventDisableTiming) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(t->snap_ev[j]);
            (void)hipHostFree(t->snap_host);
            delete t;
            return EMB_ERR_HIP;
        }
    }
    const size_t words = emb_table_state_bytes() / 4;
    hipLaunchKernelGGL(k_zero_bytes, dim3(blocks_for(words, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint32_t*>(state), words);
    if (hipGetLastError() != hipSuccess) {
        emb_table_destroy(t);
        return EMB_ERR_HIP;
    }
    *out = t;
    return EMB_OK;
}

int emb_table_destroy(emb_table_t* t) {
    if (!t) return EMB_OK;
    for (int i = 0; i < emb_table::kSnaps; ++i) (void)hipEventDestroy(t->snap_ev[i]);
    if (t->snap_host) (void)hipHostFree(t->snap_host);
    delete t;
    return EMB_OK;
}

static unsigned fill_grid(uint64_t n) {
    const unsigned g = blocks_for(n, 256 * 8);
    return g > (1u << 20) ? (1u << 20) : g;
}

int ht_set_key_storage(emb_table_t* t, void* slots, int capacity_log2, void* stream) {
    if (!t || !slots || capacity_log2 < 6 || capacity_log2 > 30) return EMB_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(slots) & 127) return EMB_ERR_INVALID_ARG;
    if (t->slots && t->live_bound() > 0) return EMB_ERR_INVALID_ARG; // non-empty table: use ht_rehash
    const uint64_t n = 1ull << capacity_log2;
    hipLaunchKernelGGL(k_fill_slots, dim3(fill_grid(n)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<Slot*>(slots), n);
    MTGR_LAUNCH_CHECK();
    // an emptied table may still count deleted markers of its old key structure: they are gone with it
    hipLaunchKernelGGL(k_after_rehash, dim3(1), dim3(kWave), 0, static_cast<hipStream_t>(stream), t->st);
    MTGR_LAUNCH_CHECK();
    t->slots = static_cast<Slot*>(slots);
    t->cap_log2 = capacity_log2;
    t->base_tomb = 0;
    t->min_valid_seq = t->seq + 1;
    return EMB_OK;
}

int ht_add_chunk(emb_table_t* t, void* values, void* meta, uint32_t* free_list, void* stream) {
    if (!t || !values || !meta || !free_list) return EMB_ERR_INVALID_ARG;
    if (t->n_chunks >= kMaxChunks) return EMB_ERR_NO_STORAGE;
    if (((uint64_t)(t->n_chunks + 1) << t->desc.chunk_rows_log2) > 0x7FFFFFFFull) return EMB_ERR_NO_STORAGE;
    if ((reinterpret_cast<uintptr_t>(values) & 15) || (reinterpret_cast<uintptr_t>(meta) & 15)) return EMB_ERR_INVALID_ARG;
    const uint64_t rows = 1ull << t->desc.chunk_rows_log2;
    hipLaunchKernelGGL(k_set_chunk, dim3(fill_grid(rows)), dim3(256), 0, static_cast<hipStream_t>(stream), t->st,
                       t->n_chunks, values, static_cast<RowMeta*>(meta), free_list, rows);
    MTGR_LAUNCH_CHECK();
    t->n_chunks += 1;
    return EMB_OK;
}

int ht_add_chunk_adam_state(emb_table_t* t, float* m, float* v, void* stream) {
    if (!t || !m || !v) return EMB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(m) & 15) || (reinterpret_cast<uintptr_t>(v) & 15)) return EMB_ERR_INVALID_ARG;
    if (t->n_adam_chunks >= t->n_chunks) return EMB_ERR_NO_STORAGE; // register the value chunk first
    // rows already in use in this chunk would start from garbage moments: only allowed while the chunk is unused
    const uint64_t first_row = (uint64_t)t->n_adam_chunks << t->desc.chunk_rows_log2;
    t->refresh();
    if (t->rows_used_bound() > first_row) return EMB_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_set_adam, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), t->st, t->n_adam_chunks, m, v);
    MTGR_LAUNCH_CHECK();
    t->n_adam_chunks += 1;
    return EMB_OK;
}

int ht_plan(emb_table_t* t, int64_t n_incoming, int* new_capacity_log2, int* chunks_needed) {
    if (!t || n_incoming < 0) return EMB_ERR_INVALID_ARG;
    t->refresh();
    if (new_capacity_log2) {
        *new_capacity_log2 = 0;
        if (t->slots) {
            const double lf = t->desc.max_load_factor;
            if (t->occupied_bound() + (uint64_t)n_incoming > (uint64_t)t->slot_limit()) {
                int c = t->cap_log2;
                while ((double)(t->live_bound() + (uint64_t)n_incoming) > 0.5 * lf * (double)(1ull << c) && c < 30) ++c;
                *new_capacity_log2 = c;
            }
        }
    }
    if (chunks_needed) {
        const uint64_t have = (uint64_t)t->n_chunks << t->desc.chunk_rows_log2;
        const uint64_t want = t->rows_used_bound() + (uint64_t)n_incoming;
        const uint64_t per = 1ull << t->desc.chunk_rows_log2;
        *chunks_needed = want > have ? (int)((want - have + per - 1) / per) : 0;
    }
    return EMB_OK;
}

// EMB_OK: the host-side upper bounds prove that n_max new keys fit under the load-factor limit and
// into the registered rows.  EMB_CHECK_STATUS: they do not - the device admits what fits and turns
// the rest away.
static int check_insert_room(emb_table_t* t, int64_t n_max) {
    if (!t->slots || t->n_chunks == 0) return EMB_ERR_NO_STORAGE;
    t->refresh();
    if (t->occupied_bound() + (uint64_t)n_max > (uint64_t)t->slot_limit()) return EMB_CHECK_STATUS;
    const uint64_t have = (uint64_t)t->n_chunks << t->desc.chunk_rows_log2;
    if (t->rows_used_bound() + (uint64_t)n_max > have) return EMB_CHECK_STATUS;
    return EMB_OK;
}

static int find_or_insert_impl(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, uint32_t step,
                               int32_t* row_idx, uint8_t* inserted, void* stream, bool touch, bool retry) {
    if (!t || n_max < 0 || n_max > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (n_max == 0) return EMB_OK;
    if (!key || !row_idx) return EMB_ERR_INVALID_ARG;
    const int room = check_insert_room(t, n_max);
    if (room < 0) return room;
    // the device checks every block's new keys against the limit unless the bound shows that all fit
    const int admit = t->occupied_bound() + (uint64_t)n_max > (uint64_t)t->slot_limit() ? 1 : 0;
    HtView v = t->view();
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = blocks_for((uint64_t)n_max, kFoiBlock);
#define MTGR_FOI(C_, T_)                                                                                          \
    hipLaunchKernelGGL((k_find_or_insert<C_, T_>), dim3(grid), dim3(kFoiBlock), 0, s, v, key, n_dev, n_max, step, \
                       row_idx, inserted, retry ? 1 : 0, admit)
    if (v.count) {
        if (touch) MTGR_FOI(true, true); else MTGR_FOI(true, false);
    } else {
        if (touch) MTGR_FOI(false, true); else MTGR_FOI(false, false);
    }
#undef MTGR_FOI
    MTGR_LAUNCH_CHECK();
    const unsigned need_t = blocks_for((uint64_t)n_max, kBlock);
    hipLaunchKernelGGL(k_touch, dim3(need_t < kTouchMaxGrid ? need_t : kTouchMaxGrid), dim3(kBlock), 0, s, v, n_dev, n_max,
                       step, row_idx, touch ? 1 : 0);
    MTGR_LAUNCH_CHECK();
    t->issued((uint64_t)n_max);
    const int rc = t->snapshot(s);
    return rc != EMB_OK ? rc : room;
}

int ht_find_or_insert(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, uint32_t step,
                      int32_t* row_idx, uint8_t* inserted, void* stream) {
    return find_or_insert_impl(t, key, n_dev, n_max, step, row_idx, inserted, stream, true, false);
}

int ht_find_or_insert_notouch(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, uint32_t step,
                              int32_t* row_idx, uint8_t* inserted, void* stream) {
    return find_or_insert_impl(t, key, n_dev, n_max, step, row_idx, inserted, stream, false, false);
}

int ht_find_or_insert_retry(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, uint32_t step,
                            int32_t* row_idx, uint8_t* inserted, int touch, void* stream) {
    return find_or_insert_impl(t, key, n_dev, n_max, step, row_idx, inserted, stream, touch != 0, true);
}

int ht_clear_status(emb_table_t* t, uint32_t bits, void* stream) {
    if (!t) return EMB_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_clear_status, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), t->st, bits);
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

int ht_find(emb_table_t* t, const uint64_t* key, const int64_t* n_dev, int64_t n_max, int32_t* row_idx,
            void* stream) {
    if (!t || n_max < 0 || n_max > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (n_max == 0) return EMB_OK;
    if (!key || !row_idx) return EMB_ERR_INVALID_ARG;
    if (!t->slots) return EMB_ERR_NO_STORAGE;
    HtView v = t->view();
    const unsigned grid = blocks_for((uint64_t)n_max, kBlock);
    if (v.count)
        hipLaunchKernelGGL(k_find<true>, dim3(grid), dim3(kBlock), 0, static_cast<hipStream_t>(stream), v, key, n_dev,
                           n_max, row_idx);
    else
        hipLaunchKernelGGL(k_find<false>, dim3(grid), dim3(kBlock), 0, static_cast<hipStream_t>(stream), v, key, n_dev,
                           n_max, row_idx);
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

int ht_evict(emb_table_t* t, uint32_t now, uint32_t ttl, uint32_t min_freq, uint32_t grace,
             uint64_t* evicted_keys, int64_t evicted_cap, int64_t* n_evicted, void* stream) {
    if (!t || !n_evicted || evicted_cap < 0) return EMB_ERR_INVALID_ARG;
    if (!t->slots) return EMB_ERR_NO_STORAGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_zero_bytes, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(n_evicted), (size_t)2);
    MTGR_LAUNCH_CHECK();
    HtView v = t->view();
    const uint64_t n_slots = 1ull << t->cap_log2;
    hipLaunchKernelGGL(k_evict, dim3(blocks_for(n_slots, kBigBlock)), dim3(kBigBlock), 0, s, v, n_slots, now, ttl, min_freq,
                       grace, evicted_keys, evicted_cap, reinterpret_cast<unsigned long long*>(n_evicted));
    MTGR_LAUNCH_CHECK();
    return t->snapshot(s);
}

int ht_rehash(emb_table_t* t, void* new_slots, int new_capacity_log2, void* stream) {
    if (!t || !new_slots || new_capacity_log2 < 6 || new_capacity_log2 > 30) return EMB_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(new_slots) & 127) return EMB_ERR_INVALID_ARG;
    if (!t->slots) return EMB_ERR_NO_STORAGE;
    if (new_slots == t->slots) return EMB_ERR_INVALID_ARG;
    // the live keys (newest counter copy plus inserts issued since) must fit under the limit
    t->refresh();
    if ((double)t->live_bound() > (double)t->desc.max_load_factor * (double)(1ull << new_capacity_log2))
        return EMB_ERR_NEED_REHASH;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t n_new = 1ull << new_capacity_log2;
    const uint64_t n_old = 1ull << t->cap_log2;
    if (new_capacity_log2 >= t->cap_log2 && new_capacity_log2 - t->cap_log2 <= 3) {
        // same size (purge of deleted markers) or 2, 4, 8 times larger: two streaming passes (a lane of the first
        // pass writes 2^k slots, so a jump from a tiny structure to a huge one is left to the general path)
        hipLaunchKernelGGL(k_rehash_split, dim3(blocks_for(n_old, kBlock)), dim3(kBlock), 0, s, t->slots, n_old,
                           static_cast<Slot*>(new_slots), t->cap_log2 - 3, new_capacity_log2 - t->cap_log2);
        MTGR_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_rehash<true>, dim3(blocks_for(n_old, kBlock)), dim3(kBlock), 0, s, t->slots, n_old,
                           static_cast<Slot*>(new_slots), n_new / kLineSlots - 1ull, t->st);
        MTGR_LAUNCH_CHECK();
    } else {
        hipLaunchKernelGGL(k_fill_slots, dim3(fill_grid(n_new)), dim3(256), 0, s, static_cast<Slot*>(new_slots), n_new);
        MTGR_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_rehash<false>, dim3(blocks_for(n_old, kBlock)), dim3(kBlock), 0, s, t->slots, n_old,
                           static_cast<Slot*>(new_slots), n_new / kLineSlots - 1ull, t->st);
        MTGR_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(k_after_rehash, dim3(1), dim3(kWave), 0, s, t->st);
    MTGR_LAUNCH_CHECK();
    t->slots = static_cast<Slot*>(new_slots);
    t->cap_log2 = new_capacity_log2;
    t->n_rehash += 1;
    t->base_tomb = 0;                   // deleted markers are gone;
    t->min_valid_seq = t->seq + 1;      // counter copies queued before this point still show them
    return t->snapshot(s);
}

int ht_set_hot_storage(emb_table_t* t, float* hot_values, uint32_t* hot_free, int64_t hot_rows, void* stream) {
    if (!t || !hot_values || !hot_free || hot_rows <= 0 || hot_rows > 0x7FFFFFFFll) return EMB_ERR_INVALID_ARG;
    if (t->desc.dtype != EMB_BF16) return EMB_ERR_INVALID_ARG; // fp32 tables have nothing to gain
    if (reinterpret_cast<uintptr_t>(hot_values) & 15) return EMB_ERR_INVALID_ARG;
    if (t->hot_values) return EMB_ERR_INVALID_ARG;              // one hot store per table, for its lifetime
    (void)stream; // counters were zeroed with the state block
    t->hot_values = hot_values;
    t->hot_free = hot_free;
    t->hot_capacity = (uint32_t)hot_rows;
    return EMB_OK;
}

int ht_export_hot(emb_table_t* t, uint64_t* keys, float* values, int64_t cap, int64_t* n, void* stream) {
    if (!t || !keys || !n || cap < 0) return EMB_ERR_INVALID_ARG;
    if (!t->slots || !t->hot_values) return EMB_ERR_NO_STORAGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_zero_bytes, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(n), (size_t)2);
    MTGR_LAUNCH_CHECK();
    const uint64_t n_slots = 1ull << t->cap_log2;
    hipLaunchKernelGGL(k_export_hot, dim3(blocks_for(n_slots, kBlock)), dim3(kBlock), 0, s, t->view(), n_slots, keys, values, cap,
                       reinterpret_cast<unsigned long long*>(n));
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

int ht_stats(emb_table_t* t, ht_stats_t* out, void* stream) {
    if (!t || !out) return EMB_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    static_assert(offsetof(HtHead, stat) % 128 == 0, "stat stripes must be line aligned");
    HtHead full;
    if (hipMemcpyAsync(&full, t->st, sizeof(HtHead), hipMemcpyDeviceToHost, s) != hipSuccess) return EMB_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return EMB_ERR_HIP;
    const HtCounts h = HtCounts::from(full);
    out->live = h.live;
    out->tombstones = h.tombstones;
    out->capacity = t->slots ? (1ull << t->cap_log2) : 0ull;
    out->rows_used = h.bump;
    out->rows_free = h.free_count > 0 ? (uint64_t)h.free_count : 0ull;
    out->rows_capacity = (uint64_t)t->n_chunks << t->desc.chunk_rows_log2;
    out->n_rehash = t->n_rehash;
    out->n_chunks = (uint64_t)t->n_chunks;
    out->status = h.status;
    out->lookups = h.stat[kStatLookups];
    out->probes = h.stat[kStatProbes];
    out->cas_attempts = h.stat[kStatCas];
    out->cas_failures = h.stat[kStatCasFail];
    out->alloc_atomics = h.stat[kStatAlloc];
    for (int b = 0; b < 8; ++b) out->probe_hist[b] = h.probe_hist[b];
    out->hot_rows_used = h.hot_bump;
    out->hot_rows_free = h.hot_free_count > 0 ? (uint64_t)h.hot_free_count : 0ull;
    out->hot_rows_capacity = t->hot_capacity;
    out->refused = h.refused;
    out->occupied = full.occupied;
    // exact numbers replace the running upper bounds; older counter copies are obsolete
    t->adopt(h, 0, t->seq);
    t->min_valid_seq = t->seq + 1;
    return EMB_OK;
}

int ht_export(emb_table_t* t, uint64_t* keys, void* values, float* acc, uint32_t* last_seen, uint32_t* freq,
              int64_t cap, int64_t* n, void* stream) {
    if (!t || !keys || !n || cap < 0) return EMB_ERR_INVALID_ARG;
    if (!t->slots) return EMB_ERR_NO_STORAGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_zero_bytes, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(n), (size_t)2);
    MTGR_LAUNCH_CHECK();
    HtView v = t->view();
    const uint64_t n_slots = 1ull << t->cap_log2;
    hipLaunchKernelGGL(k_export, dim3(blocks_for(n_slots, kBlock)), dim3(kBlock), 0, s, v, n_slots, keys,
                       static_cast<char*>(values), acc, last_seen, freq, cap, reinterpret_cast<unsigned long long*>(n));
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}

} // extern "C"
