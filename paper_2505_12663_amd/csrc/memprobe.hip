// Bare access patterns over 256-byte rows: what the memory system of the part gives a kernel that only reads, only
// writes, or mixes the two, in the shapes this library's row kernels use (16 lanes x 16 bytes per row, rows picked
// through an index).  A measuring aid next to the row kernels, not a step of the embedding path: bench.py's
// --ceiling-probes runs it so that the rates quoted for the row kernels have a yardstick that anybody can re-run.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"
#include "mtgr_emb.h"

namespace {
using namespace mtgr;

constexpr int kProbeBlock = 256;
constexpr int kProbeSpan = 64;      // rows a 16-lane group reads in a row, as in the segment reduce
constexpr int kProbeBatch = 4;      // rows in flight per batch, the next batch issued before the current one is summed

// EVERY = 0: reads only.  EVERY > 0: the running sum is stored (non-temporally) to dst row r / EVERY after every
// EVERY-th row and restarted, i.e. dst row q = sum of src rows idx[q*EVERY .. q*EVERY+EVERY-1] added in that order.
template <int EVERY>
__global__ __launch_bounds__(kProbeBlock) void k_probe_read(const char* __restrict__ src, const int32_t* __restrict__ idx,
                                                            int64_t rows, char* __restrict__ dst, float* sink) {
    const int lane = lane_id(), sub = lane & 15, gbase = lane - sub;
    const int64_t span = ((int64_t)blockIdx.x * kProbeBlock + threadIdx.x) >> 4;
    const int64_t first = span * kProbeSpan;
    if (first + kProbeSpan > rows) return;
    int my[kProbeSpan / 16];
#pragma unroll
    for (int u = 0; u < kProbeSpan / 16; ++u) {
        const int64_t r = first + u * 16 + sub;
        my[u] = idx ? __builtin_nontemporal_load(&idx[r]) : (int)r;
    }
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    auto issue = [&](int b, V16* v) {
#pragma unroll
        for (int k = 0; k < kProbeBatch; ++k) {
            const int f = b * kProbeBatch + k;
            const int row = __shfl(my[f / 16], gbase + f % 16, kWave);
            v[k] = ld16_nt(src + (size_t)row * 256 + sub * 16);
        }
    };
    auto fold = [&](int b, const V16* v) {
#pragma unroll
        for (int k = 0; k < kProbeBatch; ++k) {
            a0 += __uint_as_float(v[k].x);
            a1 += __uint_as_float(v[k].y);
            a2 += __uint_as_float(v[k].z);
            a3 += __uint_as_float(v[k].w);
            const int f = b * kProbeBatch + k;
            if (EVERY > 0 && (f + 1) % (EVERY > 0 ? EVERY : 1) == 0) {
                st16_nt(dst + (size_t)((first + f) / (EVERY > 0 ? EVERY : 1)) * 256 + sub * 16,
                        V16{__float_as_uint(a0), __float_as_uint(a1), __float_as_uint(a2), __float_as_uint(a3)});
                a0 = a1 = a2 = a3 = 0.0f;
            }
        }
    };
    V16 va[kProbeBatch], vb[kProbeBatch];
    issue(0, va);
#pragma unroll
    for (int b = 0; b < kProbeSpan / kProbeBatch; b += 2) {
        issue(b + 1, vb);
        fold(b, va);
        if (b + 2 < kProbeSpan / kProbeBatch) issue(b + 2, va);
        fold(b + 1, vb);
    }
    if (EVERY == 0 && a0 + a1 + a2 + a3 == 1.2345678e-30f) *sink = a0;     // keeps the loads; never true for finite rows of 1.0
}

// dst row idx[r] (r itself without an index) <- (float)r in every element; every wave stores 1 KB per instruction
__global__ __launch_bounds__(kProbeBlock) void k_probe_write(char* __restrict__ dst, const int32_t* __restrict__ idx, int64_t rows) {
    const int sub = threadIdx.x & 15;
    const int64_t r = ((int64_t)blockIdx.x * kProbeBlock + threadIdx.x) >> 4;
    if (r >= rows) return;
    const int64_t d = idx ? (int64_t)idx[r] : r;
    const uint32_t w = __float_as_uint((float)r);
    st16_nt(dst + (size_t)d * 256 + sub * 16, V16{w, w, w, w});
}

} // namespace

extern "C" int emb_probe_memory(int pattern, const void* src, void* dst, const int32_t* idx, int64_t rows, void* stream) {
    if (rows <= 0 || rows > 0x7FFFFFFFll || rows % kProbeSpan != 0) return EMB_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const char* sp = static_cast<const char*>(src);
    char* dp = static_cast<char*>(dst);
    const unsigned read_grid = (unsigned)((rows / kProbeSpan * 16 + kProbeBlock - 1) / kProbeBlock);
    switch (pattern) {
    case EMB_PROBE_READ:
        if (!src || !dst) return EMB_ERR_INVALID_ARG;
        hipLaunchKernelGGL(k_probe_read<0>, dim3(read_grid), dim3(kProbeBlock), 0, s, sp, idx, rows, dp, static_cast<float*>(dst));
        break;
    case EMB_PROBE_WRITE:
        if (!dst) return EMB_ERR_INVALID_ARG;
        hipLaunchKernelGGL(k_probe_write, dim3((unsigned)((rows * 16 + kProbeBlock - 1) / kProbeBlock)), dim3(kProbeBlock), 0, s, dp, idx, rows);
        break;
    case EMB_PROBE_READ_STORE_4TH:
        if (!src || !dst) return EMB_ERR_INVALID_ARG;
        hipLaunchKernelGGL(k_probe_read<4>, dim3(read_grid), dim3(kProbeBlock), 0, s, sp, idx, rows, dp, static_cast<float*>(nullptr));
        break;
    case EMB_PROBE_READ_STORE_64TH:
        if (!src || !dst) return EMB_ERR_INVALID_ARG;
        hipLaunchKernelGGL(k_probe_read<64>, dim3(read_grid), dim3(kProbeBlock), 0, s, sp, idx, rows, dp, static_cast<float*>(nullptr));
        break;
    default:
        return EMB_ERR_INVALID_ARG;
    }
    MTGR_LAUNCH_CHECK();
    return EMB_OK;
}
