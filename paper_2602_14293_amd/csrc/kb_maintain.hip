// Knowledge-base maintenance (gfx950): revising predicted gains, removing entries, compaction.
//   kb_update_gain : update_gain_kernel   (scatter of an exponential moving average)
//   kb_remove      : remove_kernel        (sets the removed bit of the entries' 1/|k|)
//   kb_compact     : live_count_kernel -> offset_scan_kernel -> compact_kernel (stable gather into a second store)
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "kb_internal.hpp"

using namespace kbi;

namespace {

constexpr int BLOCK_ROWS = 256;       // rows per workgroup in the counting and gathering kernels (one per thread)
constexpr size_t WS_ALIGN = 256;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void update_gain_kernel(float *gain, int64_t n, const int32_t *indices, const float *values, int64_t m, float alpha)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= m) return;
    const int64_t i = indices[j];
    if (i < 0 || i >= n) return;
    const float g = gain[i], v = values[j];
    gain[i] = alpha == 1.0f ? v : __builtin_fmaf(alpha, v - g, g);
}

__global__ __launch_bounds__(256) void remove_kernel(float *inv_norm, int64_t n, const int32_t *indices, int64_t m)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= m) return;
    const int64_t i = indices[j];
    if (i < 0 || i >= n) return;
    atomicOr(reinterpret_cast<unsigned int *>(inv_norm + i), REMOVED_BIT);      // the same index twice is harmless
}

// live rows of each block of BLOCK_ROWS rows
__global__ __launch_bounds__(256) void live_count_kernel(const float *inv_norm, int64_t n, uint32_t *block_live)
{
    __shared__ uint32_t wave_live[4];
    const int64_t row = (int64_t)blockIdx.x * BLOCK_ROWS + threadIdx.x;
    const bool live = row < n && !row_removed(inv_norm[row]);
    const uint64_t m = __builtin_amdgcn_ballot_w64(live);
    if ((threadIdx.x & 63) == 0) wave_live[threadIdx.x >> 6] = (uint32_t)__builtin_popcountll(m);
    __syncthreads();
    if (threadIdx.x == 0) block_live[blockIdx.x] = wave_live[0] + wave_live[1] + wave_live[2] + wave_live[3];
}

// Exclusive prefix sums of the block counts in place, total appended: one workgroup, each thread a contiguous run.
__global__ __launch_bounds__(1024) void offset_scan_kernel(uint32_t *block_live, int64_t blocks)
{
    __shared__ uint32_t part[1024];
    const int tid = threadIdx.x;
    const int64_t per = (blocks + 1023) / 1024, begin = tid * per, end = begin + per < blocks ? begin + per : blocks;
    uint32_t sum = 0;
    for (int64_t b = begin; b < end; ++b) sum += block_live[b];
    part[tid] = sum;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {          // inclusive scan of the per-thread sums
        const uint32_t add = tid >= off ? part[tid - off] : 0u;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    uint32_t run = part[tid] - sum;
    for (int64_t b = begin; b < end; ++b) {
        const uint32_t c = block_live[b];
        block_live[b] = run;
        run += c;
    }
    if (tid == 1023) block_live[blocks] = part[1023];
}

struct CompactArgs {
    const unsigned char *keys_src;
    unsigned char *keys_dst;
    const float *scale_src, *inv_src, *gain_src;
    float *scale_dst, *inv_dst, *gain_dst;
    const uint64_t *tags_src;
    uint64_t *tags_dst;
    int32_t *index_map;
    const uint32_t *block_offset;
    int64_t n;
    uint32_t row_bytes;      // multiple of 16
};

// Each thread places one source row (index map and the per-entry scalars).  The block's live rows go to
// consecutive destination rows, so their keys are one contiguous run of 16-byte pieces in the destination; the
// workgroup copies that run piece by piece (four loads in flight per thread), looking the source row of a piece
// up in a list of the block's live rows.  Destinations of different blocks never overlap and source and
// destination stores are distinct, so no ordering between workgroups is needed.
__global__ __launch_bounds__(256) void compact_kernel(CompactArgs a)
{
    __shared__ uint32_t wave_live[4];
    __shared__ uint16_t live_row[BLOCK_ROWS];      // block-local source row of the block's i-th live row
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * BLOCK_ROWS, row = row0 + tid;
    const bool live = row < a.n && !row_removed(a.inv_src[row]);
    const uint64_t m = __builtin_amdgcn_ballot_w64(live);
    if (lane == 0) wave_live[wave] = (uint32_t)__builtin_popcountll(m);
    __syncthreads();
    uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    for (int w = 0; w < wave; ++w) rank += wave_live[w];
    const uint32_t first = a.block_offset[blockIdx.x], to = first + rank;
    if (live) live_row[rank] = (uint16_t)tid;
    if (row < a.n) {
        if (a.index_map) a.index_map[row] = live ? (int32_t)to : -1;
        if (live) {
            a.inv_dst[to] = a.inv_src[row];
            if (a.scale_src) a.scale_dst[to] = a.scale_src[row];
            if (a.tags_src) a.tags_dst[to] = a.tags_src[row];
            if (a.gain_src) a.gain_dst[to] = a.gain_src[row];
        }
    }
    __syncthreads();
    const uint32_t pieces = a.row_bytes / 16, n_live = wave_live[0] + wave_live[1] + wave_live[2] + wave_live[3];
    const uint32_t total = n_live * pieces;                            // < 2^20
    const unsigned char *src0 = a.keys_src + (size_t)row0 * a.row_bytes;
    u32x4 *dst = reinterpret_cast<u32x4 *>(a.keys_dst + (size_t)first * a.row_bytes);
    auto source = [&](uint32_t x) {
        const uint32_t r = x / pieces, p = x - r * pieces;
        return reinterpret_cast<const u32x4 *>(src0 + (size_t)live_row[r] * a.row_bytes) + p;
    };
    uint32_t x = tid;
    for (; x + 768 < total; x += 1024) {
        const u32x4 v0 = *source(x), v1 = *source(x + 256), v2 = *source(x + 512), v3 = *source(x + 768);
        dst[x] = v0;
        dst[x + 256] = v1;
        dst[x + 512] = v2;
        dst[x + 768] = v3;
    }
    for (; x < total; x += 256) dst[x] = *source(x);
}

size_t compact_workspace(int64_t n)
{
    const int64_t blocks = (n + BLOCK_ROWS - 1) / BLOCK_ROWS;
    return ((size_t)(blocks + 1) * 4 + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN;
}

}  // namespace

extern "C" {

kb_status_t kb_update_gain(float *gain_dev, int64_t n, const int32_t *indices_dev, const float *values_dev, int64_t m, float alpha,
                           void *hip_stream)
{
    if (!gain_dev || !indices_dev || !values_dev) return KB_ERR_NULL;
    if (n < 0 || m < 0 || m >= (int64_t(1) << 31) || !(alpha >= 0.f && alpha <= 1.f)) return KB_ERR_INVALID_ARG;
    if (((reinterpret_cast<uintptr_t>(gain_dev) | reinterpret_cast<uintptr_t>(indices_dev) | reinterpret_cast<uintptr_t>(values_dev)) & 3) != 0)
        return KB_ERR_INVALID_ARG;
    if (m == 0) return KB_OK;
    hipLaunchKernelGGL(update_gain_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream), gain_dev, n,
                       indices_dev, values_dev, m, alpha);
    return hipGetLastError() == hipSuccess ? KB_OK : KB_ERR_DEVICE;
}

kb_status_t kb_remove(kb_t *kb, const int32_t *indices_dev, int64_t m, void *hip_stream)
{
    if (!kb || !indices_dev) return KB_ERR_NULL;
    if (m < 0 || m >= (int64_t(1) << 31) || (reinterpret_cast<uintptr_t>(indices_dev) & 3) != 0) return KB_ERR_INVALID_ARG;
    if (kb->n_normalized != kb->n) return KB_ERR_NOT_NORMALIZED;     // kb_normalize would overwrite the mark of an unnormalised row
    if (m == 0 || kb->n == 0) return KB_OK;
    hipLaunchKernelGGL(remove_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(hip_stream), kb->inv_norm, kb->n,
                       indices_dev, m);
    return hipGetLastError() == hipSuccess ? KB_OK : KB_ERR_DEVICE;
}

size_t kb_compact_workspace_bytes(const kb_t *kb) { return kb ? compact_workspace(kb->capacity) : 0; }

kb_status_t kb_compact(kb_t *src, kb_t *dst, const float *gain_src_dev, float *gain_dst_dev, int32_t *index_map_out_dev,
                       void *workspace_dev, size_t workspace_bytes, void *hip_stream, int64_t *live_out)
{
    if (!src || !dst) return KB_ERR_NULL;
    if (src == dst || src->keys == dst->keys || src->inv_norm == dst->inv_norm) return KB_ERR_INVALID_ARG;
    if (src->d != dst->d || (src->tags != nullptr) != (dst->tags != nullptr) || dst->n != 0) return KB_ERR_INVALID_ARG;
    if (src->dtype != dst->dtype) return KB_ERR_DTYPE;
    if ((gain_src_dev != nullptr) != (gain_dst_dev != nullptr)) return KB_ERR_NULL;
    if (((reinterpret_cast<uintptr_t>(gain_src_dev) | reinterpret_cast<uintptr_t>(gain_dst_dev) | reinterpret_cast<uintptr_t>(index_map_out_dev)) & 3) != 0)
        return KB_ERR_INVALID_ARG;
    if (src->n_normalized != src->n) return KB_ERR_NOT_NORMALIZED;
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & (WS_ALIGN - 1)) != 0 || workspace_bytes < compact_workspace(src->n))
        return KB_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int64_t n = src->n;
    int64_t live = 0;
    if (n > 0) {
        const int64_t blocks = (n + BLOCK_ROWS - 1) / BLOCK_ROWS;
        uint32_t *block_live = static_cast<uint32_t *>(workspace_dev);
        hipLaunchKernelGGL(live_count_kernel, dim3((unsigned)blocks), dim3(256), 0, s, src->inv_norm, n, block_live);
        hipLaunchKernelGGL(offset_scan_kernel, dim3(1), dim3(1024), 0, s, block_live, blocks);
        if (hipGetLastError() != hipSuccess) return KB_ERR_DEVICE;
        uint32_t total = 0;
        if (hipMemcpyAsync(&total, block_live + blocks, sizeof total, hipMemcpyDeviceToHost, s) != hipSuccess) return KB_ERR_DEVICE;
        if (hipStreamSynchronize(s) != hipSuccess) return KB_ERR_DEVICE;
        live = total;
        if (live > dst->capacity) return KB_ERR_CAPACITY;       // nothing has been written yet
        CompactArgs a;
        memset(&a, 0, sizeof a);
        a.keys_src = static_cast<const unsigned char *>(src->keys);
        a.keys_dst = static_cast<unsigned char *>(dst->keys);
        a.scale_src = src->row_scale;
        a.scale_dst = dst->row_scale;
        a.inv_src = src->inv_norm;
        a.inv_dst = dst->inv_norm;
        a.gain_src = gain_src_dev;
        a.gain_dst = gain_dst_dev;
        a.tags_src = src->tags;
        a.tags_dst = dst->tags;
        a.index_map = index_map_out_dev;
        a.block_offset = block_live;
        a.n = n;
        a.row_bytes = (uint32_t)src->d * (src->dtype == KB_F32 ? 4u : src->dtype == KB_BF16 ? 2u : 1u);
        hipLaunchKernelGGL(compact_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
        if (hipGetLastError() != hipSuccess) return KB_ERR_DEVICE;
    }
    dst->n = dst->n_normalized = live;
    if (live_out) *live_out = live;
    return KB_OK;
}

}  // extern "C"
