// kb_quantize_rows: fp32 / bf16 rows to e4m3 codes with one fp32 scale per row, the storage form of
// compressed keys and of fp8 queries (gfx950).  Memory-bound: every element is read once from HBM (a
// second time from registers or the cache) and one byte is written.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kb.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int ROWS_PER_WG = 4;      // one wavefront per row
constexpr int CACHED = 4;           // 16-byte pieces of the row a lane keeps in registers between the two passes
constexpr float E4M3_MAX = 448.0f;

// Four quotients to four e4m3 codes (nearest, ties to the even code, sign kept) with the conversion instruction
// of gfx950, which implements exactly that rounding for the OCP e4m3 format, subnormal range included.  No
// quotient exceeds 448 (1 + 2^-23), which rounds to 448, so the overflow behaviour of the instruction never
// comes into play.
__device__ inline uint32_t encode_e4m3_x4(float y0, float y1, float y2, float y3)
{
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(y0, y1, 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(y2, y3, w, true);
    return (uint32_t)w;
}

template <int DT> struct Piece;     // 16 bytes of a row
template <> struct Piece<KB_F32> {
    static constexpr int ELEMS = 4;
    static __device__ float value(const u32x4 &v, int i) { return __uint_as_float(v[i]); }
};
template <> struct Piece<KB_BF16> {
    static constexpr int ELEMS = 8;
    static __device__ float value(const u32x4 &v, int i) { return __uint_as_float((i & 1) ? (v[i >> 1] & 0xFFFF0000u) : (v[i >> 1] << 16)); }
};

template <int DT> __device__ inline float piece_amax(const u32x4 &v)
{
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < Piece<DT>::ELEMS; ++i) m = fmaxf(m, fabsf(Piece<DT>::value(v, i)));
    return m;
}

template <int DT> __device__ inline void piece_store(const u32x4 &v, float scale, unsigned char *dst)
{
    uint32_t w[Piece<DT>::ELEMS / 4];
#pragma unroll
    for (int j = 0; j < Piece<DT>::ELEMS / 4; ++j) {
        w[j] = encode_e4m3_x4(Piece<DT>::value(v, 4 * j) / scale, Piece<DT>::value(v, 4 * j + 1) / scale,
                              Piece<DT>::value(v, 4 * j + 2) / scale, Piece<DT>::value(v, 4 * j + 3) / scale);
    }
    if constexpr (Piece<DT>::ELEMS == 8)
        *reinterpret_cast<uint2 *>(dst) = make_uint2(w[0], w[1]);
    else
        *reinterpret_cast<uint32_t *>(dst) = w[0];
}

template <int DT> __global__ __launch_bounds__(64 * ROWS_PER_WG) void quantize_rows_kernel(const unsigned char *rows, int64_t n, int d, unsigned char *codes, float *scale_out)
{
    constexpr int ELEMS = Piece<DT>::ELEMS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pieces = d / ELEMS;
    for (int64_t row = (int64_t)blockIdx.x * ROWS_PER_WG + wave; row < n; row += (int64_t)gridDim.x * ROWS_PER_WG) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(rows + (size_t)row * d * (16 / ELEMS));
        u32x4 keep[CACHED];
        float m = 0.f;
#pragma unroll
        for (int c = 0; c < CACHED; ++c) {
            const int p = lane + 64 * c;
            keep[c] = p < pieces ? src[p] : u32x4{0, 0, 0, 0};
            m = fmaxf(m, piece_amax<DT>(keep[c]));
        }
        for (int p = lane + 64 * CACHED; p < pieces; p += 64) m = fmaxf(m, piece_amax<DT>(src[p]));
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, 64));
        const float scale = m > 0.f ? m / E4M3_MAX : 1.0f;
        if (scale_out && lane == 0) scale_out[row] = scale;
        unsigned char *dst = codes + (size_t)row * d;
#pragma unroll
        for (int c = 0; c < CACHED; ++c) {
            const int p = lane + 64 * c;
            if (p < pieces) piece_store<DT>(keep[c], scale, dst + (size_t)p * ELEMS);
        }
        for (int p = lane + 64 * CACHED; p < pieces; p += 64) piece_store<DT>(src[p], scale, dst + (size_t)p * ELEMS);
    }
}

}  // namespace

extern "C" kb_status_t kb_quantize_rows(const void *rows_dev, kb_dtype_t dtype, int64_t n, int32_t d, void *codes_out_dev,
                                        float *scale_out_dev, void *hip_stream)
{
    if (!rows_dev || !codes_out_dev) return KB_ERR_NULL;
    if (dtype != KB_F32 && dtype != KB_BF16) return KB_ERR_DTYPE;
    if (n < 0 || n >= (int64_t(1) << 31) || d < 16 || d > 16384 || d % 16 != 0) return KB_ERR_INVALID_ARG;
    if (((reinterpret_cast<uintptr_t>(rows_dev) | reinterpret_cast<uintptr_t>(codes_out_dev)) & 15) != 0) return KB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(scale_out_dev) & 3) != 0) return KB_ERR_INVALID_ARG;
    if (n == 0) return KB_OK;
    const int64_t want = (n + ROWS_PER_WG - 1) / ROWS_PER_WG;
    const int grid = (int)(want < 256 * 32 ? want : 256 * 32);      // 32 workgroups per compute unit keep HBM busy; the rest loops
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (dtype == KB_F32)
        hipLaunchKernelGGL(quantize_rows_kernel<KB_F32>, dim3(grid), dim3(64 * ROWS_PER_WG), 0, s, static_cast<const unsigned char *>(rows_dev), n, d,
                           static_cast<unsigned char *>(codes_out_dev), scale_out_dev);
    else
        hipLaunchKernelGGL(quantize_rows_kernel<KB_BF16>, dim3(grid), dim3(64 * ROWS_PER_WG), 0, s, static_cast<const unsigned char *>(rows_dev), n, d,
                           static_cast<unsigned char *>(codes_out_dev), scale_out_dev);
    return hipGetLastError() == hipSuccess ? KB_OK : KB_ERR_DEVICE;
}
