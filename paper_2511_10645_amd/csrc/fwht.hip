// Fast Walsh-Hadamard transform of activation rows: the yardstick that Section 4.3's figure
// ("speedup of scaled pairwise rotation over the Hadamard transform") compares the transform
// kernel with.  Not part of the method's path; textbook radix-2 butterflies.
//
//      y = H_n x / sqrt(n),   H_n[i][j] = (-1)^popcount(i & j)   (Sylvester order), n = 2^k
//
// One block per row.  A thread loads 8 consecutive fp16 values (one 16-byte access), runs the
// three lowest butterfly levels in registers and leaves the row in LDS as fp32; the remaining
// k - 3 levels go three at a time: a thread gathers the 8 values that differ only in the three
// index bits of the pass, runs the three levels in registers and puts them back (one block
// barrier per pass); finally the row is read back in order, scaled, rounded once to fp16 and
// stored 16 bytes per thread.  HBM traffic 4 bytes per element, 32 bytes of LDS traffic per
// element at n = 4096; fp32 arithmetic throughout.  LDS addresses are padded by one word per 32
// so that the 8-word strides of the first and last step fall on distinct banks.
#include "paro_internal.h"

namespace paro {

__device__ inline int fw_pad(int a) { return a + (a >> 5); }

template <int B>
__device__ inline void butterflies(float (&v)[8])
{
#pragma unroll
    for (int lvl = 0; lvl < B; ++lvl)
#pragma unroll
        for (int i = 0; i < (1 << B); ++i)
            if (!(i & (1 << lvl))) {
                const float a = v[i], b = v[i | (1 << lvl)];
                v[i] = a + b;
                v[i | (1 << lvl)] = a - b;
            }
}

// one pass over index bits [lo, lo + B): every thread takes tasks of 2^B values
template <int B>
__device__ inline void lds_pass(float *s, int n, int lo)
{
    const int tasks = n >> B;
    for (int q = threadIdx.x; q < tasks; q += blockDim.x) {
        const int base = ((q >> lo) << (lo + B)) | (q & ((1 << lo) - 1));
        float v[8];
#pragma unroll
        for (int i = 0; i < (1 << B); ++i) v[i] = s[fw_pad(base + (i << lo))];
        butterflies<B>(v);
#pragma unroll
        for (int i = 0; i < (1 << B); ++i) s[fw_pad(base + (i << lo))] = v[i];
    }
}

__global__ __launch_bounds__(256) void fwht_kernel(const _Float16 *X, int64_t ldx, _Float16 *Y, int64_t ldy, int T, int n,
                                                   int log2n, float scale)
{
    extern __shared__ __attribute__((aligned(16))) float s_row[];
    typedef _Float16 half8f __attribute__((ext_vector_type(8)));
    for (int t = blockIdx.x; t < T; t += gridDim.x) {
        // levels 0..2 in registers, straight from the 16-byte load
        for (int q = threadIdx.x; q < n / 8; q += blockDim.x) {
            const half8f h = *(const half8f *)(X + (size_t)t * ldx + 8 * q);
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = (float)h[i];
            butterflies<3>(v);
#pragma unroll
            for (int i = 0; i < 8; ++i) s_row[fw_pad(8 * q + i)] = v[i];
        }
        __syncthreads();
        int lo = 3;
        for (; lo + 3 <= log2n; lo += 3) { lds_pass<3>(s_row, n, lo); __syncthreads(); }
        if (log2n - lo == 2) { lds_pass<2>(s_row, n, lo); __syncthreads(); }
        else if (log2n - lo == 1) { lds_pass<1>(s_row, n, lo); __syncthreads(); }
        for (int q = threadIdx.x; q < n / 8; q += blockDim.x) {
            half8f h;
#pragma unroll
            for (int i = 0; i < 8; ++i) h[i] = (_Float16)(s_row[fw_pad(8 * q + i)] * scale);
            *(half8f *)(Y + (size_t)t * ldy + 8 * q) = h;
        }
        __syncthreads();          // the row buffer is reused by the block's next row
    }
}

}  // namespace paro

extern "C" paro_status paro_fwht(const paro_half_t *X, int64_t ldx, paro_half_t *Y, int64_t ldy, int32_t T, int32_t n,
                                 void *stream)
{
    if (!X || !Y) return PARO_ERR_NULL;
    if (T <= 0 || n < 8 || (n & (n - 1)) || ldx < n || ldy < n) return PARO_ERR_SHAPE;
    if (n > 32768) return PARO_ERR_UNSUPPORTED;                       // one row (fp32, padded) must fit the LDS of a compute unit
    if (ldx % 8 || ldy % 8 || (uintptr_t)X % 16 || (uintptr_t)Y % 16) return PARO_ERR_ALIGN;
    if (X == Y && ldx != ldy) return PARO_ERR_SHAPE;
    int log2n = 0;
    while ((1 << log2n) < n) ++log2n;
    const size_t lds = (size_t)(n + n / 32 + 1) * sizeof(float);
    static std::atomic<uint64_t> attr_done{0};
    if (const int dev = paro::once_pending(attr_done); dev >= 0) {
        if (hipFuncSetAttribute((const void *)paro::fwht_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return PARO_ERR_HIP;
        paro::once_done(attr_done, dev);
    }
    const int threads = n / 8 < 256 ? (n / 8 < 64 ? 64 : n / 8) : 256;
    const int blocks = T < 65536 ? T : 65536;
    hipLaunchKernelGGL(paro::fwht_kernel, dim3(blocks), dim3(threads), lds, (hipStream_t)stream, (const _Float16 *)X, ldx,
                       (_Float16 *)Y, ldy, T, n, log2n, 1.0f / sqrtf((float)n));
    return hipGetLastError() == hipSuccess ? PARO_OK : PARO_ERR_HIP;
}
