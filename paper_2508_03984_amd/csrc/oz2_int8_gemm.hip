// Batched INT8 GEMM with exact (wrapping) INT32 accumulation on the gfx950 matrix cores:
// Algorithm 1 line 6, C'_s = A'_s B'_s for all moduli s in one launch.
//
// Operands are the padded, K-contiguous residue slices: A [batch][Mp][Kp] and
// B [batch][Np][Kp] (B transposed), so both tiles are staged through LDS the same way
// and every MFMA operand is a 16-byte K-run read with one ds_read_b128.
//
// Tiling: workgroup = 4 wavefronts (2 x 2), block tile (64 TM) x (64 TN) x BK, each
// wavefront owns (32 TM) x (32 TN) = TM x TN v_mfma_i32_32x32x32_i8 accumulators.
// LDS holds two stages; 16-byte chunks of a row are XOR-swizzled with the row index so
// that the 32 rows a fragment read touches fall in distinct bank groups.
#include "oz2_kernels.hpp"

namespace oz2 {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

template <int CPR>
__device__ inline int swizzle(int row, int chunk) {
    // CPR chunks of 16 B per row; rows that share LDS bank groups get distinct XOR masks.
    return chunk ^ ((row / (8 / CPR)) & (CPR - 1));
}

template <int TM, int TN, int BK>
__global__ __launch_bounds__(256) void k_int8_gemm(const int8_t *__restrict__ A,
                                                   const int8_t *__restrict__ B,
                                                   int32_t *__restrict__ C, int64_t Mp,
                                                   int64_t Np, int64_t Kp) {
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int CPR = BK / 16;                       // 16-byte chunks per tile row
    constexpr int ROWS = BM + BN;                      // A rows then B rows in one LDS stage
    constexpr int CHUNKS = ROWS * CPR;
    constexpr int LPT = CHUNKS / 256;                  // global 16-byte loads per thread and stage
    static_assert(CHUNKS % 256 == 0, "tile must split evenly over the workgroup");
    static_assert(CPR == 4 || CPR == 8, "BK must be 64 or 128");

    extern __shared__ v4i lds[];                       // [2][ROWS][CPR]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t bm = (int64_t)blockIdx.y * BM, bn = (int64_t)blockIdx.x * BN;
    const int64_t s = blockIdx.z;
    const int8_t *Ab = A + (s * Mp + bm) * Kp;
    const int8_t *Bb = B + (s * Np + bn) * Kp;

    // Global source of each of this thread's chunks (row-major over [ROWS][CPR]).
    const int8_t *src[LPT];
    int dst[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        int ci = tid + 256 * i, row = ci / CPR, ch = ci % CPR;
        src[i] = (row < BM ? Ab + (int64_t)row * Kp : Bb + (int64_t)(row - BM) * Kp) + ch * 16;
        dst[i] = row * CPR + swizzle<CPR>(row, ch);
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    v4i stage[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) stage[i] = *reinterpret_cast<const v4i *>(src[i]);
#pragma unroll
    for (int i = 0; i < LPT; ++i) lds[dst[i]] = stage[i];
    __syncthreads();

    const int KT = (int)(Kp / BK);
    const int lrow = lane & 31, lhalf = lane >> 5;
    for (int kt = 0; kt < KT; ++kt) {
        const v4i *cur = lds + (kt & 1) * CHUNKS;
        v4i *nxt = lds + ((kt + 1) & 1) * CHUNKS;
        const bool more = kt + 1 < KT;
        if (more) {
#pragma unroll
            for (int i = 0; i < LPT; ++i)
                stage[i] = *reinterpret_cast<const v4i *>(src[i] + (int64_t)(kt + 1) * BK);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 32; ++kk) {
            v4i a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int row = wm * 32 * TM + i * 32 + lrow;
                a[i] = cur[row * CPR + swizzle<CPR>(row, kk * 2 + lhalf)];
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int row = BM + wn * 32 * TN + j * 32 + lrow;
                b[j] = cur[row * CPR + swizzle<CPR>(row, kk * 2 + lhalf)];
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < LPT; ++i) nxt[dst[i]] = stage[i];
        }
        __syncthreads();
    }

    // Accumulator layout of the 32x32 MFMA: lane l, register r holds
    // row 8*(r/4) + 4*(l/32) + r%4, column l%32.
    int32_t *Cb = C + (s * Mp + bm) * Np + bn;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = wm * 32 * TM + i * 32 + 8 * (r / 4) + 4 * lhalf + (r % 4);
                int col = wn * 32 * TN + j * 32 + lrow;
                Cb[(int64_t)row * Np + col] = acc[i][j][r];
            }
}

template <int TM, int TN, int BK>
hipError_t launch(const int8_t *A, const int8_t *B, int32_t *C, int batch, int64_t Mp, int64_t Np,
                  int64_t Kp, hipStream_t stream) {
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr size_t lds_bytes = 2ull * (BM + BN) * BK;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_int8_gemm<TM, TN, BK>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)(Np / BN), (unsigned)(Mp / BM), (unsigned)batch);
    hipLaunchKernelGGL((k_int8_gemm<TM, TN, BK>), grid, dim3(256), lds_bytes, stream, A, B, C, Mp,
                       Np, Kp);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_int8_gemm(const int8_t *A, const int8_t *B, int32_t *C, int batch, int64_t Mp,
                            int64_t Np, int64_t Kp, hipStream_t stream) {
    // Small problems get the 128 x 128 tile so that more workgroups exist.
    if (Mp * Np * batch < (int64_t)256 * 256 * 512)
        return launch<2, 2, 64>(A, B, C, batch, Mp, Np, Kp, stream);
    return launch<4, 4, 64>(A, B, C, batch, Mp, Np, Kp, stream);
}

}  // namespace oz2
