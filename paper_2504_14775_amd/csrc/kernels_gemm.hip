// bf16 x bf16 -> fp32 GEMM on the CDNA4 matrix cores:  out[m][n] (op)= sum_k a[m][k] * w[n][k].
//
// Both operands are contiguous along k, which is the order the MFMA operand registers want
// (each lane feeds 8 consecutive k of one row), so tiles go global -> LDS -> registers without
// any transposition.  One workgroup of 4 wavefronts (2 x 2) owns a BM x BN output tile and walks
// k in steps of 64 through two LDS buffers: the global loads of step i+1 are issued before the
// MFMAs of step i and written to the other buffer afterwards.
//
// LDS tile layout: row r holds its 64 k-values as eight 16-byte groups; group c is stored at
// group position c ^ (r & 7).  A wavefront's 16-byte operand reads (32 rows x 2 groups) and the
// loader's 16-byte writes then spread evenly over the banks.
//
// Workgroup -> tile mapping: hardware hands consecutive workgroup ids to the 8 XCDs in turn, each
// with its own L2.  Ids are therefore first regrouped so that an XCD receives a contiguous range of
// tile numbers; tiles are numbered band by band (a band is 8 tile-columns wide, walked row by row),
// so the tiles an XCD works on at one time share a few A row-panels and W row-panels in its L2.
#include "common.h"

namespace {

constexpr int BK = 64;

__device__ __forceinline__ float silu(float z) { return z / (1.0f + __expf(-z)); }

template <int BM, int BN, int MODE>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                         const bf16_t* __restrict__ W, int64_t ldw,
                                                         void* __restrict__ out, int64_t ldc, int M, int N, int K,
                                                         int tiles_m, int tiles_n) {
    constexpr int TM = BM / 64;  // 32x32 blocks per wave along m
    constexpr int TN = BN / 64;
    constexpr int A_CHUNKS = BM / 32;  // 16-byte groups each thread moves per k-step
    constexpr int W_CHUNKS = BN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* lds_a = reinterpret_cast<bf16_t*>(smem);                       // [2][BM][64]
    bf16_t* lds_w = lds_a + 2 * BM * BK;                                   // [2][BN][64]

    // ---- tile assignment (XCD aware) ----
    const int num_tiles = tiles_m * tiles_n;
    int wg = blockIdx.x;
    {
        // XCD x receives workgroups x, x+8, ...: q of them, one more for x < rem
        const int q = num_tiles >> 3, rem = num_tiles & 7;
        const int xcd = wg & 7, idx = wg >> 3;
        wg = xcd * q + min(xcd, rem) + idx;
    }
    constexpr int BAND = 8;  // tile columns per band
    const int band = wg / (BAND * tiles_m);
    const int band_cols = min(BAND, tiles_n - band * BAND);
    const int in_band = wg - band * BAND * tiles_m;
    const int tile_m = in_band / band_cols;
    const int tile_n = band * BAND + in_band % band_cols;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- loader addressing: thread moves group c of rows r0 + 32 i ----
    const int c = tid & 7, r0 = tid >> 3;
    const bf16_t* ga = A + (int64_t)(m0 + r0) * lda + c * 8;
    const bf16_t* gw = W + (int64_t)(n0 + r0) * ldw + c * 8;
    const int lds_off = r0 * BK + ((c ^ (r0 & 7)) * 8);

    u32x4 ra[A_CHUNKS], rw[W_CHUNKS];
    auto load_global = [&](int kt) {
        const int64_t k0 = (int64_t)kt * BK;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) ra[i] = *reinterpret_cast<const u32x4*>(ga + (int64_t)(32 * i) * lda + k0);
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) rw[i] = *reinterpret_cast<const u32x4*>(gw + (int64_t)(32 * i) * ldw + k0);
    };
    auto store_lds = [&](int buf) {
        bf16_t* pa = lds_a + buf * BM * BK + lds_off;
        bf16_t* pw = lds_w + buf * BN * BK + lds_off;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<u32x4*>(pa + 32 * i * BK) = ra[i];
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) *reinterpret_cast<u32x4*>(pw + 32 * i * BK) = rw[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // operand read addressing: lane supplies row (lane % 32), k-group (lane / 32) of each 16-wide k step
    const int frow = lane & 31, fgrp = lane >> 5, fsw = lane & 7;
    const int a_row_off = (wm * (BM / 2) + frow) * BK;
    const int w_row_off = (wn * (BN / 2) + frow) * BK;

    const int KT = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_global(kt + 1);
        const bf16_t* pa = lds_a + buf * BM * BK + a_row_off;
        const bf16_t* pw = lds_w + buf * BN * BK + w_row_off;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int g = ((kk * 2 + fgrp) ^ fsw) * 8;
            bf16x8 fa[TM], fw[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(pa + i * 32 * BK + g);
#pragma unroll
            for (int j = 0; j < TN; ++j) fw[j] = *reinterpret_cast<const bf16x8*>(pw + j * 32 * BK + g);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fw[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue.  Accumulator element v of a 32x32 block: row 8*(v/4) + 4*(lane/32) + v%4, column lane%32.
    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int mb = m0 + wm * (BM / 2) + i * 32 + row_in;
        if (MODE == GEMM_SWIGLU_BF16) {
            // block columns alternate gate (even j) / up (odd j) for the same 32 outputs
#pragma unroll
            for (int j = 0; j < TN; j += 2) {
                const int n_packed = n0 + wn * (BN / 2) + j * 32;
                const int oc = n_packed / 2 + col_in;
                bf16_t* o = reinterpret_cast<bf16_t*>(out);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = mb + 8 * (v / 4) + (v % 4);
                    if (m < M) o[(int64_t)m * ldc + oc] = (bf16_t)(silu(acc[i][j][v]) * acc[i][j + 1][v]);
                }
            }
        } else {
            float* o = reinterpret_cast<float*>(out);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * (BN / 2) + j * 32 + col_in;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = mb + 8 * (v / 4) + (v % 4);
                    if (m < M) {
                        float* p = o + (int64_t)m * ldc + n;
                        if (MODE == GEMM_ADD_F32) *p += acc[i][j][v];
                        else *p = acc[i][j][v];
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int MODE>
hipError_t launch_tile(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc, int m,
                       int n, int k, hipStream_t stream) {
    const int tiles_m = (int)ceil_div(m, BM), tiles_n = n / BN;
    const size_t smem = 2 * (BM + BN) * BK * sizeof(bf16_t);
    auto kern = gemm_bf16_kernel<BM, BN, MODE>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kern<<<tiles_m * tiles_n, 256, smem, stream>>>(a, lda, w, ldw, out, ldc, m, n, k, tiles_m, tiles_n);
    return hipGetLastError();
}

template <int MODE>
hipError_t launch_mode(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc, int m,
                       int n, int k, hipStream_t stream) {
    return launch_tile<128, 128, MODE>(a, lda, w, ldw, out, ldc, m, n, k, stream);
}

}  // namespace

hipError_t launch_gemm_bf16(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc,
                            int m, int n, int k, int mode, hipStream_t stream) {
    if (m <= 0) return hipSuccess;
    if (n <= 0 || k <= 0 || n % 128 != 0 || k % BK != 0) return hipErrorInvalidValue;
    switch (mode) {
        case GEMM_STORE_F32: return launch_mode<GEMM_STORE_F32>(a, lda, w, ldw, out, ldc, m, n, k, stream);
        case GEMM_ADD_F32: return launch_mode<GEMM_ADD_F32>(a, lda, w, ldw, out, ldc, m, n, k, stream);
        case GEMM_SWIGLU_BF16: return launch_mode<GEMM_SWIGLU_BF16>(a, lda, w, ldw, out, ldc, m, n, k, stream);
        default: return hipErrorInvalidValue;
    }
}
