// bf16 x bf16 -> fp32 GEMM on the CDNA4 matrix cores:  out[m][n] (op)= sum_k a[m][k] * w[n][k].
//
// Both operands are contiguous along k, which is the order the MFMA operand registers want
// (each lane feeds 8 consecutive k of one row), so tiles go global -> LDS -> registers without
// any transposition.  A workgroup of WGM x WGN wavefronts owns a BM x BN output tile and walks k
// in steps of 64 through two LDS stages.  Tiles are brought in with global_load_lds (16 bytes per
// lane straight into LDS, no staging registers): the loads of step i+1 are issued right after the
// barrier that ends step i-1 and complete under the MFMAs of step i.
//
// LDS stage layout: rows of 64 k-values (128 bytes = eight 16-byte groups), A rows first, then W
// rows.  Two consecutive rows form a 256-byte line of 16 group positions (the width of the 64 LDS
// banks); group c of row r sits at position ((r & 1) * 8 + c) ^ ((r >> 1) & 7) of line r >> 1.  The
// 16-byte operand reads of the MFMA loop take, per 16 lanes, one group index of 16 consecutive rows:
// with this placement those 16 reads fall into 16 different bank groups (measured: the plain
// c ^ (r & 7) placement costs a 2-way bank conflict on every read).  A global_load_lds instruction
// fills 1 KiB = 4 lines: lane l owns position l % 16 of line l / 16 and fetches the global group that
// belongs there; the 16 lanes of a line still cover the full 128 bytes of both of its rows.
//
// Workgroup -> tile mapping: hardware hands consecutive workgroup ids to the 8 XCDs in turn, each
// with its own L2.  Ids are first regrouped so that an XCD receives a contiguous range of tile
// numbers; tiles are numbered band by band (a band is 8 tile-columns wide, walked row by row), so
// the tiles an XCD works on at one time share a few A row-panels and W row-panels in its L2.
#include "common.h"

#include <cmath>

namespace {

constexpr int BK = 64;
constexpr int kAuxNonTemporal = 2;  // cache-policy operand of global_load_lds: the nt bit

// silu(z) = z / (1 + e^-z) with the hardware exp2 and reciprocal (1 ulp each; the result is rounded to bf16)
__device__ __forceinline__ float silu(float z) {
    return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Hardware hands consecutive workgroup ids to the 8 XCDs in turn; this turns id `wg` of `count` into a work number such
// that every XCD receives one contiguous range of work numbers (XCD x gets workgroups x, x+8, ...: count / 8 of them,
// one more for x < count % 8).
__device__ __forceinline__ int xcd_contiguous(int wg, int count) {
    const int q = count >> 3, rem = count & 7;
    const int xcd = wg & 7, idx = wg >> 3;
    return xcd * q + min(xcd, rem) + idx;
}

// The work of one workgroup: output tile number `tile_idx` (in XCD-contiguous numbering, see above) of a tiles_m x
// tiles_n grid of BM x BN tiles whose first column is n_base and whose first row is m_base, k-share `split` of
// `num_splits` (each share has its own output plane).
// NS LDS stages of 64 k-values for the A tile and NSW (NS or NS + 1) for the W tile.  The weights stream from HBM,
// the activations are re-read from the caches by every tile column, so where LDS cannot hold one more stage of both
// (256x256: two of each fill 128 of the 160 KiB) the W tile alone gets the third: its loads then have two k-steps
// to land instead of one.
template <int BM, int BN, int WGM, int WGN, int MODE, int NS = 2, int NSW = NS, bool W_ONCE = false>
__device__ __forceinline__ void gemm_tile(const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ W,
                                          int64_t ldw, void* __restrict__ out, int64_t ldc, int M, int K,
                                          int tiles_m, int tiles_n, int n_base, int tile_idx, int split, int num_splits,
                                          int64_t split_stride, int m_base = 0) {
    constexpr int NW = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 blocks per wave
    constexpr int GA = BM / 8 / NW, GW = BN / 8 / NW;  // 1 KiB load groups per wave and stage: A, W
    constexpr int GPW = GA + GW;
    constexpr int A_STAGE = BM * BK * 2, W_STAGE = BN * BK * 2, W_BASE = NS * A_STAGE;
    constexpr int LDS_BYTES = NS * A_STAGE + NSW * W_STAGE;
    static_assert(NSW == NS || NSW == NS + 1, "the W tile has as many stages as the A tile, or one more");
    static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0 && NW % 2 == 0, "load groups must divide among an even number of waves");
    static_assert(MODE != GEMM_SWIGLU_BF16 || TN % 2 == 0, "SwiGLU needs gate and up blocks in one wave");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // ---- tile assignment: tiles are numbered band by band ----
    const int wg = tile_idx;
    constexpr int BAND = 8;  // tile columns per band
    const int band = wg / (BAND * tiles_m);
    const int band_cols = min(BAND, tiles_n - band * BAND);
    const int in_band = wg - band * BAND * tiles_m;
    const int tile_m = in_band / band_cols;
    const int tile_n = band * BAND + in_band % band_cols;
    const int m0 = m_base + tile_m * BM, n0 = n_base + tile_n * BN;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // split-K: a share is a contiguous part of the k range with its own output plane
    const int KT = (K / BK) / num_splits;
    const int kt_base = split * KT;
    const int64_t split_off = (int64_t)split * split_stride;

    // ---- loader: wave w fills groups w, w + NW, ...; lane offsets are the same for every group ----
    // group g covers rows 8g .. 8g+7 = lines 4g .. 4g+3; NW is even, so g has the parity of `wave`
    const int lline = lane >> 4;
    const int lq = (lane & 15) ^ ((4 * (wave & 1) + lline) & 7);
    const int lrow = 2 * lline + (lq >> 3), lgrp = lq & 7;
    const uint32_t voff_a = (uint32_t)(lrow * lda + lgrp * 8) * 2u;
    // W is tiled (see w_tiled_index): a group's 8 rows x 64 k values are 1 KiB in a row, a 64-row block 8 KiB, so a load
    // instruction reads one contiguous KiB and a k-step of the tile whole 8 KiB pieces
    const uint32_t voff_w = (uint32_t)(lrow * 64 + lgrp * 8) * 2u;
    const int64_t w_blocks_k = ldw >> 6;
    const char* a_tile = reinterpret_cast<const char*>(A + (int64_t)m0 * lda);
    const char* w_tile = reinterpret_cast<const char*>(W) + (int64_t)(n0 >> 6) * w_blocks_k * kWBlockBytes;
    // tile kt of A into A stage `stage` / of W into W stage `stage` (wave w fills groups w, w + NW, ...)
    auto issue_a = [&](int kt, int stage) {
        unsigned char* sbase = smem + stage * A_STAGE;
        const int64_t kbyte = (int64_t)(kt + kt_base) * (BK * 2);
#pragma unroll
        for (int i = 0; i < GA; ++i) {
            const int g = wave + i * NW;  // wave-uniform
            __builtin_amdgcn_global_load_lds((gptr_t)(a_tile + (int64_t)(g * 8) * lda * 2 + kbyte + voff_a), (lptr_t)(sbase + g * 1024), 16, 0, 0);
        }
    };
    auto issue_w = [&](int kt, int stage) {
        unsigned char* sbase = smem + W_BASE + stage * W_STAGE;
        const char* w_kt = w_tile + (int64_t)(kt + kt_base) * kWBlockBytes + voff_w;
        // group g = rows 8g .. 8g+7 of the tile: row block g / 8, KiB g % 8 of that block.  With one band of rows
        // (W_ONCE) every byte of W is read by one workgroup, once: those loads carry the non-temporal hint, which
        // keeps the one-pass stream from displacing the A panel in L2 (5-10 % on the weight-streaming products).
#pragma unroll
        for (int i = 0; i < GW; ++i) {
            const int g = wave + i * NW;
            __builtin_amdgcn_global_load_lds((gptr_t)(w_kt + (int64_t)(g >> 3) * w_blocks_k * kWBlockBytes + (g & 7) * 1024), (lptr_t)(sbase + g * 1024), 16, 0, W_ONCE ? kAuxNonTemporal : 0);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // operand reads: lane supplies row (lane % 32), k-group (lane / 32) of each 16-wide k step
    const int frow = lane & 31, fgrp = lane >> 5;
    bf16x8 fa[2][TM], fw[2][TN];
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fw[buf][j], acc[i][j], 0, 0, 0);
    };
    constexpr int kReads = TM + TN, kMfma = TM * TN;
    constexpr int kPaired = kReads < kMfma ? kReads : kMfma;

    {
        const int fsw = (frow >> 1) & 7, fpar = (frow & 1) * 8;
        const int a_off = (wm * WTM + (frow & ~1)) * (BK * 2);
        const int w_off = W_BASE + (wn * WTN + (frow & ~1)) * (BK * 2);
        auto load_frags = [&](int kt, int kk, int buf) {  // fragments of k-step kk of tile kt
            const unsigned char* sa = smem + (kt % NS) * A_STAGE + a_off;
            const unsigned char* sw = smem + (kt % NSW) * W_STAGE + w_off;
            const int g = ((fpar + kk * 2 + fgrp) ^ fsw) * 16;
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * (BK * 2) + g);
#pragma unroll
            for (int j = 0; j < TN; ++j) fw[buf][j] = *reinterpret_cast<const bf16x8*>(sw + j * 32 * (BK * 2) + g);
        };
        // scheduling hint for one "fetch fragments of the next k-step, multiply the current one" step:
        // spread the LDS reads between the MFMAs so that their latency is covered
        auto interleave = [&]() {
            // reads first, one per MFMA, so that the MFMAs left over cover the latency of the last read
#pragma unroll
            for (int r = 0; r < kPaired; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA (first, so that the wait for the
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // previous reads precedes every new read)
            }
            __builtin_amdgcn_sched_group_barrier(0x100, kReads - kPaired, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, kMfma - kPaired, 0);
        };
        // the step after the barrier also issues the next tile's global loads: one per MFMA, so that the
        // matrix cores keep running while the loads are handed to the memory pipeline
        constexpr int kLoadsPerMfma = (GPW + kMfma - 1) / kMfma;
        auto interleave_with_loads = [&]() {
#pragma unroll
            for (int r = 0; r < kMfma; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (r * kLoadsPerMfma < GPW) __builtin_amdgcn_sched_group_barrier(0x020, kLoadsPerMfma, 0);
                if (r < kReads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        };

        // Software pipeline.  Global: tiles kt+1 .. kt+NS-1 of A (.. kt+NSW-1 of W) are in flight while tile kt is
        // multiplied.  LDS -> registers: the fragments of k-step kk+1 are fetched while k-step kk is multiplied, also
        // across the tile boundary: the barrier sits before the last k-step of a tile, after which the next tile's
        // first fragments are fetched under the MFMAs of that last k-step.  Loads past the last tile re-read it into
        // a stage nobody reads again, so every iteration issues the same number of loads and the wait counts are
        // compile-time constants.  Loads complete in issue order: each step issues its A tile before its W tile, so
        // "all but the newest ..." leaves exactly the tiles that may still be in flight.
        constexpr int KK = BK / 16;
        constexpr int kInFlight = (NS - 2) * GPW + (NSW - NS) * GW;  // loads that may be outstanding at a step's barrier
        static_assert(kInFlight + GPW < 64, "outstanding loads must fit the vmcnt field");
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            issue_a(min(i, KT - 1), i);
            issue_w(min(i, KT - 1), i);
        }
        if (NSW > NS) issue_w(min(NS, KT - 1), NS);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 1) * GPW + (NSW - NS) * GW) : "memory");
        __builtin_amdgcn_s_barrier();
        load_frags(0, 0, 0);
        for (int kt = 0; kt < KT - 1; ++kt) {
#pragma unroll
            for (int kk = 0; kk < KK - 1; ++kk) {
                load_frags(kt, kk + 1, (kk + 1) & 1);
                mfmas(kk & 1);
                interleave();
            }
            // tile kt+1 must have landed (later tiles may still be in flight) and this wave's last fragments of
            // tile kt must be in registers before anybody overwrites its stages
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(kInFlight) : "memory");
            __builtin_amdgcn_s_barrier();
            // branch-free tail (one scheduling region): the loads into the stages just vacated, the first fragments
            // of tile kt+1, the last MFMAs of tile kt
            issue_a(min(kt + NS, KT - 1), kt % NS);
            issue_w(min(kt + NSW, KT - 1), kt % NSW);
            load_frags(kt + 1, 0, KK & 1);
            mfmas((KK - 1) & 1);
            interleave_with_loads();
        }
        {
#pragma unroll
            for (int kk = 0; kk < KK - 1; ++kk) {
                load_frags(KT - 1, kk + 1, (kk + 1) & 1);
                mfmas(kk & 1);
                interleave();
            }
            mfmas((KK - 1) & 1);
        }
    }

    // ---- epilogue, staged through LDS so that every global access is a 16-byte piece of a long row
    // segment.  Accumulator element v of a 32x32 block sits at row 8*(v/4) + 4*(lane/32) + v%4, column
    // lane%32; a wave writes one 32-row slab of its tile to its private LDS area, then reads it back row
    // by row, 4 consecutive columns per lane.  Only the first barrier is needed (the slabs overlay the tiles).
    constexpr int C = (MODE == GEMM_SWIGLU_BF16) ? WTN / 2 : WTN;  // result columns of a wave slab
    constexpr int CS = C + 8;                                       // padded row stride (floats)
    constexpr int LPR = C / 4;                                      // lanes per row on the way out
    constexpr int RPI = 64 / LPR;                                   // rows per read instruction (lanes >= RPI*LPR idle)
    static_assert(32 % RPI == 0, "a slab must be a whole number of read instructions");
    static_assert(NW * 32 * CS * 4 <= LDS_BYTES, "epilogue slab must fit in the tile buffers");
    float* slab = reinterpret_cast<float*>(smem) + wave * (32 * CS);
    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
    const int orow = lane / LPR, ocol = (lane % LPR) * 4;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the redundant tail loads have landed too
    __syncthreads();  // all waves have finished reading the last tile
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (MODE == GEMM_SWIGLU_BF16) {
            // block columns alternate gate (even j) / up (odd j) for the same 32 outputs
#pragma unroll
            for (int j = 0; j < TN; j += 2)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    slab[(8 * (v / 4) + row_in + (v % 4)) * CS + (j / 2) * 32 + col_in] =
                        silu(acc[i][j][v]) * acc[i][j + 1][v];
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    slab[(8 * (v / 4) + row_in + (v % 4)) * CS + j * 32 + col_in] = acc[i][j][v];
        }
        // the slab is private to the wave and LDS executes a wave's instructions in order: no barrier needed
        const int mrow0 = m0 + wm * WTM + i * 32;
        const bool lane_on = RPI * LPR == 64 || lane < RPI * LPR;
        f32x4 val[32 / RPI];
#pragma unroll
        for (int r = 0; r < 32; r += RPI)  // all reads first, so that their latencies overlap
            val[r / RPI] = *reinterpret_cast<const f32x4*>(slab + (r + (lane_on ? orow : 0)) * CS + (lane_on ? ocol : 0));
#pragma unroll
        for (int r = 0; r < 32; r += RPI) {
            const int m = mrow0 + r + orow;
            if (!lane_on || m >= M) continue;
            if (MODE == GEMM_SWIGLU_BF16) {
                bf16_t* p = reinterpret_cast<bf16_t*>(out) + (int64_t)m * ldc + (n0 + wn * WTN) / 2 + ocol;
                *reinterpret_cast<bf16x4*>(p) = __builtin_convertvector(val[r / RPI], bf16x4);
            } else {
                float* p = reinterpret_cast<float*>(out) + split_off + (int64_t)m * ldc + n0 + wn * WTN + ocol;
                if (MODE == GEMM_ADD_F32) {
                    f32x4 old = *reinterpret_cast<const f32x4*>(p);
                    *reinterpret_cast<f32x4*>(p) = old + val[r / RPI];
                } else {
                    *reinterpret_cast<f32x4*>(p) = val[r / RPI];
                }
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN, int MODE, int NS = 2, int NSW = NS, bool W_ONCE = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                    const bf16_t* __restrict__ W, int64_t ldw,
                                                                    void* __restrict__ out, int64_t ldc, int M,
                                                                    int K, int tiles_m, int tiles_n,
                                                                    int64_t split_stride) {
    // Split-K launches are a (tiles, splits) grid; workgroup ids run over the tiles first.  All of it is renumbered at
    // once, k-share by k-share, so that an XCD works on tiles of ONE k-share at a time where it can: the tiles that
    // share its L2 then read the same k range of their A and W panels (with both shares of a tile range on one XCD,
    // as the plain per-share numbering would place them, the L2 sees half as many tiles per panel).
    const int num_tiles = tiles_m * tiles_n;
    const int v = xcd_contiguous(blockIdx.x + blockIdx.y * num_tiles, num_tiles * (int)gridDim.y);
    gemm_tile<BM, BN, WGM, WGN, MODE, NS, NSW, W_ONCE>(A, lda, W, ldw, out, ldc, M, K, tiles_m, tiles_n, 0, v % num_tiles,
                                                       v / num_tiles, gridDim.y, split_stride);
}

// Two tile shapes in one launch: the first big_tiles workgroups cover columns [0, n_split) with 256x256
// tiles (whole rounds of the 256 compute units), the rest cover [n_split, N) with 256x128 tiles, so that
// the last, partial round still gives every compute unit a (half-size) tile.  8 waves either way.
template <int MODE, int NSW>
__global__ __launch_bounds__(512) void gemm_bf16_mixed_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                               const bf16_t* __restrict__ W, int64_t ldw,
                                                               void* __restrict__ out, int64_t ldc, int M, int K,
                                                               int tiles_m, int big_cols, int small_cols) {
    const int big_tiles = tiles_m * big_cols;
    if ((int)blockIdx.x < big_tiles)
        gemm_tile<256, 256, 2, 4, MODE, 2, NSW>(A, lda, W, ldw, out, ldc, M, K, tiles_m, big_cols, 0,
                                                xcd_contiguous(blockIdx.x, big_tiles), 0, 1, 0);
    else
        gemm_tile<256, 128, 4, 2, MODE, 2, NSW>(A, lda, W, ldw, out, ldc, M, K, tiles_m, small_cols, big_cols * 256,
                                                xcd_contiguous(blockIdx.x - big_tiles, tiles_m * small_cols), 0, 1, 0);
}

// Two tile heights in one launch: the first big_tiles workgroups cover the whole bands of 256 rows with 256x256
// tiles, the rest cover the last band -- at most BMR rows are left -- with BMR x 256 tiles, so a row count just above a
// multiple of 256 does not pay for a whole band of padding.  8 waves either way; blockIdx.y is the split-K share.
template <int MODE, int BMR, int NSW>
__global__ __launch_bounds__(512) void gemm_bf16_rowmix_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                const bf16_t* __restrict__ W, int64_t ldw,
                                                                void* __restrict__ out, int64_t ldc, int M, int K,
                                                                int bands, int tiles_n, int64_t split_stride) {
    const int big_tiles = bands * tiles_n;
    if ((int)blockIdx.x < big_tiles)
        gemm_tile<256, 256, 2, 4, MODE, 2, NSW>(A, lda, W, ldw, out, ldc, M, K, bands, tiles_n, 0,
                                                xcd_contiguous(blockIdx.x, big_tiles), blockIdx.y, gridDim.y, split_stride);
    else
        gemm_tile<BMR, 256, 2, 4, MODE, 2, NSW>(A, lda, W, ldw, out, ldc, M, K, 1, tiles_n, 0,
                                                xcd_contiguous(blockIdx.x - big_tiles, tiles_n), blockIdx.y, gridDim.y,
                                                split_stride, bands * 256);
}

template <int BM, int BN, int WGM, int WGN, int MODE, int NS, int NSW, bool W_ONCE>
hipError_t launch_tile_w(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc, int m,
                         int n, int k, int splits, int64_t split_stride, hipStream_t stream) {
    const int tiles_m = (int)ceil_div(m, BM), tiles_n = n / BN;
    const size_t smem = (NS * BM + NSW * BN) * BK * sizeof(bf16_t);
    auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, MODE, NS, NSW, W_ONCE>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kern<<<dim3(tiles_m * tiles_n, splits), 64 * WGM * WGN, smem, stream>>>(a, lda, w, ldw, out, ldc, m, k, tiles_m,
                                                                          tiles_n, split_stride);
    return hipGetLastError();
}

// All rows in one band: the weights are read once (W_ONCE, see gemm_tile).
template <int BM, int BN, int WGM, int WGN, int MODE, int NS = 2, int NSW = NS>
hipError_t launch_tile(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc, int m,
                       int n, int k, int splits, int64_t split_stride, hipStream_t stream) {
    if (n % BN != 0) return hipErrorInvalidValue;
    return m <= BM ? launch_tile_w<BM, BN, WGM, WGN, MODE, NS, NSW, true>(a, lda, w, ldw, out, ldc, m, n, k, splits, split_stride, stream)
                   : launch_tile_w<BM, BN, WGM, WGN, MODE, NS, NSW, false>(a, lda, w, ldw, out, ldc, m, n, k, splits, split_stride, stream);
}

template <int MODE>
hipError_t launch_mode(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc, int m,
                       int n, int k, int tile, int splits, int64_t split_stride, hipStream_t stream) {
#define GLLM_TILE_ARGS a, lda, w, ldw, out, ldc, m, n, k, splits, split_stride, stream
    switch (tile) {
        case 0: return launch_tile<128, 128, 2, 2, MODE>(GLLM_TILE_ARGS);
        case 1: return launch_tile<256, 128, 2, 2, MODE>(GLLM_TILE_ARGS);
        case 2: return launch_tile<256, 256, 2, 2, MODE>(GLLM_TILE_ARGS);
        case 3: return launch_tile<256, 256, 2, 4, MODE>(GLLM_TILE_ARGS);
        case 10: return launch_tile<256, 256, 2, 4, MODE, 2, 3>(GLLM_TILE_ARGS);  // third LDS stage for the W tile: all 160 KiB
        case 6: return launch_tile<128, 128, 2, 2, MODE, 4>(GLLM_TILE_ARGS);
        case 7: return launch_tile<64, 128, 2, 2, MODE, 3>(GLLM_TILE_ARGS);
        case 9:  // one 288-row tile covers all rows; it reads 288 of them, which the row padding (to 256) covers above 256
            if constexpr (MODE != GEMM_SWIGLU_BF16) {
                if (m <= 256 || m > 288) return hipErrorInvalidValue;
                return launch_tile<288, 192, 3, 2, MODE>(GLLM_TILE_ARGS);
            } else return hipErrorInvalidValue;
        case 5:
            if constexpr (MODE != GEMM_SWIGLU_BF16) return launch_tile<256, 192, 4, 2, MODE>(GLLM_TILE_ARGS);
            else return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
#undef GLLM_TILE_ARGS
}

// Mixed launch (see gemm_bf16_mixed_kernel); rem_cols 256-wide tile columns are turned into 2*rem_cols
// 128-wide ones.
template <int MODE, int NSW>
hipError_t launch_mixed(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc, int m,
                        int n, int k, int rem_cols, hipStream_t stream) {
    const int tiles_m = (int)ceil_div(m, 256), big_cols = n / 256 - rem_cols, small_cols = 2 * rem_cols;
    const size_t smem = (2 * 256 + NSW * 256) * BK * sizeof(bf16_t);
    auto kern = gemm_bf16_mixed_kernel<MODE, NSW>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kern<<<tiles_m * (big_cols + small_cols), 512, smem, stream>>>(a, lda, w, ldw, out, ldc, m, k, tiles_m, big_cols,
                                                                   small_cols);
    return hipGetLastError();
}

// Row-mixed launch (see gemm_bf16_rowmix_kernel); rem_rows is 64 or 128.
template <int MODE, int NSW>
hipError_t launch_rowmix(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc, int m,
                         int n, int k, int rem_rows, int splits, int64_t split_stride, hipStream_t stream) {
    const int bands = m / 256, tiles_n = n / 256;
    const size_t smem = (2 * 256 + NSW * 256) * BK * sizeof(bf16_t);
    const dim3 grid((bands + 1) * tiles_n, splits);
#define GLLM_ROWMIX(R)                                                                                             \
    do {                                                                                                           \
        auto kern = gemm_bf16_rowmix_kernel<MODE, R, NSW>;                                                           \
        static bool configured = false;                                                                            \
        if (!configured) {                                                                                         \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);             \
            if (e != hipSuccess) return e;                                                                         \
            configured = true;                                                                                     \
        }                                                                                                          \
        kern<<<grid, 512, smem, stream>>>(a, lda, w, ldw, out, ldc, m, k, bands, tiles_n, split_stride);          \
    } while (0)
    if (rem_rows == 64) GLLM_ROWMIX(64);
    else GLLM_ROWMIX(128);
#undef GLLM_ROWMIX
    return hipGetLastError();
}

}  // namespace

// Height of the last row band for a row-mixed launch (64 or 128), or 0 when the shape does not call for one: at
// least one whole band of 256 rows and at most 128 rows left over.
int gemm_rowmix_rem_rows(int m, int n) {
    if (n % 256 != 0 || m <= 256) return 0;
    const int r = m % 256;
    return r == 0 || r > 128 ? 0 : r <= 64 ? 64 : 128;
}

// Number of 256-wide tile columns to split in two for a mixed launch, or 0 when a plain launch is as good:
// worth it when the last round of 256x256 tiles would occupy at most half of the compute units.
int gemm_mixed_rem_cols(int m, int n) {
    if (n % 256 != 0) return 0;
    const int tiles_m = (int)ceil_div(m, 256), cols = n / 256;
    const int tiles = tiles_m * cols, rem = tiles % 256;
    if (tiles < 256 || rem == 0 || rem > 128 || rem % tiles_m != 0) return 0;
    return rem / tiles_m;
}

// Tile shape and split-K factor for a problem, from a small cost model fitted to measurements on MI355X with
// operands streaming from HBM (weights are cold in the stage).  Unit: the time of one k-step of a 256x256 tile
// (~1.65 us).  A 256x256 tile (8 waves, one workgroup per compute unit) costs k_steps + 6 (prologue, epilogue)
// per round of 256 tiles; a 256x192 tile 0.88 k_steps + 6; a 128x128 tile 0.70 k_steps + 2.3 per round of 512
// tiles when two share a compute unit, 0.49 k_steps + 2.3 when alone (15 % less with four LDS stages, used
// for few rows).  A partial last round of 256x256 tiles that covers at most half of the compute units can be
// run with half-width tiles instead (mixed launch, ~0.55 of a round).  Split-K multiplies the number of tiles
// and divides the k-steps, at the price of writing one fp32 plane per split (mostly hidden under other tiles).
// For 257..288 rows a 288x192 tile (6 waves, wave tile 96x96) covers all rows in one band.
// Up to 64 rows the product is a stream of the weights: a 64x128 tile with three LDS stages (two workgroups per
// compute unit, 64 KiB of weights in flight on each, half the activation traffic of a 128-row tile) costs
// 0.30 k_steps per tile, but not less than the weights take at 5.5 TB/s, plus 2; measured 20-35 % faster than
// every other shape there, so it is the only candidate for such problems and the model only picks its split.
GemmPlan gemm_plan(int m, int n, int k, int mode, int max_splits, bool row_mixed) {
    const int its = k / BK;
    GemmPlan best{0, 1};
    double best_cost = 1e30;
    if (mode != GEMM_STORE_F32) max_splits = 1;
    for (int s = 1; s <= max_splits; s *= 2) {
        if (its % s != 0 || (s > 1 && its / s < 8)) continue;
        const double steps = (double)its / s;
        const double plane_cost = (double)m * n * 4.0 * s / 8e12 / 1.65e-6;  // mostly hidden under other tiles
        const bool skinny = m <= 64 && n % 128 == 0;
        if (row_mixed && gemm_rowmix_rem_rows(m, n) > 0) {
            // (evaluated first: on equal cost it is kept -- whole rounds hide that it always does less work)
            // whole bands as 256x256 tiles; the last band's tiles go first into the compute units the last round of
            // big tiles leaves idle; those that do not fit there stream their weights from HBM once more and cost
            // 0.8 (64 rows) or 0.9 (128 rows) of a big tile (measured on the 128256-column vocabulary projection)
            const int rr = gemm_rowmix_rem_rows(m, n);
            const double frac = rr == 64 ? 0.8 : 0.9;
            const int64_t big = (int64_t)(m / 256) * (n / 256) * s, small = (int64_t)(n / 256) * s;
            const int64_t rem_big = big % 256;
            const int64_t room = rem_big > 0 ? (256 - rem_big) * (rr == 64 ? 2 : 1) : 0;
            double rounds = (double)ceil_div(big, 256);
            if (small > room) rounds += frac * (double)ceil_div(small - room, 256);
            const double cost = rounds * (steps + 6.0) + plane_cost;
            if (cost < best_cost) { best_cost = cost; best = GemmPlan{8, s}; }
        }
        if (n % 256 == 0 && !skinny) {
            const int64_t tiles = ceil_div(m, 256) * (int64_t)(n / 256) * s;
            const bool mixed = s == 1 && gemm_mixed_rem_cols(m, n) > 0;
            const double rounds = mixed ? (double)(tiles / 256) + 0.55 : (double)ceil_div(tiles, 256);
            const double cost = rounds * (steps + 6.0) + plane_cost;
            if (cost < best_cost) { best_cost = cost; best = GemmPlan{mixed ? 4 : 3, s}; }
        }
        if (n % 192 == 0 && mode != GEMM_SWIGLU_BF16 && !skinny) {
            const int64_t tiles = ceil_div(m, 256) * (int64_t)(n / 192) * s;
            const double cost = (double)ceil_div(tiles, 256) * (steps * 0.88 + 6.0) + plane_cost;
            if (cost < best_cost) { best_cost = cost; best = GemmPlan{5, s}; }
        }
        if (m > 256 && m <= 288 && n % 192 == 0 && mode != GEMM_SWIGLU_BF16) {
            // 257..288 rows (a micro-batch of 256 decode rows plus the ends of a few chunks): one 288x192 tile per
            // column block reads the weights once where every 256-row shape needs a second band; a k-step of it costs
            // 1.07 of a 256x256 one when the weights stream from HBM
            const int64_t tiles = (int64_t)(n / 192) * s;
            const double cost = (double)ceil_div(tiles, 256) * (steps * 1.07 + 6.0) + plane_cost;
            if (cost < best_cost) { best_cost = cost; best = GemmPlan{9, s}; }
        }
        if (n % 128 == 0 && !skinny) {
            const int64_t tiles = ceil_div(m, 128) * (int64_t)(n / 128) * s;
            const int64_t full = tiles / 512, rem = tiles % 512;
            double cost = (double)full * (steps * 0.70 + 2.3) + plane_cost;
            if (rem > 256) cost += steps * 0.70 + 2.3;
            else if (rem > 0) cost += steps * 0.49 + 2.3;
            // few rows: every tile is alone on its compute unit; the 4-stage variant keeps three k-steps of
            // loads in flight (measured +10..20 % there)
            const bool deep = m <= 256 && tiles <= 256;
            if (deep) cost *= 0.85;
            if (cost < best_cost) { best_cost = cost; best = GemmPlan{deep ? 6 : 0, s}; }
        }
        if (m > 128 && m <= 256 && n % 128 == 0) {
            // 129..256 rows: 256x128 tiles take all rows in one band, so the weights are read once (with the
            // non-temporal hint) where the 128-row shapes read them twice; measured 0.67 of a 256x256 k-step and a
            // fixed 3; wins where the product cannot be split along k (gate/up: 4-9 % over the 128x128 tiles)
            const int64_t tiles = (int64_t)(n / 128) * s;
            const double cost = (double)ceil_div(tiles, 256) * (steps * 0.67 + 3.0) + plane_cost;
            if (cost < best_cost) { best_cost = cost; best = GemmPlan{1, s}; }
        }
        if (skinny) {
            const int64_t tiles = (int64_t)(n / 128) * s;
            const double stream = (double)n * k * 2.0 / 5.5e12 / 1.65e-6;
            const double cost = std::max((double)ceil_div(tiles, 512) * steps * 0.30, stream) + 2.0 + plane_cost;
            if (cost < best_cost) { best_cost = cost; best = GemmPlan{7, s}; }
        }
    }
    // The 256x256 tile shapes exist with a third LDS stage for the W tile (ids 10, 11, 12 for 3, 4, 8): two k-steps for the
    // weight loads to land instead of one.  Measured against the two-stage forms on the four stage shapes (weights cold):
    // +3..5 % where a tile walks 80 or more k-steps (hidden >= 5120; the down projection), +15..20 % at 512 rows and
    // below, where the product is bound by the weight stream; even or -2 % on short k with many rows (hidden 4096 at
    // 2048 rows), where the loads land in time anyway.
    const int steps = its / best.splits;
    if ((best.tile == 3 || best.tile == 4 || best.tile == 8) && (steps >= 80 || m <= 1024))
        best.tile = best.tile == 3 ? 10 : best.tile == 4 ? 11 : 12;
    return best;
}

hipError_t launch_gemm_bf16(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc,
                            int m, int n, int k, int mode, int tile, int splits, int64_t split_stride,
                            hipStream_t stream) {
    if (m <= 0) return hipSuccess;
    if (n <= 0 || k <= 0 || n % 64 != 0 || k % BK != 0) return hipErrorInvalidValue;
    if (lda * 16 >= (int64_t)1 << 31 || ldw % kWBlock != 0 || ldw < k) return hipErrorInvalidValue;
    if (splits < 1 || (k / BK) % splits != 0) return hipErrorInvalidValue;
    if (splits > 1 && mode != GEMM_STORE_F32) return hipErrorInvalidValue;
    if (tile < 0) {
        tile = gemm_plan(m, n, k, splits == 1 ? mode : GEMM_ADD_F32, 1).tile;  // tile for the given split count
        if (splits > 1) {
            // splits fixed by the caller: compare the two tile shapes at that split count
            const int64_t t3 = ceil_div(m, 256) * (int64_t)(n / 256) * splits, t0 = ceil_div(m, 128) * (int64_t)(n / 128) * splits;
            const double steps = (double)(k / BK) / splits;
            const double c3 = n % 256 == 0 ? (double)ceil_div(t3, 256) * (steps + 6.0) : 1e30;
            const double c0 = (double)(t0 / 512) * (steps * 0.70 + 2.3) +
                              (t0 % 512 > 256 ? steps * 0.70 + 2.3 : t0 % 512 > 0 ? steps * 0.49 + 2.3 : 0.0);
            tile = m <= 64 ? 7 : c3 <= c0 ? ((steps >= 80 || m <= 1024) ? 10 : 3) : (m <= 256 && t0 <= 256) ? 6 : 0;
        }
    }
    if (tile == 8 || tile == 12) {  // 256x256 tiles plus a last band of 64 or 128 rows (12: third W stage)
        const int rem_rows = gemm_rowmix_rem_rows(m, n);
        if (rem_rows == 0) return hipErrorInvalidValue;
#define GLLM_ROWMIX_MODE(MODE_)                                                                                              \
    (tile == 8 ? launch_rowmix<MODE_, 2>(a, lda, w, ldw, out, ldc, m, n, k, rem_rows, splits, split_stride, stream)          \
               : launch_rowmix<MODE_, 3>(a, lda, w, ldw, out, ldc, m, n, k, rem_rows, splits, split_stride, stream))
        switch (mode) {
            case GEMM_STORE_F32: return GLLM_ROWMIX_MODE(GEMM_STORE_F32);
            case GEMM_ADD_F32: return GLLM_ROWMIX_MODE(GEMM_ADD_F32);
            case GEMM_SWIGLU_BF16: return GLLM_ROWMIX_MODE(GEMM_SWIGLU_BF16);
            default: return hipErrorInvalidValue;
        }
#undef GLLM_ROWMIX_MODE
    }
    if (tile == 4 || tile == 11) {  // mixed 256x256 / 256x128 launch (11: third W stage)
        const int rem_cols = gemm_mixed_rem_cols(m, n);
        if (rem_cols == 0 || splits != 1) return hipErrorInvalidValue;
#define GLLM_MIXED_MODE(MODE_)                                                                    \
    (tile == 4 ? launch_mixed<MODE_, 2>(a, lda, w, ldw, out, ldc, m, n, k, rem_cols, stream)      \
               : launch_mixed<MODE_, 3>(a, lda, w, ldw, out, ldc, m, n, k, rem_cols, stream))
        switch (mode) {
            case GEMM_STORE_F32: return GLLM_MIXED_MODE(GEMM_STORE_F32);
            case GEMM_ADD_F32: return GLLM_MIXED_MODE(GEMM_ADD_F32);
            case GEMM_SWIGLU_BF16: return GLLM_MIXED_MODE(GEMM_SWIGLU_BF16);
            default: return hipErrorInvalidValue;
        }
#undef GLLM_MIXED_MODE
    }
    switch (mode) {
        case GEMM_STORE_F32:
            return launch_mode<GEMM_STORE_F32>(a, lda, w, ldw, out, ldc, m, n, k, tile, splits, split_stride, stream);
        case GEMM_ADD_F32:
            return launch_mode<GEMM_ADD_F32>(a, lda, w, ldw, out, ldc, m, n, k, tile, splits, split_stride, stream);
        case GEMM_SWIGLU_BF16:
            return launch_mode<GEMM_SWIGLU_BF16>(a, lda, w, ldw, out, ldc, m, n, k, tile, splits, split_stride, stream);
        default: return hipErrorInvalidValue;
    }
}
