// Internal declarations shared by the HIP translation units of libgllm_stage (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPage = 16;        // KV slots per page
constexpr int kWave = 64;        // lanes per wavefront

// GEMM tile constants that the weight packer and the activation buffers must agree on.
constexpr int kMaxPlanes = 8;    // split-K partial outputs a consumer kernel can sum
constexpr int kGemmPadM = 256;   // activation rows are readable up to a multiple of this
constexpr int kGemmPadN = 256;   // packed weight rows are padded to a multiple of this
constexpr int kGemmPadK = 64;    // packed weight columns / activation row strides are multiples of this
constexpr int kSwigluGroup = 32; // gate/up interleave granularity of the packed gate-up matrix

// Weight operand of every GEMM here ("tiled"): blocks of 64 output rows x 64 k values, a block contiguous (64 rows of
// 128 bytes = 8 KiB), blocks ordered [row block][k block].  A k-step of a workgroup tile then reads whole 8 KiB pieces
// instead of one 128-byte piece per output row, which is what HBM serves well when the weights stream (few token rows).
// Element (n, k) of an [N][K] matrix, N and K multiples of 64:
constexpr int kWBlock = 64;
constexpr int kWBlockBytes = kWBlock * kWBlock * 2;
__host__ __device__ static inline int64_t w_tiled_index(int64_t n, int64_t k, int64_t K) {
    return (((n >> 6) * (K >> 6) + (k >> 6)) << 12) + ((n & 63) << 6) + (k & 63);
}

static inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

enum GemmMode { GEMM_STORE_F32 = 0, GEMM_ADD_F32 = 1, GEMM_SWIGLU_BF16 = 2 };

// ---- launchers (each enqueues on `stream` and returns the launch status) ----------------

// out (op)= a[m x k] * w[n x k]^T, see gllm_op_gemm_bf16 in the public header; w is tiled (w_tiled_index) with ldw its k
// extent (a multiple of 64, >= k).
// tile: -1 picks a tile shape from m and n; 0..3 force one (128x128, 256x128, 256x256, 256x256 with 8 waves);
// 4 forces the mixed 256x256 + 256x128 launch (only where gemm_mixed_rem_cols(m, n) > 0); 5 = 256x192 (not SwiGLU);
// 6 = 128x128 with four LDS stages; 7 = 64x128 with three LDS stages (up to 64 rows per tile row: weight streaming);
// 8 = 256x256 tiles for the whole bands of 256 rows plus 64x256 or 128x256 tiles for a last band of at most 128 rows
// (only where gemm_rowmix_rem_rows(m, n) > 0); 9 = 288x192; 10, 11, 12 = tiles 3, 4, 8 with a third LDS stage for the W tile.
// splits > 1 (store mode only): split s covers k range [s*k/splits, (s+1)*k/splits) and writes its partial
// product to out + s*split_stride floats; the consumer sums the planes in order.
hipError_t launch_gemm_bf16(const bf16_t* a, int64_t lda, const bf16_t* w, int64_t ldw, void* out, int64_t ldc,
                            int m, int n, int k, int mode, int tile, int splits, int64_t split_stride,
                            hipStream_t stream);
int gemm_mixed_rem_cols(int m, int n);
int gemm_rowmix_rem_rows(int m, int n);
// Tile id and split-K factor the cost model prefers (splits stays 1 unless mode is GEMM_STORE_F32); row_mixed says
// whether it may pick tile 8.
struct GemmPlan { int tile; int splits; };
GemmPlan gemm_plan(int m, int n, int k, int mode, int max_splits, bool row_mixed = true);

// Residual stream entry: x = float(in_bf16), h = bf16(rmsnorm(x) * gamma).
hipError_t launch_rmsnorm_from_bf16(const bf16_t* in, float* x, const bf16_t* gamma, bf16_t* h, int64_t ldh,
                                    int rows, int hidden, float eps, hipStream_t stream);
// x += y[0] + ... + y[planes-1] (planes may be 0; plane p at y + p*plane_stride), then
// h = bf16(rmsnorm(x) * gamma).  x is updated in place when planes > 0.
hipError_t launch_add_rmsnorm(float* x, const float* y, int planes, int64_t plane_stride, const bf16_t* gamma,
                              bf16_t* h, int64_t ldh, int rows, int hidden, float eps, hipStream_t stream);
// out_bf16 = RNE(x + y planes), and optionally out_f32 = that sum.
hipError_t launch_add_cast_out(const float* x, const float* y, int planes, int64_t plane_stride, bf16_t* out,
                               float* out_f32, int64_t count, hipStream_t stream);

// Weight repacking (device to device) into the tiled layout: rows [dst_row0, dst_row0 + rows) x columns [0, cols) of a
// tiled matrix whose k extent is k_dst come from the row-major src (row stride ld_src); cols a multiple of 8.  What lies
// outside stays as it is (the caller zeroes the padding).
hipError_t launch_pack_rows_tiled(const bf16_t* src, int64_t ld_src, int rows, int cols, bf16_t* dst, int64_t k_dst,
                                  int dst_row0, hipStream_t stream);
// The gate/up matrix, rows interleaved in groups of kSwigluGroup (gate group, then the matching up group), tiled.
hipError_t launch_pack_gate_up(const bf16_t* gate, const bf16_t* up, int inter, int hidden, bf16_t* dst,
                               int64_t k_dst, hipStream_t stream);

// A run of consecutive new tokens of one sequence that fall into one page: rows row0 .. row0 + n - 1 go to slots
// slot0 .. slot0 + n - 1 of `page`.
struct VTile {
    int32_t row0, n, page, slot0;
};
struct RopeKvArgs {
    const float* qkv;        // planes x [T][ld_qkv] fp32: q heads, then k heads, then v heads; planes are summed
    int64_t ld_qkv;
    int planes;
    int64_t plane_stride;
    const bf16_t* bias;      // [n_qkv] or null
    const float* rope_cs;    // [max_position][d/2][2] (cos, sin)
    const int32_t* tok_pos;  // [T]
    const int32_t* tok_page; // [T] physical page of the token's own position
    bf16_t* q_out;           // [T][n_q*d] bf16, rotated
    int64_t ld_q;
    bf16_t* k_pool;          // this layer's K pool
    bf16_t* v_pool;          // this layer's V pool
    int T, n_q, n_kv, d;
    // V of the rows listed in v_tiles (runs of new tokens inside one page) is written by extra workgroups, one per
    // (run, KV head), in 16-byte pieces of 8 slots; a token workgroup writes its own V only where tok_own_v says so (a run
    // of one: a decode row).  Without v_tiles every token writes its own V.
    const VTile* v_tiles;
    int n_vtiles;
    const int32_t* tok_own_v;  // [T], nonzero: the token's workgroup writes its V
};
hipError_t launch_rope_kv_write(const RopeKvArgs& a, hipStream_t stream);

struct AttnArgs {
    const bf16_t* q;          // [T][ld_q] rotated queries
    int64_t ld_q;
    const bf16_t* k_pool;     // this layer
    const bf16_t* v_pool;
    const int32_t* bt_flat;   // page ids, all sequences back to back
    bf16_t* out;              // [T][ld_o] bf16 attention output
    int64_t ld_o;
    int n_q, n_kv, d;
    float scale_log2;         // log2(e) / sqrt(d)
};

// Decode rows (one new token per sequence).  Work items split the keys of a row into
// partitions; every item writes one partial per query head, then a second kernel merges the rows
// that have more than one item (DecodeRow lists only those).
struct DecodeItem {
    int32_t row;       // token row
    int32_t bt_off;    // offset of the sequence's first page id in bt_flat
    int32_t kv_begin;  // first key of this partition (multiple of 32)
    int32_t kv_end;    // one past the last key of this partition
    int32_t single;    // 1: the row's only item; the kernel writes the normalised output itself
};
struct DecodeRow {
    int32_t row;        // token row
    int32_t first_item; // first partial of this row
    int32_t num_items;
    int32_t pad;
};
// order[i] = index of the item that workgroup group i works on (a permutation of 0 .. num_items-1)
hipError_t launch_decode_attention(const AttnArgs& a, const DecodeItem* items, const int32_t* order, int num_items,
                                   float* part_o, float* part_ml, hipStream_t stream);
hipError_t launch_decode_combine(const AttnArgs& a, const DecodeRow* rows, int num_rows, const float* part_o,
                                 const float* part_ml, hipStream_t stream);

// Prefill chunks: one work item per prefill_item_rows() consecutive query rows of a chunk.
int prefill_item_rows(int n_q, int n_kv);
struct PrefillItem {
    int32_t row0;      // first token row of the tile
    int32_t n_rows;    // valid query rows in the tile (1 .. prefill_item_rows)
    int32_t pos0;      // position of the first query row
    int32_t bt_off;    // offset of the sequence's first page id in bt_flat
};
hipError_t launch_prefill_attention(const AttnArgs& a, const PrefillItem* items, int num_items, hipStream_t stream);

// Ceiling probes (see kernels_peak.hip).  peak_mfma: workgroups x 4 waves x iters x 16 MFMAs of
// 2*32*32*16 flop each.  peak_read: reads `bytes` once.
hipError_t launch_peak_mfma(float* sink, int workgroups, int iters, hipStream_t stream);
hipError_t launch_peak_read(const void* src, int64_t bytes, void* sink, int workgroups, hipStream_t stream, bool non_temporal = false);
