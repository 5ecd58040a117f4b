// Memory-bound helper kernels of the stage: RMSNorm, residual-stream entry/exit casts,
// RoPE + paged KV write, weight repacking.  All are bound by HBM traffic and tiny next to
// the GEMMs and the attention kernels.
#include "common.h"

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Sum over the 256 threads of a workgroup; every thread receives the total.
__device__ __forceinline__ float block_sum_256(float v, float* red /*[4]*/) {
    v = wave_sum(v);
    int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = red[0] + red[1] + red[2] + red[3];
    __syncthreads();
    return t;
}

// One workgroup per row.  FROM_BF16: the row comes from the bf16 stage input and is also written out
// as the fp32 residual stream.  Otherwise the row is the fp32 residual stream plus `planes` partial
// GEMM outputs (summed in plane order and written back), so the residual add costs no extra pass.
// The row is kept in registers between the two phases (MAXV 16-byte pieces per thread).  PLANES >= 0 fixes the
// number of planes at compile time (the loop unrolls and all loads of a piece are issued together: with a few
// hundred rows the kernel is all latency); PLANES < 0 takes it from the argument.
template <bool FROM_BF16, int MAXV, int PLANES>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const bf16_t* __restrict__ in, float* __restrict__ x,
                                                       const float* __restrict__ y, int planes, int64_t plane_stride,
                                                       const bf16_t* __restrict__ gamma, bf16_t* __restrict__ h,
                                                       int64_t ldh, int hidden, float eps) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    float* xr = x + row * hidden;
    f32x4 keep[MAXV];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int j = (threadIdx.x + i * 256) * 4;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (j < hidden) {
            if (FROM_BF16) {
                v = __builtin_convertvector(*reinterpret_cast<const bf16x4*>(in + row * hidden + j), f32x4);
                *reinterpret_cast<f32x4*>(xr + j) = v;
            } else {
                v = *reinterpret_cast<const f32x4*>(xr + j);
                if constexpr (PLANES >= 0) {
                    f32x4 part[PLANES > 0 ? PLANES : 1];
#pragma unroll
                    for (int p = 0; p < PLANES; ++p)
                        part[p] = *reinterpret_cast<const f32x4*>(y + p * plane_stride + row * hidden + j);
#pragma unroll
                    for (int p = 0; p < PLANES; ++p) v += part[p];
                } else {
                    for (int p = 0; p < planes; ++p)
                        v += *reinterpret_cast<const f32x4*>(y + p * plane_stride + row * hidden + j);
                }
                if (planes > 0) *reinterpret_cast<f32x4*>(xr + j) = v;
            }
        }
        keep[i] = v;
        ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    }
    // the gains are fetched before the reduction's barriers, so that their latency overlaps the row's (with a few
    // hundred rows this kernel is a chain of latencies, not a stream)
    f32x4 gain[MAXV];
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int j = (threadIdx.x + i * 256) * 4;
        gain[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (j < hidden) gain[i] = __builtin_convertvector(*reinterpret_cast<const bf16x4*>(gamma + j), f32x4);
    }
    const float total = block_sum_256(ss, red);
    const float inv = 1.0f / sqrtf(total / (float)hidden + eps);
    bf16_t* hr = h + row * ldh;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int j = (threadIdx.x + i * 256) * 4;
        if (j < hidden) {
            f32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = keep[i][e] * inv * gain[i][e];
            *reinterpret_cast<bf16x4*>(hr + j) = __builtin_convertvector(o, bf16x4);
        }
    }
}

__global__ __launch_bounds__(256) void cast_out_kernel(const float* __restrict__ x, const float* __restrict__ y,
                                                        int planes, int64_t plane_stride, bf16_t* __restrict__ out,
                                                        float* __restrict__ out_f32, int64_t count4) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count4) return;
    f32x4 v = reinterpret_cast<const f32x4*>(x)[i];
    for (int p = 0; p < planes; ++p) v += reinterpret_cast<const f32x4*>(y + p * plane_stride)[i];
    reinterpret_cast<bf16x4*>(out)[i] = __builtin_convertvector(v, bf16x4);
    if (out_f32) reinterpret_cast<f32x4*>(out_f32)[i] = v;
}

// Element (dst_row0 + r, c) of the tiled dst (k extent k_dst) = src[r][c] for c < cols; the padding is left as it is
// (zeroed by the caller).
__global__ __launch_bounds__(256) void pack_rows_tiled_kernel(const bf16_t* __restrict__ src, int64_t ld_src, int rows,
                                                               int cols, bf16_t* __restrict__ dst, int64_t k_dst,
                                                               int dst_row0) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one 8-element group per thread
    int groups = cols / 8;
    if (i >= (int64_t)rows * groups) return;
    int r = (int)(i / groups), g = (int)(i % groups);
    *reinterpret_cast<u32x4*>(dst + w_tiled_index(dst_row0 + r, g * 8, k_dst)) =
        *reinterpret_cast<const u32x4*>(src + (int64_t)r * ld_src + g * 8);
}

// Packed gate/up matrix: outputs are taken 32 at a time; packed rows 64b .. 64b+31 are the gate
// rows 32b .. 32b+31, packed rows 64b+32 .. 64b+63 the matching up rows.
__global__ __launch_bounds__(256) void pack_gate_up_kernel(const bf16_t* __restrict__ gate, const bf16_t* __restrict__ up,
                                                            int inter, int hidden, bf16_t* __restrict__ dst,
                                                            int64_t k_dst) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int groups = hidden / 8;
    if (i >= (int64_t)inter * groups) return;
    int r = (int)(i / groups), g = (int)(i % groups);
    int64_t prow = (int64_t)(r / kSwigluGroup) * (2 * kSwigluGroup) + r % kSwigluGroup;
    *reinterpret_cast<u32x4*>(dst + w_tiled_index(prow, g * 8, k_dst)) =
        *reinterpret_cast<const u32x4*>(gate + (int64_t)r * hidden + g * 8);
    *reinterpret_cast<u32x4*>(dst + w_tiled_index(prow + kSwigluGroup, g * 8, k_dst)) =
        *reinterpret_cast<const u32x4*>(up + (int64_t)r * hidden + g * 8);
}

// V of one head of one run of tokens inside a page (see VTile): the page keeps the 16 slots of one head dimension contiguous
// (32 bytes), so a thread gathers one dimension of up to 8 consecutive tokens -- neighbouring lanes read
// neighbouring columns of the same rows -- and stores them as one 16-byte piece; neighbouring lanes store
// neighbouring pieces.  Pieces that the run covers only in part are stored slot by slot.  The value of an
// element is formed exactly as in the token workgroups (planes in order, then the bias).
__device__ __forceinline__ void write_v_tile(const RopeKvArgs& a, const VTile vt, int hd) {
    const int v_col0 = (a.n_q + a.n_kv) * a.d;
    const int pieces = a.d * 2;  // (dim, half of the slots) of head hd
    for (int pc = threadIdx.x; pc < pieces; pc += 256) {
        const int hf = pc & 1, e = pc >> 1, he = hd * a.d + e;
        const int s_lo = max(vt.slot0, hf * 8), s_hi = min(vt.slot0 + vt.n, hf * 8 + 8);  // slots of this piece in the run
        if (s_lo >= s_hi) continue;
        const int col = v_col0 + he;
        const int64_t row_of_slot0 = (int64_t)vt.row0 - vt.slot0;  // row of slot s is row_of_slot0 + s (used for s_lo <= s < s_hi only)
        const float b = a.bias ? (float)a.bias[col] : 0.f;
        f32x8 val;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int sl = hf * 8 + k;
            val[k] = 0.f;
            if (sl >= s_lo && sl < s_hi) {
                const float* src = a.qkv + (row_of_slot0 + sl) * a.ld_qkv + col;
                float v = src[0];
                for (int p = 1; p < a.planes; ++p) v += src[p * a.plane_stride];
                if (a.bias) v += b;
                val[k] = v;
            }
        }
        const bf16x8 o = __builtin_convertvector(val, bf16x8);
        bf16_t* vb = a.v_pool + ((int64_t)vt.page * a.n_kv + hd) * (int64_t)(a.d * kPage) + e * kPage + hf * 8;
        if (s_hi - s_lo == 8) {
            *reinterpret_cast<bf16x8*>(vb) = o;
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (hf * 8 + k >= s_lo && hf * 8 + k < s_hi) vb[k] = o[k];
        }
    }
}

// One workgroup per token row.  q heads and k heads are rotated (rotate-half pairing: element j
// pairs with j + d/2, angle pos * theta^(-2j/d) taken from the table); k and v are rounded to
// bf16 and stored at (page, slot = pos % 16) in the layer's pool:
//   K element (head h, dim e) -> ((page*n_kv + h)*d*16) + (e/8)*128 + slot*8 + e%8
//   V element (head h, dim e) -> ((page*n_kv + h)*d*16) + e*16 + slot
// PLANES >= 1 fixes the number of split-K planes at compile time (their loads are then issued together), PLANES < 0
// takes it from the arguments.
template <int PLANES>
__global__ __launch_bounds__(256) void rope_kv_write_kernel(RopeKvArgs a) {
    const int v_wgs = a.n_vtiles * a.n_kv;  // the first workgroups write the V runs, one (run, head) each
    if ((int)blockIdx.x < v_wgs) {
        write_v_tile(a, a.v_tiles[blockIdx.x / a.n_kv], blockIdx.x % a.n_kv);
        return;
    }
    const int t = blockIdx.x - v_wgs;
    const int d = a.d, half = d / 2, hq = half / 4;  // a thread handles 4 consecutive pairs
    const int pos = a.tok_pos[t];
    const int64_t page = a.tok_page[t];
    const int slot = pos & (kPage - 1);
    const float* row = a.qkv + (int64_t)t * a.ld_qkv;
    const f32x4* cs = reinterpret_cast<const f32x4*>(a.rope_cs + (int64_t)pos * half * 2);
    const int q_quads = a.n_q * hq, k_quads = a.n_kv * hq;
    const int k_col0 = a.n_q * d, v_col0 = k_col0 + a.n_kv * d;
    auto gather = [&](int col) {  // sum of the partial planes (+ bias) of 4 consecutive columns
        f32x4 v = *reinterpret_cast<const f32x4*>(row + col);
        if constexpr (PLANES >= 1) {
            f32x4 part[PLANES];
#pragma unroll
            for (int p = 1; p < PLANES; ++p) part[p] = *reinterpret_cast<const f32x4*>(row + p * a.plane_stride + col);
#pragma unroll
            for (int p = 1; p < PLANES; ++p) v += part[p];
        } else {
            for (int p = 1; p < a.planes; ++p) v += *reinterpret_cast<const f32x4*>(row + p * a.plane_stride + col);
        }
        if (a.bias) v += __builtin_convertvector(*reinterpret_cast<const bf16x4*>(a.bias + col), f32x4);
        return v;
    };
    for (int i = threadIdx.x; i < q_quads + k_quads; i += 256) {
        const bool is_q = i < q_quads;
        const int ii = is_q ? i : i - q_quads;
        const int hd = ii / hq, j = (ii % hq) * 4;
        const int col = (is_q ? 0 : k_col0) + hd * d + j;
        const f32x4 lo = gather(col), hi = gather(col + half);
        const f32x4 c01 = cs[j / 2], c23 = cs[j / 2 + 1];  // (cos, sin) of pairs j, j+1 | j+2, j+3
        const f32x4 co = {c01[0], c01[2], c23[0], c23[2]}, si = {c01[1], c01[3], c23[1], c23[3]};
        f32x4 rlo, rhi;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            rlo[v] = lo[v] * co[v] - hi[v] * si[v];
            rhi[v] = hi[v] * co[v] + lo[v] * si[v];
        }
        const bf16x4 blo = __builtin_convertvector(rlo, bf16x4), bhi = __builtin_convertvector(rhi, bf16x4);
        if (is_q) {
            bf16_t* q = a.q_out + (int64_t)t * a.ld_q + hd * d;
            *reinterpret_cast<bf16x4*>(q + j) = blo;
            *reinterpret_cast<bf16x4*>(q + j + half) = bhi;
        } else {
            bf16_t* kb = a.k_pool + (page * a.n_kv + hd) * (int64_t)(d * kPage);
            const int e0 = j, e1 = j + half;  // multiples of 4: the 4 elements stay inside one group of 8
            *reinterpret_cast<bf16x4*>(kb + (e0 >> 3) * (kPage * 8) + slot * 8 + (e0 & 7)) = blo;
            *reinterpret_cast<bf16x4*>(kb + (e1 >> 3) * (kPage * 8) + slot * 8 + (e1 & 7)) = bhi;
        }
    }
    if (a.tok_own_v && !a.tok_own_v[t]) return;  // wave-uniform: a V run covers this token
    const int v_quads = a.n_kv * d / 4;
    for (int i = threadIdx.x; i < v_quads; i += 256) {
        const int hd = (i * 4) / d, e = (i * 4) % d;
        const bf16x4 v = __builtin_convertvector(gather(v_col0 + i * 4), bf16x4);
        bf16_t* vb = a.v_pool + (page * a.n_kv + hd) * (int64_t)(d * kPage) + e * kPage + slot;
#pragma unroll
        for (int u = 0; u < 4; ++u) vb[u * kPage] = v[u];
    }
}

// The same for a single plane (the many-row case, where this kernel's time matters), with a token's work cut into
// units of four columns -- rotated (lo, hi) quads of the q and k heads first, then v quads -- and unit
// threadIdx.x + 256 * it handled in pass `it`: all loads of all ITERS passes are issued before the first result
// is computed, so a workgroup waits for memory once instead of once per pass.
template <int ITERS>
__global__ __launch_bounds__(256) void rope_kv_write_batched_kernel(RopeKvArgs a) {
    const int v_wgs = a.n_vtiles * a.n_kv;
    if ((int)blockIdx.x < v_wgs) {
        write_v_tile(a, a.v_tiles[blockIdx.x / a.n_kv], blockIdx.x % a.n_kv);
        return;
    }
    const int t = blockIdx.x - v_wgs;
    const int d = a.d, half = d / 2, hq = half / 4;
    const int pos = a.tok_pos[t];
    const int64_t page = a.tok_page[t];
    const int slot = pos & (kPage - 1);
    const float* row = a.qkv + (int64_t)t * a.ld_qkv;
    const f32x4* cs = reinterpret_cast<const f32x4*>(a.rope_cs + (int64_t)pos * half * 2);
    const bool own_v = !a.tok_own_v || a.tok_own_v[t];
    const int q_quads = a.n_q * hq, rope_units = (a.n_q + a.n_kv) * hq, units = rope_units + (own_v ? a.n_kv * d / 4 : 0);
    const int k_col0 = a.n_q * d, v_col0 = k_col0 + a.n_kv * d;
    f32x4 lo[ITERS], hi[ITERS], c01[ITERS], c23[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int i = threadIdx.x + it * 256;
        if (i < rope_units) {
            const int ii = i < q_quads ? i : i - q_quads;
            const int j = (ii % hq) * 4;
            const int col = (i < q_quads ? 0 : k_col0) + (ii / hq) * d + j;
            lo[it] = *reinterpret_cast<const f32x4*>(row + col);
            hi[it] = *reinterpret_cast<const f32x4*>(row + col + half);
            c01[it] = cs[j / 2];
            c23[it] = cs[j / 2 + 1];
            if (a.bias) {
                lo[it] += __builtin_convertvector(*reinterpret_cast<const bf16x4*>(a.bias + col), f32x4);
                hi[it] += __builtin_convertvector(*reinterpret_cast<const bf16x4*>(a.bias + col + half), f32x4);
            }
        } else if (i < units) {
            const int col = v_col0 + (i - rope_units) * 4;
            lo[it] = *reinterpret_cast<const f32x4*>(row + col);
            if (a.bias) lo[it] += __builtin_convertvector(*reinterpret_cast<const bf16x4*>(a.bias + col), f32x4);
        }
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int i = threadIdx.x + it * 256;
        if (i < rope_units) {
            const bool is_q = i < q_quads;
            const int ii = is_q ? i : i - q_quads;
            const int hd = ii / hq, j = (ii % hq) * 4;
            const f32x4 co = {c01[it][0], c01[it][2], c23[it][0], c23[it][2]}, si = {c01[it][1], c01[it][3], c23[it][1], c23[it][3]};
            f32x4 rlo, rhi;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                rlo[v] = lo[it][v] * co[v] - hi[it][v] * si[v];
                rhi[v] = hi[it][v] * co[v] + lo[it][v] * si[v];
            }
            const bf16x4 blo = __builtin_convertvector(rlo, bf16x4), bhi = __builtin_convertvector(rhi, bf16x4);
            if (is_q) {
                bf16_t* q = a.q_out + (int64_t)t * a.ld_q + hd * d;
                *reinterpret_cast<bf16x4*>(q + j) = blo;
                *reinterpret_cast<bf16x4*>(q + j + half) = bhi;
            } else {
                bf16_t* kb = a.k_pool + (page * a.n_kv + hd) * (int64_t)(d * kPage);
                const int e0 = j, e1 = j + half;
                *reinterpret_cast<bf16x4*>(kb + (e0 >> 3) * (kPage * 8) + slot * 8 + (e0 & 7)) = blo;
                *reinterpret_cast<bf16x4*>(kb + (e1 >> 3) * (kPage * 8) + slot * 8 + (e1 & 7)) = bhi;
            }
        } else if (i < units) {
            const int e4 = (i - rope_units) * 4, hd = e4 / d, e = e4 % d;
            const bf16x4 v = __builtin_convertvector(lo[it], bf16x4);
            bf16_t* vb = a.v_pool + (page * a.n_kv + hd) * (int64_t)(d * kPage) + e * kPage + slot;
#pragma unroll
            for (int u = 0; u < 4; ++u) vb[u * kPage] = v[u];
        }
    }
}

}  // namespace

template <bool FROM_BF16>
hipError_t launch_rmsnorm_any(const bf16_t* in, float* x, const float* y, int planes, int64_t plane_stride,
                              const bf16_t* gamma, bf16_t* h, int64_t ldh, int rows, int hidden, float eps,
                              hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    if (hidden % 4 != 0 || hidden > 16 * 1024 || planes < 0 || planes > kMaxPlanes) return hipErrorInvalidValue;
    const int vecs = (int)ceil_div(hidden, 1024);
#define GLLM_RMS_P(V, P) rmsnorm_kernel<FROM_BF16, V, P><<<rows, 256, 0, stream>>>(in, x, y, planes, plane_stride, gamma, h, ldh, hidden, eps)
#define GLLM_RMS(V)                                              \
    do {                                                         \
        if (FROM_BF16 || planes == 0) GLLM_RMS_P(V, 0);          \
        else if (planes == 1) GLLM_RMS_P(V, 1);                  \
        else if (planes == 2) GLLM_RMS_P(V, 2);                  \
        else if (planes == 4) GLLM_RMS_P(V, 4);                  \
        else if (planes == 8) GLLM_RMS_P(V, 8);                  \
        else GLLM_RMS_P(V, -1);                                  \
    } while (0)
    if (vecs <= 1) GLLM_RMS(1);
    else if (vecs <= 2) GLLM_RMS(2);
    else if (vecs <= 4) GLLM_RMS(4);
    else if (vecs <= 5) GLLM_RMS(5);
    else if (vecs <= 8) GLLM_RMS(8);
    else GLLM_RMS(16);
#undef GLLM_RMS
#undef GLLM_RMS_P
    return hipGetLastError();
}

hipError_t launch_rmsnorm_from_bf16(const bf16_t* in, float* x, const bf16_t* gamma, bf16_t* h, int64_t ldh,
                                    int rows, int hidden, float eps, hipStream_t stream) {
    return launch_rmsnorm_any<true>(in, x, nullptr, 0, 0, gamma, h, ldh, rows, hidden, eps, stream);
}

hipError_t launch_add_rmsnorm(float* x, const float* y, int planes, int64_t plane_stride, const bf16_t* gamma,
                              bf16_t* h, int64_t ldh, int rows, int hidden, float eps, hipStream_t stream) {
    return launch_rmsnorm_any<false>(nullptr, x, y, planes, plane_stride, gamma, h, ldh, rows, hidden, eps, stream);
}

hipError_t launch_add_cast_out(const float* x, const float* y, int planes, int64_t plane_stride, bf16_t* out,
                               float* out_f32, int64_t count, hipStream_t stream) {
    if (count <= 0) return hipSuccess;
    int64_t c4 = count / 4;
    cast_out_kernel<<<(unsigned)ceil_div(c4, 256), 256, 0, stream>>>(x, y, planes, plane_stride, out, out_f32, c4);
    return hipGetLastError();
}

hipError_t launch_pack_rows_tiled(const bf16_t* src, int64_t ld_src, int rows, int cols, bf16_t* dst, int64_t k_dst,
                                  int dst_row0, hipStream_t stream) {
    if (cols % 8 || k_dst % kWBlock || cols > k_dst || ld_src < cols || dst_row0 < 0) return hipErrorInvalidValue;
    int64_t n = (int64_t)rows * (cols / 8);
    if (n <= 0) return hipSuccess;
    pack_rows_tiled_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, stream>>>(src, ld_src, rows, cols, dst, k_dst, dst_row0);
    return hipGetLastError();
}

hipError_t launch_pack_gate_up(const bf16_t* gate, const bf16_t* up, int inter, int hidden, bf16_t* dst,
                               int64_t k_dst, hipStream_t stream) {
    if (hidden % 8 || k_dst % kWBlock || hidden > k_dst) return hipErrorInvalidValue;
    int64_t n = (int64_t)inter * (hidden / 8);
    if (n <= 0) return hipSuccess;
    pack_gate_up_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, stream>>>(gate, up, inter, hidden, dst, k_dst);
    return hipGetLastError();
}

hipError_t launch_rope_kv_write(const RopeKvArgs& a, hipStream_t stream) {
    if (a.T <= 0) return hipSuccess;
    if (a.n_vtiles < 0 || (a.n_vtiles > 0 && (!a.v_tiles || !a.tok_own_v))) return hipErrorInvalidValue;
    const int grid = a.T + a.n_vtiles * a.n_kv;
    const int units = ((a.n_q + a.n_kv) * (a.d / 8) + a.n_kv * a.d / 4 + 255) / 256;  // passes of 256 four-column units
    if (a.planes == 1 && units <= 8) {
        switch (units) {
            case 1: rope_kv_write_batched_kernel<1><<<grid, 256, 0, stream>>>(a); break;
            case 2: rope_kv_write_batched_kernel<2><<<grid, 256, 0, stream>>>(a); break;
            case 3: rope_kv_write_batched_kernel<3><<<grid, 256, 0, stream>>>(a); break;
            case 4: rope_kv_write_batched_kernel<4><<<grid, 256, 0, stream>>>(a); break;
            case 5: rope_kv_write_batched_kernel<5><<<grid, 256, 0, stream>>>(a); break;
            case 6: rope_kv_write_batched_kernel<6><<<grid, 256, 0, stream>>>(a); break;
            case 7: rope_kv_write_batched_kernel<7><<<grid, 256, 0, stream>>>(a); break;
            default: rope_kv_write_batched_kernel<8><<<grid, 256, 0, stream>>>(a); break;
        }
        return hipGetLastError();
    }
    switch (a.planes) {
        case 1: rope_kv_write_kernel<1><<<grid, 256, 0, stream>>>(a); break;
        case 2: rope_kv_write_kernel<2><<<grid, 256, 0, stream>>>(a); break;
        case 4: rope_kv_write_kernel<4><<<grid, 256, 0, stream>>>(a); break;
        case 8: rope_kv_write_kernel<8><<<grid, 256, 0, stream>>>(a); break;
        default: rope_kv_write_kernel<-1><<<grid, 256, 0, stream>>>(a); break;
    }
    return hipGetLastError();
}
