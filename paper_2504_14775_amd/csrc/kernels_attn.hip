// Ragged paged attention for decode rows and prefill chunks on the CDNA4 matrix cores.
//
// Both kernels run the same inner step on a block of 32 keys (two pages) and one or more groups
// of 16 "columns" (for a decode row: the query heads that share a KV head; for a prefill chunk:
// 16 consecutive query rows of one head), in transposed form so that nothing has to be moved
// between lanes:
//     S^T[key][col]  = K[key][:] . Q[col][:]          two 16x16x32 MFMA chains (16 of the 32 keys each)
//     O^T[dim][col] += V^T[dim][key] . P^T[key][col]  one 16x16x32 MFMA per 16 dims
// A 16x16x32 MFMA takes, per lane (r = lane % 16, G = lane / 16), 8 consecutive k-values of row r
// (A operand) or column r (B operand), k-slots 8G..8G+7, and returns for column r the rows
// 4G..4G+3.  The 32 keys are dealt to the rows of the two S^T tiles so that the 4 + 4 results a lane holds for
// its column are the 8 consecutive keys 8G..8G+7 of the block (tile t, row i = slot 8((i>>2)&1) + 4t + (i&3) of
// page i>>3) -- exactly the 8 k-slots it must supply as the B operand of the P.V product.  The pool layouts
// make the matching A operands 16-byte pieces:
//   K page [d/8][16 slots][8]: k-step s, tile t reads (group 4s + G, the slot above) of page r>>3;
//   V page [d][16 slots]:      dims 16b..16b+15 of P.V read slots 8(G&1)..+7 of dim 16b + r of page G>>1.
// Softmax is the running-reference form in base 2 (exponent s*log2(e)/sqrt(d) - m, see update_group);
// all reductions follow logical key order, so the result does not depend on which physical pages
// hold the keys.
#include "common.h"

#include <type_traits>
#include <utility>

namespace {

constexpr float kNegBig = -1.0e30f;

// K and V operands of one block of 32 keys (two pages) in the layout score_group expects: a lane owns the 8
// consecutive keys 8G .. 8G+7 of the block.
template <int D>
struct KvFrag {
    u32x4 k[2][D / 32];  // [fragment t][k-step]: operand row r = slot 8 ((r >> 2) & 1) + 4 t + (r & 3) of page r >> 3
    u32x4 v[D / 16];     // [16-dim block]: slots 8 (G & 1) .. + 7 of dim r of page G >> 1
};

// The loads carry the non-temporal hint: a decode row's K and V are read once and never again, and without the hint the
// stream is allocated in the caches on its way (measured: 5.78 -> 6.20 TB/s on 256 rows of 512 .. 4096 keys, 5.94 -> 6.35
// on 512 rows of 1024 .. 8192 keys; a bare streaming read without the hint sustains 5.9 - 6.2).
template <int D>
__device__ __forceinline__ void load_kv(KvFrag<D>& f, const bf16_t* __restrict__ kp, const bf16_t* __restrict__ vp,
                                        int64_t page0, int64_t page1, int n_kv, int kvh, int lane) {
    constexpr int64_t PH = (int64_t)D * kPage;  // elements of one (page, head)
    const int r = lane & 15, G = lane >> 4;
    // K page layout [d/8 groups][16 slots][8]: 16 bytes per (group, slot); V page layout [d][16 slots]
    const bf16_t* kb = kp + (((r >> 3) ? page1 : page0) * n_kv + kvh) * PH + (G * kPage + ((r >> 2) & 1) * 8 + (r & 3)) * 8;
    const bf16_t* vb = vp + (((G >> 1) ? page1 : page0) * n_kv + kvh) * PH + r * kPage + (G & 1) * 8;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < D / 32; ++s) f.k[t][s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + s * 512 + t * 32));
#pragma unroll
    for (int b = 0; b < D / 16; ++b) f.v[b] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + b * 256));
}

// State of NB column groups across the key loop.
template <int D, int NB>
struct AttnState {
    f32x4 o[NB][D / 16];
    float m[NB];
    float l[NB];
};

// Masks the V fragments of keys >= valid_end (slots that hold no data yet may contain any bit pattern,
// also NaN, and 0 * NaN would poison the P.V product).  v[b] holds this lane's 8 keys tb + 8G .. tb + 8G + 7 of dims
// block b, two per register.
template <int D>
__device__ __forceinline__ void mask_unwritten_v(u32x4 (&v)[D / 16], int tb, int valid_end, int lane) {
    const int G = lane >> 4;
    int nv = valid_end - (tb + G * 8);
    nv = nv < 0 ? 0 : (nv > 8 ? 8 : nv);
    uint32_t m[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) m[w] = nv >= 2 * w + 2 ? 0xFFFFFFFFu : (nv == 2 * w + 1 ? 0x0000FFFFu : 0u);
#pragma unroll
    for (int b = 0; b < D / 16; ++b)
#pragma unroll
        for (int w = 0; w < 4; ++w) v[b][w] &= m[w];
}

// One column group against one block of 32 keys starting at key index tb, in two phases so that callers
// can fetch the V fragments only after the K fragments are dead.
// Phase 1: raw scores q.k of this lane's 8 keys (not yet scaled), masked keys set to a huge negative.
// The rows of the two K operands are permuted -- row i of fragment t is key tb + 16 (i >> 3) + 8 ((i >> 2) & 1) +
// 4 t + (i & 3) -- so that the accumulators of lane group G are the 8 consecutive keys tb + 8G .. tb + 8G + 7
// (fragment 0 gives the first four, fragment 1 the last four): exactly the 8 k-values this lane supplies to the
// P.V product, whose V operand is then 8 consecutive slots of one page (16 contiguous bytes).
//   limit     : last key visible to this lane's column (causal / partition limit)
//   need_mask : wave-uniform, false when the whole block is visible to every column of the group
template <int D>
__device__ __forceinline__ void score_group(float (&sc)[8], const u32x4 (&kf)[2][D / 32], const bf16x8 (&qf)[D / 32],
                                            int tb, int limit, bool need_mask, int lane) {
    const int G = lane >> 4;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[0][s]), qf[s], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[1][s]), qf[s], s1, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        sc[v] = s0[v];
        sc[4 + v] = s1[v];
    }
    if (need_mask) {
        const int t0 = tb + G * 8;
#pragma unroll
        for (int v = 0; v < 8; ++v)
            if (t0 + v > limit) sc[v] = kNegBig;
    }
}

// Phase 2, for all NB column groups of a wave at once: softmax update in base 2 and O^T += V^T P^T.
//
// m is the reference exponent of a column (identical in the four lanes that share the column); p =
// 2^(s*c - m) with c = log2(e)/sqrt(d).  Softmax does not care which reference is used as long as nothing
// overflows.  DEFER = true lets the reference lag: it is only moved (to the exact running maximum: two
// cross-lane exchanges per group, then m, l and the accumulators are rescaled) when some lane sees a score
// more than 64 above it -- always in a wave's first block, where the reference is still the huge negative
// start value, and practically never afterwards -- so p stays below 2^64, sums of 2^13 of them stay finite,
// and the common path has no cross-lane traffic and no rescaling at all: a lane-local maximum, one wave vote,
// the exponentials, the MFMAs.  DEFER = false moves the reference whenever a lane's maximum exceeds it (the
// textbook order): the memory-bound decode kernel, with one group per wave, gains nothing from deferring.
constexpr float kRefSlack = 64.0f;

// issue_v() is called before the exponentials (a caller that fetches V from LDS starts its reads there),
// get_v() after them (it returns the fragments, waiting for them if need be).
template <int D, int NB, bool DEFER, typename IssueV, typename GetV>
__device__ __forceinline__ void update_groups(AttnState<D, NB>& st, const float (&sc)[NB][8], float scale_log2,
                                              IssueV&& issue_v, GetV&& get_v) {
    float lm[NB];
    bool low = false;
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        float x = sc[c][0];
#pragma unroll
        for (int v = 1; v < 8; ++v) x = fmaxf(x, sc[c][v]);
        lm[c] = x * scale_log2;
        low |= DEFER ? lm[c] > st.m[c] + kRefSlack : lm[c] > st.m[c];
    }
    if (__any(low)) {  // wave-uniform
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            float bm = fmaxf(lm[c], __shfl_xor(lm[c], 16));
            bm = fmaxf(bm, __shfl_xor(bm, 32));
            const float m_new = fmaxf(st.m[c], bm);
            const float alpha = __builtin_amdgcn_exp2f(st.m[c] - m_new);
            st.l[c] *= alpha;
#pragma unroll
            for (int b = 0; b < D / 16; ++b)
#pragma unroll
                for (int v = 0; v < 4; ++v) st.o[c][b][v] *= alpha;
            st.m[c] = m_new;
        }
    }
    issue_v();
    bf16x8 pb[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        f32x8 p;
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            p[v] = __builtin_amdgcn_exp2f(fmaf(sc[c][v], scale_log2, -st.m[c]));
            psum += p[v];
        }
        st.l[c] += psum;
        pb[c] = __builtin_convertvector(p, bf16x8);
    }
    const u32x4 (&vf)[D / 16] = get_v();
#pragma unroll
    for (int b = 0; b < D / 16; ++b)
#pragma unroll
        for (int c = 0; c < NB; ++c)
            st.o[c][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf[b]), pb[c], st.o[c][b], 0, 0, 0);
}

// One block of 32 keys for NB column groups, K/V fragments in registers.
//   limit[c]   : last key visible to this lane's column in group c
//   valid_end  : keys >= valid_end hold no data yet
template <int D, int NB>
__device__ __forceinline__ void attend_block(AttnState<D, NB>& st, KvFrag<D>& f, const bf16x8 (&qf)[NB][D / 32],
                                             int tb, const int (&limit)[NB], int min_limit, int valid_end,
                                             float scale_log2, int lane) {
    if (tb + 32 > valid_end) mask_unwritten_v<D>(f.v, tb, valid_end, lane);  // wave-uniform
    const bool need_mask = tb + 31 > min_limit;                              // wave-uniform
    float sc[NB][8];
#pragma unroll
    for (int c = 0; c < NB; ++c) score_group<D>(sc[c], f.k, qf[c], tb, limit[c], need_mask, lane);
    update_groups<D, NB, false>(st, sc, scale_log2, []() {}, [&]() -> const u32x4 (&)[D / 16] { return f.v; });
}

// Walks key blocks [blk_begin, blk_end) (units of 32 keys) of one sequence.  Page ids are fetched 64
// at a time, one per lane, and handed out with readlane.  last_page is the last page index of the
// sequence that may be read (page ids past it are never dereferenced).
template <int D, int NB>
__device__ __forceinline__ void attend_range(AttnState<D, NB>& st, const bf16x8 (&qf)[NB][D / 32],
                                             const bf16_t* __restrict__ kp, const bf16_t* __restrict__ vp,
                                             const int32_t* __restrict__ bt, int blk_begin, int blk_end,
                                             int last_page, const int (&limit)[NB], int min_limit, int valid_end,
                                             int n_kv, int kvh, float scale_log2, int lane) {
    if (blk_begin >= blk_end) return;
    int ids_base = blk_begin * 2;  // page index held by lane 0
    int ids = bt[min(ids_base + lane, last_page)];
    auto page_of = [&](int pi) -> int64_t {  // pi wave-uniform, within [ids_base, ids_base + 64)
        return (int64_t)__builtin_amdgcn_readlane(ids, pi - ids_base);
    };
    auto load_block = [&](KvFrag<D>& f, int blk) {
        int p0 = min(blk * 2, last_page), p1 = min(blk * 2 + 1, last_page);
        load_kv<D>(f, kp, vp, page_of(p0), page_of(p1), n_kv, kvh, lane);
    };
    KvFrag<D> fa, fb;
    load_block(fa, blk_begin);
    for (int blk = blk_begin; blk < blk_end; blk += 2) {
        // blocks blk and blk+1 use pages 2blk .. 2blk+3; refill the id window when it runs out
        const bool has_b = blk + 1 < blk_end;
        if (has_b) load_block(fb, blk + 1);
        attend_block<D, NB>(st, fa, qf, blk * 32, limit, min_limit, valid_end, scale_log2, lane);
        if (blk + 2 < blk_end) {
            if ((blk + 2) * 2 + 3 >= ids_base + 64) {
                ids_base = (blk + 2) * 2;
                ids = bt[min(ids_base + lane, last_page)];
            }
            load_block(fa, blk + 2);
        }
        if (has_b) attend_block<D, NB>(st, fb, qf, (blk + 1) * 32, limit, min_limit, valid_end, scale_log2, lane);
    }
}

template <int D, int NB>
__device__ __forceinline__ void init_state(AttnState<D, NB>& st) {
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        st.m[c] = kNegBig;
        st.l[c] = 0.f;
#pragma unroll
        for (int b = 0; b < D / 16; ++b) st.o[c][b] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
}

// ------------------------------------------------------------------------------------------
// Decode: one workgroup of 4 waves per (item, kv head).  The item's key partition is cut into four runs of
// 32-key blocks, one per wave; the waves' partial results are merged through LDS and written as
// one partial (running max, sum, unnormalised output) per query head of the KV head.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 2) void decode_attention_kernel(AttnArgs a, const DecodeItem* __restrict__ items,
                                                                const int32_t* __restrict__ order,
                                                                float* __restrict__ part_o,
                                                                float* __restrict__ part_ml) {
    __shared__ float lds_o[4][16][D + 4];
    __shared__ float lds_m[4][16], lds_l[4][16];
    // the KV heads of one item are neighbouring workgroups: they run at the same time and read
    // neighbouring 4 KiB pieces of the same pages
    const int item_idx = order[blockIdx.x / a.n_kv];
    const int kvh = blockIdx.x % a.n_kv;
    const DecodeItem it = items[item_idx];
    const int g = a.n_q / a.n_kv;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, G = lane >> 4;

    bf16x8 qf[1][D / 32];
    {
        const bf16_t* qrow = a.q + (int64_t)it.row * a.ld_q + (int64_t)(kvh * g + r) * D;
#pragma unroll
        for (int s = 0; s < D / 32; ++s) {
            u32x4 z = {0u, 0u, 0u, 0u};
            if (r < g) z = *reinterpret_cast<const u32x4*>(qrow + (s * 4 + G) * 8);
            qf[0][s] = __builtin_bit_cast(bf16x8, z);
        }
    }
    const int blk0 = it.kv_begin / 32;
    const int nblk = (it.kv_end - it.kv_begin + 31) / 32;
    const int per_wave = (nblk + 3) / 4;
    const int b_begin = blk0 + min(wave * per_wave, nblk);
    const int b_end = blk0 + min((wave + 1) * per_wave, nblk);
    const int limit[1] = {it.kv_end - 1};
    AttnState<D, 1> st;
    init_state<D, 1>(st);
    attend_range<D, 1>(st, qf, a.k_pool, a.v_pool, a.bt_flat + it.bt_off, b_begin, b_end, (it.kv_end - 1) / kPage,
                       limit, it.kv_end - 1, it.kv_end, a.n_kv, kvh, a.scale_log2, lane);
    float l = st.l[0];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (G == 0) {
        lds_m[wave][r] = st.m[0];
        lds_l[wave][r] = l;
    }
#pragma unroll
    for (int b = 0; b < D / 16; ++b)
        *reinterpret_cast<f32x4*>(&lds_o[wave][r][b * 16 + G * 4]) = st.o[0][b];
    __syncthreads();
    // merge: thread -> (head j, 4-dim group)
    for (int idx = threadIdx.x; idx < g * (D / 4); idx += 256) {
        const int j = idx / (D / 4), e = (idx % (D / 4)) * 4;
        float mw[4], ms = kNegBig;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            mw[w] = lds_m[w][j];
            ms = fmaxf(ms, mw[w]);
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float ls = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float sc = __builtin_amdgcn_exp2f(mw[w] - ms);
            const f32x4 ov = *reinterpret_cast<const f32x4*>(&lds_o[w][j][e]);
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] += ov[v] * sc;
            ls += lds_l[w][j] * sc;
        }
        if (it.single) {  // same arithmetic as the merge kernel applies to a row with one partial
            const float inv = 1.0f / ls;
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] *= inv;
            *reinterpret_cast<bf16x4*>(a.out + (int64_t)it.row * a.ld_o + (kvh * g + j) * D + e) =
                __builtin_convertvector(acc, bf16x4);
            continue;
        }
        const int64_t slot = ((int64_t)item_idx * a.n_q + kvh * g + j);
        *reinterpret_cast<f32x4*>(part_o + slot * D + e) = acc;
        if (e == 0) {
            part_ml[slot * 2] = ms;
            part_ml[slot * 2 + 1] = ls;
        }
    }
}

// grid (rows, query heads), D/4 threads: merges the partials of a row in partition order.
template <int D>
__global__ void decode_combine_kernel(AttnArgs a, const DecodeRow* __restrict__ rows, const float* __restrict__ part_o,
                                      const float* __restrict__ part_ml) {
    const DecodeRow rw = rows[blockIdx.x];
    const int hq = blockIdx.y, e = threadIdx.x * 4;
    // the partials are read eight at a time (all loads of a batch are issued before the first use: a row has a
    // handful of partials and the kernel is all latency), and combined in partition order
    constexpr int U = 8;
    const int64_t slot0 = (int64_t)rw.first_item * a.n_q + hq, slot_step = a.n_q;
    float ms = kNegBig;
    for (int i0 = 0; i0 < rw.num_items; i0 += U) {
        float m[U];
#pragma unroll
        for (int u = 0; u < U; ++u) m[u] = i0 + u < rw.num_items ? part_ml[(slot0 + (i0 + u) * slot_step) * 2] : kNegBig;
#pragma unroll
        for (int u = 0; u < U; ++u) ms = fmaxf(ms, m[u]);
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float ls = 0.f;
    for (int i0 = 0; i0 < rw.num_items; i0 += U) {
        float m[U], l[U];
        f32x4 ov[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (i0 + u < rw.num_items) {
                const int64_t slot = slot0 + (i0 + u) * slot_step;
                m[u] = part_ml[slot * 2];
                l[u] = part_ml[slot * 2 + 1];
                ov[u] = *reinterpret_cast<const f32x4*>(part_o + slot * D + e);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (i0 + u < rw.num_items) {
                const float sc = __builtin_amdgcn_exp2f(m[u] - ms);
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[v] += ov[u][v] * sc;
                ls += l[u] * sc;
            }
        }
    }
    const float inv = 1.0f / ls;
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] *= inv;
    *reinterpret_cast<bf16x4*>(a.out + (int64_t)rw.row * a.ld_o + hq * D + e) = __builtin_convertvector(acc, bf16x4);
}

// One 16-byte LDS read at addr + 512*B (dims block B of a V page).  Written as assembly so that the reads can be
// issued early and awaited late: the result is valid only after await_lds().
template <int B>
__device__ __forceinline__ void read_v_operand(u32x4& v, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(B * 512) : "memory");
}
template <int N, int... Bs>
__device__ __forceinline__ void read_v_operands(u32x4 (&v)[N], uint32_t addr, std::integer_sequence<int, Bs...>) {
    (read_v_operand<Bs>(v[Bs], addr), ...);
}
// Waits for all outstanding LDS reads; the registers are passed through the statement so that no use of them
// can be scheduled before it.
template <int N>
__device__ __forceinline__ void await_lds(u32x4 (&v)[N]) {
    static_assert(N % 4 == 0, "fragments are awaited four at a time");
#pragma unroll
    for (int b = 0; b < N; b += 4)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[b]), "+v"(v[b + 1]), "+v"(v[b + 2]), "+v"(v[b + 3])::"memory");
}

// ------------------------------------------------------------------------------------------
// Prefill: one workgroup of 4 waves per (item, group of HW query heads of one KV head).  An item is up
// to 128/HW consecutive query rows of a chunk, so the workgroup owns 8 column groups of 16 (2 per wave)
// that all share the same K/V: every 32-key block is brought into LDS once (global_load_lds into a ring
// of 3 stages, two blocks in flight while one is processed: a block is only ~0.5 us of work, far less
// than the memory latency) and read by all 4 waves.
// A lane owns 8 consecutive keys of the block (the K operand rows are permuted accordingly, see score_group),
// so a V operand is one 16-byte LDS read of 8 slots of one page; LDS holds the pages as the pool does, except
// that the second K page is shifted by four slots (see issue_block).
// Column group cb = 2*wave + c covers head (cb % HW) and query rows 16*(cb / HW) .. +15 of the item.
// ------------------------------------------------------------------------------------------
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int D, int HW>
__global__ __launch_bounds__(256, 3) void prefill_attention_kernel(AttnArgs a, const PrefillItem* __restrict__ items) {
    constexpr int NB = 2;
    constexpr int PAGE_BYTES = D * kPage * 2;  // one (page, head) of K or of V
    constexpr int NS = 3;                      // LDS stages
    constexpr int IPB = PAGE_BYTES / 1024;     // load instructions per wave and block
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NS][4][PAGE_BYTES];  // [stage][K0,K1,V0,V1]
    const int groups = a.n_q / HW;
    const PrefillItem it = items[blockIdx.x / groups];
    const int head0 = (blockIdx.x % groups) * HW;
    const int kvh = head0 / (a.n_q / a.n_kv);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, G = lane >> 4;

    bf16x8 qf[NB][D / 32];
    int limit[NB], wave_min = 0x7FFFFFFF, wave_max = -1;
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        const int cb = wave * NB + c, qb = cb / HW;
        const int qi = min(qb * 16 + r, it.n_rows - 1);  // rows past the item repeat its last row (never stored)
        limit[c] = it.pos0 + qi;
        wave_min = min(wave_min, it.pos0 + min(qb * 16, it.n_rows - 1));
        wave_max = max(wave_max, it.pos0 + min(qb * 16 + 15, it.n_rows - 1));
        const bf16_t* qrow = a.q + (int64_t)(it.row0 + qi) * a.ld_q + (int64_t)(head0 + cb % HW) * D;
#pragma unroll
        for (int s = 0; s < D / 32; ++s)
            qf[c][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + (s * 4 + G) * 8));
    }
    const int last_pos = it.pos0 + it.n_rows - 1;
    const int nblk = last_pos / 32 + 1, last_page = last_pos / kPage;
    const int32_t* bt = a.bt_flat + it.bt_off;
    // wave w brings in piece w of a block: K page 0, K page 1, V page 0, V page 1 (4 x 1 KiB per page at d=128)
    const bf16_t* pool = (wave < 2) ? a.k_pool : a.v_pool;
    auto page_id = [&](int blk) -> int { return bt[min(blk * 2 + (wave & 1), last_page)]; };
    auto issue_block = [&](int64_t page, int stage) {
        // K page 0 and the V pages are copied as they are, K page 1 with slot s at the place of slot s ^ 4.  A 16-byte
        // LDS read is served 16 lanes at a time -- measured: lanes 0-7 together with lanes 24-31, 8-15 with 16-23,
        // and likewise in the upper half of the wave -- and is free of bank conflicts when those 16 lanes hit 16
        // different 16-byte columns of the 256-byte bank line.  The K operand rows of such a group are slots
        // {0-3, 8-11} (or {4-7, 12-15}) of page 0 and of page 1: the shift by four slots separates the two pages.
        // The V operand of such a group is one half (16 bytes) of dims 0-7 and the other half of dims 8-15 of a
        // 16-dim block: 16 different columns as stored.  A lane picks the source piece for its LDS position.
        const int src_lane = wave == 1 ? lane ^ 4 : lane;
        const char* src = reinterpret_cast<const char*>(pool + (page * a.n_kv + kvh) * (int64_t)(D * kPage)) + src_lane * 16;
#pragma unroll
        for (int i = 0; i < IPB; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(src + i * 1024), (lptr_t)(&lds[stage][wave][i * 1024]), 16, 0, 0);
    };

    AttnState<D, NB> st;
    init_state<D, NB>(st);
    auto block_step = [&](int stage, int tb, auto masked) {
        constexpr bool MASKED = decltype(masked)::value;
        float sc[NB][8];
        {
            // fragment t, row r of the operand = slot 8 ((r >> 2) & 1) + 4 t + (r & 3) of page r >> 3 (see score_group)
            u32x4 kf[2][D / 32];
            const int kpage = r >> 3, kslot = ((r >> 2) & 1) * 8 + (r & 3);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int s = 0; s < D / 32; ++s)
                    kf[t][s] = *reinterpret_cast<const u32x4*>(
                        &lds[stage][kpage][((s * 4 + G) * 16 + ((kslot + 4 * t) ^ (4 * kpage))) * 16]);
#pragma unroll
            for (int c = 0; c < NB; ++c) score_group<D>(sc[c], kf, qf[c], tb, limit[c], MASKED, lane);
        }
        // V^T operands: dims block b needs this lane's 8 consecutive keys of one dim: the 16 bytes of slots 0-7 or
        // 8-15 of page G >> 1.  The reads are issued before the exponentials and awaited after them.
        u32x4 vf[D / 16];
        update_groups<D, NB, true>(
            st, sc, a.scale_log2,
            [&]() {
                const uint32_t addr = (uint32_t)(uintptr_t)(&lds[stage][2 + (G >> 1)][r * 32 + (G & 1) * 16]);
                read_v_operands(vf, addr, std::make_integer_sequence<int, D / 16>{});
            },
            [&]() -> const u32x4 (&)[D / 16] {
                await_lds(vf);
                if (MASKED) mask_unwritten_v<D>(vf, tb, last_pos + 1, lane);
                return vf;
            });
    };
    // every wave always issues its piece (indices past the end re-read the last page into a stage nobody
    // reads), so the count of outstanding loads is the same in every iteration
#pragma unroll
    for (int i = 0; i < NS - 1; ++i) issue_block(page_id(i), i);
    int pid_next = page_id(NS - 1);  // page of block blk + NS - 1, fetched one iteration ahead
    auto ring_advance = [&](int blk) {
        // blocks blk+1 .. blk+NS-2 may still be in flight
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * IPB) : "memory");
        __syncthreads();  // block blk has landed; nobody reads stage (blk-1) % NS any more
        issue_block(pid_next, (blk + NS - 1) % NS);
        pid_next = page_id(blk + NS);
    };
    // Two loops with one barrier per block each (every wave passes nblk barriers in total): first the
    // blocks wholly visible to every row of this wave -- no masks at all, the common case -- then the
    // blocks at the causal edge / the end of the written keys (masked) and the wholly invisible ones (skipped).
    const int n_full = min((wave_min + 1) / 32, nblk);
    for (int blk = 0; blk < n_full; ++blk) {
        ring_advance(blk);
        block_step(blk % NS, blk * 32, std::false_type{});
    }
    for (int blk = n_full; blk < nblk; ++blk) {
        ring_advance(blk);
        if (blk * 32 <= wave_max) block_step(blk % NS, blk * 32, std::true_type{});
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no LDS fill may outlive the workgroup
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        float l = st.l[c];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const float inv = 1.0f / l;
        const int cb = wave * NB + c;
        const int qi = (cb / HW) * 16 + r;
        if (qi < it.n_rows) {
            bf16_t* orow = a.out + (int64_t)(it.row0 + qi) * a.ld_o + (int64_t)(head0 + cb % HW) * D;
#pragma unroll
            for (int b = 0; b < D / 16; ++b) {
                f32x4 o = st.o[c][b];
#pragma unroll
                for (int v = 0; v < 4; ++v) o[v] *= inv;
                *reinterpret_cast<bf16x4*>(orow + b * 16 + G * 4) = __builtin_convertvector(o, bf16x4);
            }
        }
    }
}

}  // namespace

hipError_t launch_decode_attention(const AttnArgs& a, const DecodeItem* items, const int32_t* order, int num_items,
                                   float* part_o, float* part_ml, hipStream_t stream) {
    if (num_items <= 0) return hipSuccess;
    dim3 grid(num_items * a.n_kv);
    if (a.d == 128) decode_attention_kernel<128><<<grid, 256, 0, stream>>>(a, items, order, part_o, part_ml);
    else if (a.d == 64) decode_attention_kernel<64><<<grid, 256, 0, stream>>>(a, items, order, part_o, part_ml);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_decode_combine(const AttnArgs& a, const DecodeRow* rows, int num_rows, const float* part_o,
                                 const float* part_ml, hipStream_t stream) {
    if (num_rows <= 0) return hipSuccess;
    dim3 grid(num_rows, a.n_q);
    if (a.d == 128) decode_combine_kernel<128><<<grid, 32, 0, stream>>>(a, rows, part_o, part_ml);
    else if (a.d == 64) decode_combine_kernel<64><<<grid, 16, 0, stream>>>(a, rows, part_o, part_ml);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

int prefill_heads_per_workgroup(int n_q, int n_kv) {
    const int g = n_q / n_kv;
    return (g == 1 || g == 2 || g == 4 || g == 8) ? g : 1;
}

int prefill_item_rows(int n_q, int n_kv) { return 128 / prefill_heads_per_workgroup(n_q, n_kv); }

hipError_t launch_prefill_attention(const AttnArgs& a, const PrefillItem* items, int num_items, hipStream_t stream) {
    if (num_items <= 0) return hipSuccess;
    const int hw = prefill_heads_per_workgroup(a.n_q, a.n_kv);
    const dim3 grid(num_items * (a.n_q / hw));
#define GLLM_PREFILL(D_, HW_) prefill_attention_kernel<D_, HW_><<<grid, 256, 0, stream>>>(a, items)
    if (a.d == 128) {
        if (hw == 8) GLLM_PREFILL(128, 8); else if (hw == 4) GLLM_PREFILL(128, 4);
        else if (hw == 2) GLLM_PREFILL(128, 2); else GLLM_PREFILL(128, 1);
    } else if (a.d == 64) {
        if (hw == 8) GLLM_PREFILL(64, 8); else if (hw == 4) GLLM_PREFILL(64, 4);
        else if (hw == 2) GLLM_PREFILL(64, 2); else GLLM_PREFILL(64, 1);
    } else {
        return hipErrorInvalidValue;
    }
#undef GLLM_PREFILL
    return hipGetLastError();
}
