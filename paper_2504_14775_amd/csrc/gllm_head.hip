// First / last pipeline-stage extras (arxiv 2504.14775, section 2.1): embedding layer, projection of the final
// hidden states to logits, sampling strategy.  Contract of every entry point: include/gllm_head.h.
#include "../../include/gllm_head.h"
#include "common.h"

#include <climits>
#include <mutex>
#include <string>

namespace {

// ---- embedding: one workgroup per token row, 16-byte pieces -----------------------------------------------
__global__ __launch_bounds__(256) void embedding_kernel(const int32_t* __restrict__ ids, const bf16_t* __restrict__ table,
                                                        bf16_t* __restrict__ out, int hidden, int vocab, int64_t ld_out) {
    const int t = blockIdx.x;
    const int id = ids[t];
    const bool known = id >= 0 && id < vocab;
    const u32x4* src = reinterpret_cast<const u32x4*>(table + (int64_t)(known ? id : 0) * hidden);
    u32x4* dst = reinterpret_cast<u32x4*>(out + (int64_t)t * ld_out);
    if (known) {
        for (int i = threadIdx.x; i < hidden / 8; i += 256) dst[i] = src[i];
    } else {
        for (int i = threadIdx.x; i < hidden / 8; i += 256) dst[i] = u32x4{0u, 0u, 0u, 0u};
    }
}

// ---- final norm of selected rows: h[i] = bf16(x[rows[i]] * rsqrt(mean x^2 + eps) * gain) --------------------
__global__ __launch_bounds__(256) void gather_rmsnorm_kernel(const float* __restrict__ x, int num_x_rows,
                                                             const int32_t* __restrict__ rows,
                                                             const bf16_t* __restrict__ gain, bf16_t* __restrict__ h,
                                                             int hidden, float eps) {
    __shared__ float part[4];
    const int r = min(max(rows[blockIdx.x], 0), num_x_rows - 1);
    const f32x4* src = reinterpret_cast<const f32x4*>(x + (int64_t)r * hidden);
    float ss = 0.f;
    for (int i = threadIdx.x; i < hidden / 4; i += 256) {
        const f32x4 v = src[i];
        ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float rstd = rsqrtf((part[0] + part[1] + part[2] + part[3]) / (float)hidden + eps);
    bf16_t* dst = h + (int64_t)blockIdx.x * hidden;
    for (int i = threadIdx.x; i < hidden / 4; i += 256) {
        const f32x4 v = src[i];
        const f32x4 g = __builtin_convertvector(*reinterpret_cast<const bf16x4*>(gain + i * 4), f32x4);
        f32x4 y;
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = v[e] * rstd * g[e];
        *reinterpret_cast<bf16x4*>(dst + i * 4) = __builtin_convertvector(y, bf16x4);
    }
}

// rows of w [vocab][hidden] -> the GEMM's tiled weight layout with vocab_pad rows, zero rows past vocab
__global__ __launch_bounds__(256) void pad_rows_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ out, int vocab,
                                                       int hidden) {
    const int v = blockIdx.x;
    const u32x4* src = reinterpret_cast<const u32x4*>(w + (int64_t)v * hidden);
    for (int i = threadIdx.x; i < hidden / 8; i += 256)
        *reinterpret_cast<u32x4*>(out + w_tiled_index(v, i * 8, hidden)) = v < vocab ? src[i] : u32x4{0u, 0u, 0u, 0u};
}

// ---- sampling: one workgroup per row ----------------------------------------------------------------------
// The row of logits (0.5 MB at a 128k vocabulary) does not fit on chip, so the cost is the number of passes over
// it.  With top-k: pass 1 takes the maximum and counts the top byte of the logits' keys, pass 2 counts the second
// byte inside the bin of the k-th largest, pass 3 gathers the tokens at or above that 16-bit prefix into a list
// in LDS, on which the k-th largest is selected (rows whose candidates do not fit the list fall back to one pass
// per key byte).  Then either
//   * at most kCompact tokens survive top-k (the usual top_k = 20..100): nucleus and draw work on that short
//     list, or
//   * the nucleus threshold is searched over the whole row, 15 candidate thresholds per pass (8 passes), and the
//     draw takes one more.
constexpr int kSampleThreads = 1024;
constexpr int kSampleWaves = kSampleThreads / 64;
constexpr int kCompact = 1024;
constexpr int kList = 4096;  // top-k candidates held in LDS while the k-th largest is selected among them
// the short-list path gives every thread one list entry (sort, masses) and keeps the list in the reduction arrays;
// the histogram is cleared by the first 256 threads; block_sums keeps up to 15 values per wave in those arrays
static_assert(kCompact == kSampleThreads, "the short list has one entry per thread");
static_assert(kSampleThreads >= 256 && 15 * kSampleWaves <= kSampleThreads, "reduction arrays too small");

// order-preserving map from float to unsigned: a < b  <=>  key(a) < key(b) (for non-NaN values)
__device__ __forceinline__ uint32_t float_key(float f) {
    const uint32_t b = __float_as_uint(f);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

// Calls f(index, logit) for the elements of a row that this thread owns, in increasing index order: groups of four
// consecutive logits (16-byte loads, two in flight) when the row starts on a 16-byte boundary, single ones otherwise.
template <class F>
__device__ __forceinline__ void for_row(const float* __restrict__ lg, int vocab, F&& f) {
    const int tid = threadIdx.x;
    if ((reinterpret_cast<uintptr_t>(lg) & 15) == 0) {
        const int groups = vocab >> 2;
        int g = tid;
        for (; g + kSampleThreads < groups; g += 2 * kSampleThreads) {
            const f32x4 a = *reinterpret_cast<const f32x4*>(lg + 4 * g);
            const f32x4 b = *reinterpret_cast<const f32x4*>(lg + 4 * (g + kSampleThreads));
#pragma unroll
            for (int e = 0; e < 4; ++e) f(4 * g + e, a[e]);
#pragma unroll
            for (int e = 0; e < 4; ++e) f(4 * (g + kSampleThreads) + e, b[e]);
        }
        if (g < groups) {
            const f32x4 a = *reinterpret_cast<const f32x4*>(lg + 4 * g);
#pragma unroll
            for (int e = 0; e < 4; ++e) f(4 * g + e, a[e]);
        }
        const int t = 4 * groups + tid;
        if (t < vocab) f(t, lg[t]);
    } else {
        for (int i = tid; i < vocab; i += kSampleThreads) f(i, lg[i]);
    }
}

// hist[bin] += 1 for every lane with `on`.  Lanes of a wave that hit the same bin are counted together (the top
// byte of the keys takes two or three values in a whole row, and same-address LDS atomics run one after the
// other); after three such rounds the rest adds singly (many different bins: those run in parallel).
__device__ __forceinline__ void hist_add(unsigned* hist, bool on, uint32_t bin) {
    const int lane = threadIdx.x & 63;
    uint64_t todo = __ballot(on);
    for (int round = 0; round < 3 && todo; ++round) {
        const int leader = __ffsll((long long)todo) - 1;
        const uint32_t b = (uint32_t)__shfl((int)bin, leader);
        const uint64_t same = __ballot(on && bin == b) & todo;
        if (lane == leader) atomicAdd(&hist[b], (unsigned)__popcll(same));
        todo &= ~same;
    }
    if ((todo >> lane) & 1) atomicAdd(&hist[bin], 1u);
}

// Sum over the workgroup with a fixed association (lanes by butterfly, then the 16 wave sums in order), so that a
// row always gives the same token.  `scratch` holds kSampleWaves floats per value.
template <int N>
__device__ __forceinline__ void block_sums(float (&v)[N], float* scratch) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < N; ++j) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v[j] += __shfl_xor(v[j], o);
        if ((tid & 63) == 0) scratch[j * kSampleWaves + (tid >> 6)] = v[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < N; ++j) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kSampleWaves; ++w) s += scratch[j * kSampleWaves + w];
        v[j] = s;
    }
    __syncthreads();
}

__global__ __launch_bounds__(kSampleThreads) void sample_kernel(const float* __restrict__ logits, int64_t ld, int vocab,
                                                                const float* __restrict__ temperature,
                                                                const int32_t* __restrict__ top_k,
                                                                const float* __restrict__ top_p,
                                                                const float* __restrict__ uniform,
                                                                int32_t* __restrict__ out) {
    __shared__ float fs[kSampleThreads];   // reductions; later the probabilities of the compact list
    __shared__ int is[kSampleThreads];     // reductions; later the token ids of the compact list
    __shared__ unsigned hist[256];
    __shared__ uint32_t list_key[kList];   // key(z) and token id of the top-k candidates
    __shared__ int list_id[kList];
    __shared__ uint32_t sh_key;
    __shared__ int sh_int;
    const int tid = threadIdx.x, row = blockIdx.x;
    const float* lg = logits + (int64_t)row * ld;

    const float temp = temperature[row];
    const int k = top_k[row];
    const bool select = temp > 0.f && k > 0 && k < vocab;  // top-k is on: the first pass also counts top bytes

    // pass 1: the largest logit and its lowest index (greedy; also the softmax reference); with top-k, the
    // histogram of the top byte of the logits' own keys (dividing by the temperature keeps their order)
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    float best = -INFINITY;
    int best_i = INT_MAX;
    for_row(lg, vocab, [&](int i, float v) {
        if (v > best) {
            best = v;
            best_i = i;
        }
        if (select) hist_add(hist, true, float_key(v) >> 24);
    });
    fs[tid] = best;
    is[tid] = best_i;
    __syncthreads();
    for (int s = kSampleThreads / 2; s > 0; s >>= 1) {
        if (tid < s) {
            const float ov = fs[tid + s];
            const int oi = is[tid + s];
            if (ov > fs[tid] || (ov == fs[tid] && oi < is[tid])) {
                fs[tid] = ov;
                is[tid] = oi;
            }
        }
        __syncthreads();
    }
    best = fs[0];
    best_i = is[0] == INT_MAX ? 0 : is[0];
    __syncthreads();
    if (!(temp > 0.f)) {
        if (tid == 0) out[row] = best_i;
        return;
    }
    const float zmax = best / temp;
    const float p = top_p[row];
    const float u = uniform[row];

    // The bin that holds the want-th largest entry of the 256-bin histogram goes to sh_key (bin 0 when there are
    // fewer entries than that), the number of entries above that bin to sh_int, the bin's own count to hist[0].
    // Wave 0 does it: lane l owns bins 4l .. 4l+3, a shuffle scan gives the count above each lane's bins.
    auto pick_bin = [&](int want) {
        if (tid < 64) {
            int c[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) c[j] = (int)hist[4 * tid + j];
            const int mine = c[0] + c[1] + c[2] + c[3];
            int incl = mine;  // entries in this lane's bins and all higher ones
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int other = __shfl_down(incl, o);
                if (tid + o < 64) incl += other;
            }
            int above = incl - mine, found = -1, found_above = 0;
#pragma unroll
            for (int j = 3; j >= 0; --j) {
                if (found < 0 && above + c[j] >= want && 4 * tid + j > 0) {
                    found = 4 * tid + j;
                    found_above = above;
                }
                above += c[j];
            }
            // the highest bin that qualifies wins; lane 0 reports bin 0 when none does
            const uint64_t have = __ballot(found >= 0);
            const int winner = have ? 63 - __clzll((long long)have) : 0;
            if (tid == winner) {
                const int bin = have ? found : 0;
                sh_key = (uint32_t)bin;
                sh_int = have ? found_above : incl - c[0];
                hist[0] = hist[bin];
            }
        }
        __syncthreads();
    };

    // top-k: tokens with key(z) >= floor_key are kept, z = logit / temperature (all of them when top-k is off)
    uint32_t floor_key = 0;
    int kept = vocab;
    bool listed = false;  // is[0 .. sh_int) already holds the ids of the kept tokens
    if (select) {
        // Two more bytes would cost two more passes over the row.  Instead: one pass for the second byte, then
        // every token whose logit key is at or above the 16-bit prefix of the k-th largest goes into a short
        // list in LDS (with its exact key(z)), and the k-th largest z is selected on that list.  The list is taken
        // by z, not by logit -- z >= (smallest logit of the prefix) / temperature -- so tokens whose z ties with a
        // listed one are listed too, whatever their logit.
        pick_bin(k);
        const uint32_t b3 = sh_key;
        const int above3 = sh_int;
        __syncthreads();
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for_row(lg, vocab, [&](int, float v) {
            const uint32_t key = float_key(v);
            hist_add(hist, (key >> 24) == b3, (key >> 16) & 255u);
        });
        __syncthreads();
        pick_bin(k - above3);
        const uint32_t prefix16 = (b3 << 8) | sh_key;
        const int candidates = above3 + sh_int + (int)hist[0];
        __syncthreads();
        bool done = false;
        if (candidates <= kList) {
            const uint32_t edge_key = prefix16 << 16;  // smallest key with that prefix; back to the float it encodes
            const float edge = __uint_as_float((edge_key & 0x80000000u) ? edge_key ^ 0x80000000u : ~edge_key);
            const uint32_t edge_z = float_key(edge / temp);
            if (tid == 0) sh_int = 0;
            __syncthreads();
            for_row(lg, vocab, [&](int i, float v) {
                const uint32_t zk = float_key(v / temp);
                if (zk >= edge_z) {
                    const int slot = atomicAdd(&sh_int, 1);
                    if (slot < kList) {
                        list_key[slot] = zk;
                        list_id[slot] = i;
                    }
                }
            });
            __syncthreads();
            const int n_list = sh_int;
            __syncthreads();
            if (n_list <= kList) {  // (ties in z can add entries beyond the count taken on logits)
                // radix select of the k-th largest key(z) on the list, most significant byte first
                uint32_t prefix = 0;
                int want = k, above_total = 0;
                for (int byte = 3; byte >= 0; --byte) {
                    if (tid < 256) hist[tid] = 0;
                    __syncthreads();
                    const int shift = byte * 8;
                    const uint32_t high_mask = byte == 3 ? 0u : 0xFFFFFFFFu << (shift + 8);
                    for (int j = tid; j < n_list; j += kSampleThreads) {
                        const uint32_t key = list_key[j];
                        if ((key & high_mask) == (prefix & high_mask)) atomicAdd(&hist[(key >> shift) & 255u], 1u);
                    }
                    __syncthreads();
                    pick_bin(want);
                    prefix |= sh_key << shift;
                    want -= sh_int;
                    above_total += sh_int;
                    if (byte == 0) kept = above_total + (int)hist[0];
                    __syncthreads();
                }
                floor_key = prefix;
                done = true;
                if (kept <= kCompact) {
                    if (tid == 0) sh_int = 0;
                    __syncthreads();
                    for (int j = tid; j < n_list; j += kSampleThreads)
                        if (list_key[j] >= floor_key) is[atomicAdd(&sh_int, 1)] = list_id[j];
                    __syncthreads();
                    listed = true;
                }
            }
        }
        if (!done) {
            // many near-equal logits around the k-th largest: radix select over the four bytes of key(z) on the
            // whole row, one pass per byte
            uint32_t prefix = 0;
            int want = k, above_total = 0;
            for (int byte = 3; byte >= 0; --byte) {
                if (tid < 256) hist[tid] = 0;
                __syncthreads();
                const int shift = byte * 8;
                const uint32_t high_mask = byte == 3 ? 0u : 0xFFFFFFFFu << (shift + 8);
                for_row(lg, vocab, [&](int, float v) {
                    const uint32_t key = float_key(v / temp);
                    hist_add(hist, (key & high_mask) == (prefix & high_mask), (key >> shift) & 255u);
                });
                __syncthreads();
                pick_bin(want);
                prefix |= sh_key << shift;
                want -= sh_int;
                above_total += sh_int;
                if (byte == 0) kept = above_total + (int)hist[0];
                __syncthreads();
            }
            floor_key = prefix;
        }
    }

    if (kept <= kCompact) {
        // ---- short list: gather the ids, order by id, nucleus and draw on the list ----
        if (!listed) {
            if (tid == 0) sh_int = 0;
            __syncthreads();
            for_row(lg, vocab, [&](int i, float v) {
                if (float_key(v / temp) >= floor_key) {
                    const int slot = atomicAdd(&sh_int, 1);
                    is[slot] = i;
                }
            });
            __syncthreads();
        }
        const int n = sh_int;
        // bitonic sort of the ids (padding sorts last): the list is in index order whatever order the atomics took
        if (tid >= n) is[tid] = INT_MAX;
        __syncthreads();
        for (int size = 2; size <= kCompact; size <<= 1)
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                const int partner = tid ^ stride;
                if (partner > tid) {
                    const int a = is[tid], b = is[partner];
                    const bool up = (tid & size) == 0;
                    if ((a > b) == up) {
                        is[tid] = b;
                        is[partner] = a;
                    }
                }
                __syncthreads();
            }
        float z = 0.f, e = 0.f;
        if (tid < n) {
            z = lg[is[tid]] / temp;
            e = __expf(z - zmax);
        }
        const uint32_t my_key = tid < n ? float_key(z) : 0u;
        float tot[1] = {e};
        block_sums(tot, fs);
        float total = tot[0];
        if (p < 1.f) {
            // the largest key t with mass(key >= t) >= p * total: bisection, the list stays in registers
            const float need = p * total;
            uint32_t lo = floor_key, hi = float_key(zmax);
            while (lo < hi) {
                const uint32_t mid = lo + (hi - lo + 1) / 2;
                float m[1] = {(tid < n && my_key >= mid) ? e : 0.f};
                block_sums(m, fs);
                if (m[0] >= need) lo = mid;
                else hi = mid - 1;
            }
            if (my_key < lo) e = 0.f;
            float t2[1] = {e};
            block_sums(t2, fs);
            total = t2[0];
        }
        fs[tid] = e;
        __syncthreads();
        if (tid == 0) {  // the draw: first token in index order whose running sum exceeds u * total
            const float target = u * total;
            float running = 0.f;
            int pick = -1, last = -1;
            for (int j = 0; j < n; ++j) {
                if (fs[j] > 0.f) {
                    last = is[j];
                    running += fs[j];
                    if (running > target) {
                        pick = last;
                        break;
                    }
                }
            }
            out[row] = pick >= 0 ? pick : (last >= 0 ? last : best_i);
        }
        return;
    }

    // ---- long list: work on the whole row ----
    auto masses = [&](const uint32_t (&from)[15], float (&m)[15]) {  // m[j] = sum of exp(z - zmax) over key >= from[j]
#pragma unroll
        for (int j = 0; j < 15; ++j) m[j] = 0.f;
        for_row(lg, vocab, [&](int, float v) {
            const float z = v / temp;
            const uint32_t key = float_key(z);
            const float e = __expf(z - zmax);
#pragma unroll
            for (int j = 0; j < 15; ++j) m[j] += key >= from[j] ? e : 0.f;
        });
        block_sums(m, fs);
    };
    uint32_t probe[15];
    float m[15];
#pragma unroll
    for (int j = 0; j < 15; ++j) probe[j] = floor_key;
    masses(probe, m);
    float total = m[0];
    if (p < 1.f) {
        // the largest key t with mass(key >= t) >= p * total; the interval [lo, hi] shrinks 16-fold per pass
        const float need = p * total;
        uint32_t lo = floor_key, hi = float_key(zmax);
        while (lo < hi) {
            const uint64_t span = (uint64_t)hi - lo;  // candidates lo < c_1 <= ... <= c_15 <= hi
#pragma unroll
            for (int j = 0; j < 15; ++j) probe[j] = lo + (uint32_t)((span * (j + 1) + 15) / 16);
            masses(probe, m);
            uint32_t new_lo = lo, new_hi = hi;
            bool closed = false;
#pragma unroll
            for (int j = 0; j < 15; ++j) {
                if (closed) continue;
                if (m[j] >= need) new_lo = probe[j];
                else {
                    new_hi = probe[j] - 1;
                    closed = true;
                }
            }
            lo = new_lo;
            hi = new_hi;
        }
        floor_key = lo;
#pragma unroll
        for (int j = 0; j < 15; ++j) probe[j] = floor_key;
        masses(probe, m);
        total = m[0];
    }

    // the draw in index order: every thread owns a run of consecutive tokens
    const float target = u * total;
    const int run = (vocab + kSampleThreads - 1) / kSampleThreads;
    const int i0 = min(tid * run, vocab), i1 = min(i0 + run, vocab);
    float own = 0.f;
    int last_kept = -1;
    for (int i = i0; i < i1; ++i) {
        const float z = lg[i] / temp;
        if (float_key(z) >= floor_key) {
            own += __expf(z - zmax);
            last_kept = i;
        }
    }
    fs[tid] = own;
    is[tid] = last_kept;
    __syncthreads();
    if (tid == 0) {  // serial prefix over 1024 partial sums: fixed order, negligible next to the passes above
        float before = 0.f;
        int winner = -1, last = -1;
        for (int t = 0; t < kSampleThreads; ++t) {
            const float v = fs[t];
            if (winner < 0 && before + v > target) {
                winner = t;
                sh_key = __float_as_uint(before);
            }
            before += v;
            if (is[t] >= 0) last = is[t];
        }
        sh_int = winner;
        if (winner < 0) out[row] = last < 0 ? best_i : last;  // u * total rounded up to the total: the last kept token
    }
    __syncthreads();
    if (tid == sh_int) {
        float running = __uint_as_float(sh_key);
        int pick = last_kept;
        for (int i = i0; i < i1; ++i) {
            const float z = lg[i] / temp;
            if (float_key(z) >= floor_key) {
                running += __expf(z - zmax);
                if (running > target) {
                    pick = i;
                    break;
                }
            }
        }
        out[row] = pick;
    }
}

}  // namespace

struct gllm_head {
    gllm_head_config cfg;
    int32_t vocab_pad = 0;
    bf16_t* w = nullptr;      // [vocab_pad][hidden]
    bf16_t* gain = nullptr;   // [hidden]
    bf16_t* h = nullptr;      // workspace: [round_up(max_rows, 256)][hidden]
    bool loaded = false;
    std::string err;
};

// Scratch of gllm_head_logits_static: the normalised bf16 rows between the two kernels of the projection, for callers
// that can neither allocate nor bind a workspace.  One array per GPU, held until the process ends; its device address
// is looked up once per device (host code must never use the array's name as an address).
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on first use there).
hipError_t static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

gllm_status fail(gllm_head* s, gllm_status st, const std::string& msg) {
    if (s) s->err = msg;
    return st;
}
}  // namespace

extern "C" {

gllm_status gllm_op_embedding(const int32_t* ids, const void* table, void* out, int32_t num_tokens, int32_t hidden,
                              int32_t vocab, int64_t ld_out, void* stream) {
    if (!ids || !table || !out || num_tokens < 0 || hidden < 8 || hidden % 8 != 0 || vocab < 1 || ld_out < hidden ||
        ld_out % 8 != 0)
        return GLLM_E_INVALID;
    if (num_tokens == 0) return GLLM_OK;
    embedding_kernel<<<num_tokens, 256, 0, (hipStream_t)stream>>>(ids, (const bf16_t*)table, (bf16_t*)out, hidden, vocab, ld_out);
    return hipGetLastError() == hipSuccess ? GLLM_OK : GLLM_E_HIP;
}

gllm_status gllm_head_create(const gllm_head_config* cfg, gllm_head** out) {
    if (!out) return GLLM_E_INVALID;
    *out = nullptr;
    if (!cfg || cfg->hidden < 64 || cfg->hidden % 64 != 0 || cfg->vocab < 1 || cfg->vocab > (1 << 24) || cfg->max_rows < 1 ||
        !(cfg->rms_eps >= 0.0))
        return GLLM_E_INVALID;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n < 1) return GLLM_E_HIP;
    gllm_head* s = new gllm_head();
    s->cfg = *cfg;
    s->vocab_pad = (int32_t)round_up(cfg->vocab, 256);
    if (hipMalloc((void**)&s->w, (size_t)s->vocab_pad * cfg->hidden * 2) != hipSuccess ||
        hipMalloc((void**)&s->gain, (size_t)cfg->hidden * 2) != hipSuccess) {
        if (s->w) (void)hipFree(s->w);
        delete s;
        return GLLM_E_HIP;
    }
    void* unused = nullptr;
    (void)static_scratch(&unused);  // set-up time: gllm_head_logits_static finds the address ready (it retries if this failed)
    *out = s;
    return GLLM_OK;
}

void gllm_head_destroy(gllm_head* s) {
    if (!s) return;
    (void)hipFree(s->w);
    (void)hipFree(s->gain);
    delete s;
}

const char* gllm_head_last_error(const gllm_head* s) { return s ? s->err.c_str() : "null head"; }

size_t gllm_head_workspace_bytes(const gllm_head* s) {
    return s ? (size_t)round_up(s->cfg.max_rows, 256) * s->cfg.hidden * 2 : 0;
}

gllm_status gllm_head_bind_workspace(gllm_head* s, void* workspace, size_t bytes) {
    if (!s || !workspace) return GLLM_E_INVALID;
    if (bytes < gllm_head_workspace_bytes(s)) return fail(s, GLLM_E_CAPACITY, "workspace too small");
    if ((uintptr_t)workspace % 256 != 0) return fail(s, GLLM_E_INVALID, "workspace must be 256-byte aligned");
    s->h = (bf16_t*)workspace;
    return GLLM_OK;
}

gllm_status gllm_head_load(gllm_head* s, const void* norm_gain, const void* w_vocab, void* stream) {
    if (!s || !norm_gain || !w_vocab) return GLLM_E_INVALID;
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(s->gain, norm_gain, (size_t)s->cfg.hidden * 2, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(s, GLLM_E_HIP, "copy of the norm gain failed");
    pad_rows_kernel<<<s->vocab_pad, 256, 0, st>>>((const bf16_t*)w_vocab, s->w, s->cfg.vocab, s->cfg.hidden);
    if (hipGetLastError() != hipSuccess) return fail(s, GLLM_E_HIP, "weight repack launch failed");
    s->loaded = true;
    return GLLM_OK;
}

int32_t gllm_head_padded_vocab(const gllm_head* s) { return s ? s->vocab_pad : 0; }

// Both projection entry points: rows of x -> normalised bf16 rows in h_buf -> logits (h_buf must hold round_up(num_rows, 256)
// rows, 288 for 257..288 rows; rows past num_rows are read by the GEMM's tiles and their products discarded).
static gllm_status head_logits_into(gllm_head* s, bf16_t* h_buf, const float* x, int32_t num_x_rows, const int32_t* rows,
                                    int32_t num_rows, float* logits, int64_t ld_logits, hipStream_t st) {
    const int H = s->cfg.hidden;
    gather_rmsnorm_kernel<<<num_rows, 256, 0, st>>>(x, num_x_rows, rows, s->gain, h_buf, H, (float)s->cfg.rms_eps);
    if (hipGetLastError() != hipSuccess) return fail(s, GLLM_E_HIP, "norm launch failed");
    const GemmPlan plan = gemm_plan(num_rows, s->vocab_pad, H, GEMM_STORE_F32, 1);
    const hipError_t e = launch_gemm_bf16(h_buf, H, s->w, H, logits, ld_logits, num_rows, s->vocab_pad, H, GEMM_STORE_F32,
                                          plan.tile, 1, 0, st);
    if (e != hipSuccess) return fail(s, GLLM_E_HIP, std::string("projection launch failed: ") + hipGetErrorString(e));
    return GLLM_OK;
}

gllm_status gllm_head_logits(gllm_head* s, const float* x, int32_t num_x_rows, const int32_t* rows, int32_t num_rows,
                             float* logits, int64_t ld_logits, void* stream) {
    if (!s || !x || !rows || !logits || num_x_rows < 1 || num_rows < 0) return GLLM_E_INVALID;
    if (!s->loaded || !s->h) return fail(s, GLLM_E_STATE, "load the weights and bind the workspace first");
    if (num_rows > s->cfg.max_rows) return fail(s, GLLM_E_CAPACITY, "more rows than max_rows");
    if (ld_logits < s->vocab_pad || ld_logits % 4 != 0) return fail(s, GLLM_E_INVALID, "ld_logits must cover the padded vocabulary");
    if (num_rows == 0) return GLLM_OK;
    return head_logits_into(s, s->h, x, num_x_rows, rows, num_rows, logits, ld_logits, (hipStream_t)stream);
}

size_t gllm_head_static_scratch_bytes(void) { return kStaticScratchBytes; }

gllm_status gllm_head_logits_static(gllm_head* s, const float* x, int32_t num_x_rows, const int32_t* rows, int32_t num_rows,
                                    float* logits, int64_t ld_logits, void* stream) {
    if (!s || !x || !rows || !logits || num_x_rows < 1 || num_rows < 0) return GLLM_E_INVALID;
    if (!s->loaded) return fail(s, GLLM_E_STATE, "load the weights first");
    if (ld_logits < s->vocab_pad || ld_logits % 4 != 0) return fail(s, GLLM_E_INVALID, "ld_logits must cover the padded vocabulary");
    // rows the projection's tiles may read: whole bands of 256 (the one 288-row tile for 257..288 rows reads fewer)
    const int64_t rows_read = round_up(num_rows, 256);
    if ((size_t)rows_read * s->cfg.hidden * 2 > kStaticScratchBytes)
        return fail(s, GLLM_E_CAPACITY, "num_rows (rounded up to the projection's row bands) x hidden x 2 bytes exceeds the " +
                                            std::to_string(kStaticScratchBytes >> 20) + " MiB static scratch: use gllm_head_logits with a bound workspace");
    if (num_rows == 0) return GLLM_OK;
    void* buf = nullptr;
    const hipError_t e = static_scratch(&buf);
    if (e != hipSuccess) return fail(s, GLLM_E_HIP, std::string("static scratch address: ") + hipGetErrorString(e));
    return head_logits_into(s, (bf16_t*)buf, x, num_x_rows, rows, num_rows, logits, ld_logits, (hipStream_t)stream);
}

gllm_status gllm_op_sample(const float* logits, int64_t ld_logits, int32_t num_rows, int32_t vocab,
                           const float* temperature, const int32_t* top_k, const float* top_p, const float* u,
                           int32_t* out_ids, void* stream) {
    if (!logits || !temperature || !top_k || !top_p || !u || !out_ids || num_rows < 0 || vocab < 1 || vocab > (1 << 24) ||
        ld_logits < vocab)
        return GLLM_E_INVALID;
    if (num_rows == 0) return GLLM_OK;
    sample_kernel<<<num_rows, kSampleThreads, 0, (hipStream_t)stream>>>(logits, ld_logits, vocab, temperature, top_k, top_p, u,
                                                                        out_ids);
    return hipGetLastError() == hipSuccess ? GLLM_OK : GLLM_E_HIP;
}

}  // extern "C"
