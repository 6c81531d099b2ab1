// sa_moe_dispatch, sa_gather_rows, sa_combine_rows: top-1 routing between the Mult and
// the Shift expert (Sec. 4.2: p = softmax(router logits), G(x) = p_i * 1{p_i >= p_j}).
//
// Dispatch is a stable partition of the token ids by expert, built without atomics so
// that the lists are unique and reproducible.  Up to 32768 tokens it is ONE launch: every
// workgroup of 1024 tokens takes the decisions of ALL tokens from the logits (raw-logit argmax,
// ties to the lowest index; the logits of 12608 tokens are 100 KB, read from the L2), which
// gives it the totals per expert and the counts of the workgroups before it, then ranks its own
// tokens with wavefront ballots / popcounts and writes them.  Longer inputs take three steps
// through a scratch buffer: (1) decisions, gate values and a per-expert histogram per workgroup;
// (2) one small workgroup turns the histograms into start offsets (up to 131072 tokens every
// workgroup of step 3 sums the few histograms itself instead, which saves that launch);
// (3) ranking and writing as above.
#include <mutex>

#include "common.h"

namespace {

using namespace sa;
constexpr int kMaxE = 8;
constexpr int kTok = 256;   // tokens per workgroup
constexpr long kSelfScanBlocks = 512;   // up to this many workgroups (131072 tokens) the scatter pass sums the histograms itself
constexpr long kOneLaunchTokens = 32768; // up to this many tokens one launch does everything (every workgroup reads all logits)

__device__ inline uint64_t lanemask_lt(int lane) { return (lane == 0) ? 0ull : (~0ull >> (64 - lane)); }

__global__ __launch_bounds__(kTok) void route_kernel(const float *__restrict__ logits, long T, int E,
                                                     int32_t *__restrict__ expert_of,
                                                     float *__restrict__ gate,
                                                     int32_t *__restrict__ block_counts) {
    __shared__ int32_t wave_cnt[kTok / 64][kMaxE];
    const long t = (long)blockIdx.x * kTok + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int best = -1;
    if (t < T) {
        const float *l = logits + (size_t)t * E;
        best = 0;
        float lb = l[0];
        for (int e = 1; e < E; ++e) {
            const float le = l[e];
            if (le > lb) { lb = le; best = e; }
        }
        float den = 0.0f;
        for (int e = 0; e < E; ++e) den += __expf(l[e] - lb);
        expert_of[t] = best;
        gate[t] = 1.0f / den;
    }
    for (int e = 0; e < E; ++e) {
        const uint64_t m = __ballot(best == e);
        if (lane == 0) wave_cnt[wave][e] = __builtin_popcountll(m);
    }
    __syncthreads();
    if (threadIdx.x < E) {
        int s = 0;
        for (int w = 0; w < kTok / 64; ++w) s += wave_cnt[w][threadIdx.x];
        block_counts[(size_t)blockIdx.x * E + threadIdx.x] = s;
    }
}

// The index of the largest logit of token t (the first one among equals).
__device__ inline int top1(const float *__restrict__ l, int E) {
    int best = 0;
    float lb = l[0];
    for (int e = 1; e < E; ++e) {
        const float le = l[e];
        if (le > lb) { lb = le; best = e; }
    }
    return best;
}

// One launch for the whole dispatch: workgroup b owns tokens [1024 b, 1024 b + 1024).  Pass 1 over all T tokens
// (thread i takes tokens i, i + 1024, ...; the loads of a thread are independent and issued together): per expert, how
// many tokens it gets in all and how many of them lie in workgroups before b.  Pass 2: the workgroup's own tokens,
// ranked by ballot / popcount behind those counts.
constexpr int kOneTok = 1024;            // tokens (and threads) per workgroup of the one-launch kernel

template <int E_FIXED>
__global__ __launch_bounds__(kOneTok) void route_scatter_kernel(const float *__restrict__ logits, long T, int E_runtime,
                                                                int32_t *__restrict__ expert_of, float *__restrict__ gate,
                                                                int32_t *__restrict__ counts, int32_t *__restrict__ perm) {
    const int E = E_FIXED > 0 ? E_FIXED : E_runtime;
    constexpr int kWaves = kOneTok / 64;
    __shared__ int32_t wave_cnt[kWaves][kMaxE];
    __shared__ int32_t red[kWaves][2 * kMaxE];
    __shared__ int32_t base_s[kMaxE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long first = (long)blockIdx.x * kOneTok;              // tokens before `first` belong to earlier workgroups
    int below[kMaxE], all[kMaxE];
#pragma unroll
    for (int e = 0; e < kMaxE; ++e) below[e] = all[e] = 0;
    float2 own = make_float2(0.0f, 0.0f);                       // E == 2: the logits of this thread's own token, met in pass 1
    if (E_FIXED == 2) {
        const float2 *l2 = reinterpret_cast<const float2 *>(logits);
        constexpr int kBatch = 16;                              // independent loads in flight per thread: 16384 tokens per round trip
        for (long t0 = tid; t0 < T; t0 += (long)kBatch * kOneTok) {
            float2 l[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const long t = t0 + (long)i * kOneTok;
                l[i] = t < T ? l2[t] : make_float2(0.0f, 0.0f);
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const long t = t0 + (long)i * kOneTok;
                const int one = (t < T && l[i].y > l[i].x) ? 1 : 0;     // expert 1 only if strictly larger
                all[1] += one;
                below[1] += t < first ? one : 0;
                if (t == first + tid) own = l[i];
            }
        }
        const int mine_all = T > tid ? (int)((T - tid + kOneTok - 1) / kOneTok) : 0;    // tokens this thread looked at
        const long fb = first - tid;
        const int mine_below = fb > 0 ? (int)((fb + kOneTok - 1) / kOneTok) : 0;          // ... and those before `first`
        all[0] = mine_all - all[1];
        below[0] = mine_below - below[1];
    } else {
        for (long t = tid; t < T; t += kOneTok) {
            const int best = top1(logits + (size_t)t * E, E);
#pragma unroll
            for (int e = 0; e < kMaxE; ++e) {
                all[e] += best == e ? 1 : 0;
                below[e] += (best == e && t < first) ? 1 : 0;
            }
        }
    }
#pragma unroll
    for (int e = 0; e < kMaxE; ++e) {
        if (e >= E) continue;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            below[e] += __shfl_xor(below[e], off, 64);
            all[e] += __shfl_xor(all[e], off, 64);
        }
        if (lane == 0) { red[wave][e] = below[e]; red[wave][kMaxE + e] = all[e]; }
    }
    __syncthreads();
    if (tid < E) {
        int bl = 0, al = 0;
        for (int w = 0; w < kWaves; ++w) { bl += red[w][tid]; al += red[w][kMaxE + tid]; }
        red[0][tid] = bl;                       // (row 0 of red has been read by this thread only)
        red[0][kMaxE + tid] = al;
    }
    __syncthreads();
    if (tid == 0) {
        int start = 0;
        for (int e = 0; e < E; ++e) {
            base_s[e] = start + red[0][e];
            if (blockIdx.x == 0) counts[e] = red[0][kMaxE + e];
            start += red[0][kMaxE + e];
        }
    }
    const long t = first + tid;
    int mine = -1;
    if (t < T) {
        if (E_FIXED == 2) {
            mine = own.y > own.x ? 1 : 0;
            const float lb = mine ? own.y : own.x;
            const float den = __expf(own.x - lb) + __expf(own.y - lb);      // the same sum, in the same order, as the general path
            expert_of[t] = mine;
            gate[t] = 1.0f / den;
        } else {
            const float *l = logits + (size_t)t * E;
            mine = top1(l, E);
            const float lb = l[mine];
            float den = 0.0f;
            for (int e = 0; e < E; ++e) den += __expf(l[e] - lb);
            expert_of[t] = mine;
            gate[t] = 1.0f / den;
        }
    }
    int rank = 0;
    for (int e = 0; e < E; ++e) {
        const uint64_t m = __ballot(mine == e);
        if (mine == e) rank = __builtin_popcountll(m & lanemask_lt(lane));
        if (lane == 0) wave_cnt[wave][e] = __builtin_popcountll(m);
    }
    __syncthreads();
    if (mine >= 0) {
        int before = 0;
        for (int w = 0; w < wave; ++w) before += wave_cnt[w][mine];
        perm[base_s[mine] + before + rank] = (int32_t)t;
    }
}

// block_base[blk][e] = first position in perm of expert e's tokens of workgroup blk: an exclusive scan
// of the per-workgroup histograms, expert by expert, 256 workgroups' counts per pass of one workgroup.
__global__ __launch_bounds__(256) void offsets_kernel(const int32_t *__restrict__ block_counts,
                                                      int32_t *__restrict__ block_base,
                                                      int32_t *__restrict__ counts, long n_blocks, int E) {
    __shared__ int32_t wave_tot[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int start = 0;                                     // position of the first token of (expert e, chunk)
    for (int e = 0; e < E; ++e) {
        const int first = start;
        for (long b0 = 0; b0 < n_blocks; b0 += 256) {
            const long b = b0 + tid;
            const int c = b < n_blocks ? block_counts[(size_t)b * E + e] : 0;
            int incl = c;                              // inclusive scan inside the wavefront
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off, 64);
                if (lane >= off) incl += up;
            }
            __syncthreads();                           // wave_tot of the previous pass has been read
            if (lane == 63) wave_tot[wave] = incl;
            __syncthreads();
            int before = 0, all = 0;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                if (w < wave) before += wave_tot[w];
                all += wave_tot[w];
            }
            if (b < n_blocks) block_base[(size_t)b * E + e] = start + before + incl - c;
            start += all;
        }
        if (tid == 0) counts[e] = start - first;
    }
}

// block_base == nullptr: every workgroup sums the histograms itself (few workgroups: cheaper than a launch of
// the scan in between) - base[e] = all tokens of lower experts + expert e's tokens of lower workgroups - and
// workgroup 0 also writes counts.
__global__ __launch_bounds__(kTok) void scatter_kernel(const int32_t *__restrict__ expert_of, long T, int E,
                                                       const int32_t *__restrict__ block_base,
                                                       const int32_t *__restrict__ block_counts, int32_t *__restrict__ counts,
                                                       int32_t *__restrict__ perm) {
    __shared__ int32_t wave_cnt[kTok / 64][kMaxE];
    __shared__ int32_t red[kTok / 64][2 * kMaxE];
    __shared__ int32_t base_s[kMaxE];
    const long t = (long)blockIdx.x * kTok + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (block_base == nullptr) {
        int below[kMaxE], all[kMaxE];                  // this thread's share of the two sums per expert
#pragma unroll
        for (int e = 0; e < kMaxE; ++e) below[e] = all[e] = 0;
        for (long b = threadIdx.x; b < (long)gridDim.x; b += kTok) {
#pragma unroll
            for (int e = 0; e < kMaxE; ++e) {
                if (e >= E) continue;
                const int c = block_counts[(size_t)b * E + e];
                all[e] += c;
                below[e] += b < (long)blockIdx.x ? c : 0;
            }
        }
#pragma unroll
        for (int e = 0; e < kMaxE; ++e) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                below[e] += __shfl_xor(below[e], off, 64);
                all[e] += __shfl_xor(all[e], off, 64);
            }
            if (lane == 0) { red[wave][e] = below[e]; red[wave][kMaxE + e] = all[e]; }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int start = 0;
            for (int e = 0; e < E; ++e) {
                int bl = 0, al = 0;
                for (int w = 0; w < kTok / 64; ++w) { bl += red[w][e]; al += red[w][kMaxE + e]; }
                base_s[e] = start + bl;
                if (blockIdx.x == 0) counts[e] = al;
                start += al;
            }
        }
        __syncthreads();
    }
    const int mine = (t < T) ? expert_of[t] : -1;
    int rank = 0;
    for (int e = 0; e < E; ++e) {
        const uint64_t m = __ballot(mine == e);
        if (mine == e) rank = __builtin_popcountll(m & lanemask_lt(lane));
        if (lane == 0) wave_cnt[wave][e] = __builtin_popcountll(m);
    }
    __syncthreads();
    if (mine >= 0) {
        int before = 0;
        for (int w = 0; w < wave; ++w) before += wave_cnt[w][mine];
        const int base = block_base ? block_base[(size_t)blockIdx.x * E + mine] : base_s[mine];
        perm[base + before + rank] = (int32_t)t;
    }
}

__global__ __launch_bounds__(256) void gather_kernel(const uint4 *__restrict__ src, int chunks_per_row,
                                                     RowSel sel, uint4 *__restrict__ dst) {
    const int32_t *rows;
    long n_rows;
    resolve_rows(sel, rows, n_rows);
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long i = idx / chunks_per_row;
    const int c = (int)(idx % chunks_per_row);
    if (i >= n_rows) return;
    const long s = rows ? rows[i] : i;
    dst[(size_t)i * chunks_per_row + c] = src[(size_t)s * chunks_per_row + c];
}

__global__ __launch_bounds__(256) void combine_kernel(const float4 *__restrict__ src, int E4, RowSel sel,
                                                      const float *__restrict__ gate,
                                                      float4 *__restrict__ y) {
    const int32_t *rows;
    long n_rows;
    resolve_rows(sel, rows, n_rows);
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long i = idx / E4;
    const int c = (int)(idx % E4);
    if (i >= n_rows) return;
    const long t = rows ? rows[i] : i;
    const float g = gate ? gate[t] : 1.0f;
    const float4 v = src[(size_t)i * E4 + c];
    y[(size_t)t * E4 + c] = make_float4(g * v.x, g * v.y, g * v.z, g * v.w);
}

// ---- forward value of the balancing loss of Eq. 4 -------------------------------------------
// Workgroup partial sums of p_i(x) and q_i(x) = Phi((p_i - max_{j != i} p_j) / noise_std) over 256 tokens,
// then one workgroup adds the partials in ascending order in fp64 and forms the two SCV values.
__device__ inline float wave_sum_f(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(kTok) void balance_partial_kernel(const float *__restrict__ logits, long T, int E,
                                                               float inv_noise_std, float *__restrict__ partial) {
    __shared__ float red[kTok / 64][2 * kMaxE];
    const long t = (long)blockIdx.x * kTok + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float p[kMaxE], q[kMaxE];
#pragma unroll
    for (int e = 0; e < kMaxE; ++e) p[e] = q[e] = 0.0f;
    if (t < T) {
        const float *l = logits + (size_t)t * E;
        float lb = l[0];
#pragma unroll
        for (int e = 1; e < kMaxE; ++e)
            if (e < E) lb = fmaxf(lb, l[e]);
        float den = 0.0f;
#pragma unroll
        for (int e = 0; e < kMaxE; ++e)
            if (e < E) { p[e] = expf(l[e] - lb); den += p[e]; }
        const float r = 1.0f / den;
#pragma unroll
        for (int e = 0; e < kMaxE; ++e) p[e] *= r;
#pragma unroll
        for (int e = 0; e < kMaxE; ++e) {
            if (e >= E) continue;
            float other = -1.0f;
#pragma unroll
            for (int j = 0; j < kMaxE; ++j)
                if (j != e && j < E) other = fmaxf(other, p[j]);
            q[e] = 0.5f * erfcf(-(p[e] - other) * inv_noise_std * 0.70710678118654752f);
        }
    }
#pragma unroll
    for (int e = 0; e < kMaxE; ++e) {
        if (e >= E) continue;
        const float sp = wave_sum_f(p[e]), sq = wave_sum_f(q[e]);
        if (lane == 0) { red[wave][e] = sp; red[wave][kMaxE + e] = sq; }
    }
    __syncthreads();
    if (threadIdx.x < 2 * kMaxE) {
        float s = 0.0f;
        for (int w = 0; w < kTok / 64; ++w) s += red[w][threadIdx.x];
        partial[(size_t)blockIdx.x * 2 * kMaxE + threadIdx.x] = s;
    }
}

__global__ __launch_bounds__(64) void balance_final_kernel(const float *__restrict__ partial, long n_blocks, int E,
                                                           const float *__restrict__ alpha, float *__restrict__ losses,
                                                           float *__restrict__ sums) {
    __shared__ double tot[2 * kMaxE];
    const int i = threadIdx.x;                 // i < 16: (kind, expert) = (i / 8, i % 8)
    if (i < 2 * kMaxE) {
        double s = 0.0;
        for (long b = 0; b < n_blocks; ++b) s += (double)partial[(size_t)b * 2 * kMaxE + i];
        const int e = i % kMaxE;
        tot[i] = e < E ? s * (double)alpha[e] : 0.0;
        if (sums && e < E) sums[(i / kMaxE) * E + e] = (float)tot[i];
    }
    __syncthreads();
    if (i < 2) {
        double mean = 0.0, var = 0.0;
        for (int e = 0; e < E; ++e) mean += tot[i * kMaxE + e];
        mean /= (double)E;
        for (int e = 0; e < E; ++e) { const double c = tot[i * kMaxE + e] - mean; var += c * c; }
        losses[i] = (float)(var / (double)E / (mean * mean));
    }
}

// Scratch of the three-step path: per-workgroup histograms, then their exclusive scan (none up to kOneLaunchTokens).
size_t dispatch_scratch_bytes(long T, int E) {
    if (T <= kOneLaunchTokens || E <= 0) return 0;
    const size_t n_blocks = (size_t)((T + kTok - 1) / kTok);
    return (2 * n_blocks * E * sizeof(int32_t) + 255) / 256 * 256;
}

// Everything of sa_moe_dispatch after the checks that both entry points share; `scratch` holds
// dispatch_scratch_bytes(T, E) bytes (not read before it is written; may be null when that is 0).
int dispatch_launch(const float *logits, long T, int E, int32_t *perm, int32_t *expert_of, int32_t *counts, float *gate,
                    void *scratch, hipStream_t st) {
    if (T <= kOneLaunchTokens) {
        const unsigned blocks = (unsigned)((T + kOneTok - 1) / kOneTok);
        if (E == 2)
            route_scatter_kernel<2><<<dim3(blocks), dim3(kOneTok), 0, st>>>(logits, T, E, expert_of, gate, counts, perm);
        else
            route_scatter_kernel<0><<<dim3(blocks), dim3(kOneTok), 0, st>>>(logits, T, E, expert_of, gate, counts, perm);
        return sa::check_launch("sa_moe_dispatch(one launch)");
    }
    const long n_blocks = (T + kTok - 1) / kTok;
    int32_t *block_counts = static_cast<int32_t *>(scratch);
    int32_t *block_base = block_counts + (size_t)n_blocks * E;
    route_kernel<<<dim3((unsigned)n_blocks), dim3(kTok), 0, st>>>(logits, T, E, expert_of, gate, block_counts);
    int rc = sa::check_launch("sa_moe_dispatch(route)");
    if (rc != SA_OK) return rc;
    if (n_blocks <= kSelfScanBlocks) {
        scatter_kernel<<<dim3((unsigned)n_blocks), dim3(kTok), 0, st>>>(expert_of, T, E, nullptr, block_counts, counts, perm);
        return sa::check_launch("sa_moe_dispatch(scatter)");
    }
    offsets_kernel<<<dim3(1), dim3(256), 0, st>>>(block_counts, block_base, counts, n_blocks, E);
    rc = sa::check_launch("sa_moe_dispatch(offsets)");
    if (rc != SA_OK) return rc;
    scatter_kernel<<<dim3((unsigned)n_blocks), dim3(kTok), 0, st>>>(expert_of, T, E, block_base, block_counts, counts, perm);
    return sa::check_launch("sa_moe_dispatch(scatter)");
}

// Argument checks of both dispatch entry points (everything but the scratch memory).
int dispatch_check(const char *who, const float *logits, long T, int E, int32_t *perm, int32_t *expert_of, int32_t *counts,
                   float *gate) {
    SA_REQUIRE(T >= 0, SA_ERR_INVALID, "%s: T < 0", who);
    SA_REQUIRE(E >= 2 && E <= kMaxE, SA_ERR_SHAPE, "%s: E must be in [2, %d] (got %d)", who, kMaxE, E);
    SA_REQUIRE(T < (1L << 31), SA_ERR_SHAPE, "%s: T >= 2^31", who);
    SA_REQUIRE(counts != nullptr, SA_ERR_INVALID, "%s: counts is NULL", who);
    SA_REQUIRE(sa::aligned16(logits) && sa::aligned16(perm) && sa::aligned16(expert_of) && sa::aligned16(counts) &&
                   sa::aligned16(gate),
               SA_ERR_ALIGN, "%s: pointers must be 16-byte aligned", who);
    SA_REQUIRE(T == 0 || (logits && perm && expert_of && gate), SA_ERR_INVALID, "%s: NULL buffer", who);
    return SA_OK;
}

}  // namespace

extern "C" size_t sa_moe_dispatch_workspace_bytes(long T, int E) { return dispatch_scratch_bytes(T, E); }

size_t sa::moe_dispatch_scratch_bytes(long T, int E) { return dispatch_scratch_bytes(T, E); }
int sa::moe_dispatch_launch(const float *logits, long T, int E, int32_t *perm, int32_t *expert_of, int32_t *counts, float *gate,
                            void *scratch, hipStream_t st) {
    return dispatch_launch(logits, T, E, perm, expert_of, counts, gate, scratch, st);
}

extern "C" int sa_moe_dispatch(const float *logits, long T, int E, int32_t *perm, int32_t *expert_of,
                               int32_t *counts, float *gate, void *workspace, size_t workspace_bytes,
                               void *stream) {
    sa::clear_error();
    int rc = dispatch_check("sa_moe_dispatch", logits, T, E, perm, expert_of, counts, gate);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(sa::aligned16(workspace), SA_ERR_ALIGN, "sa_moe_dispatch: the workspace must be 16-byte aligned");
    hipStream_t st = sa::as_stream(stream);
    if (T == 0) return sa::launch_zero(counts, ((size_t)E * 4 + 3) / 4 * 4, st);
    const size_t need = dispatch_scratch_bytes(T, E);
    SA_REQUIRE(need == 0 || (workspace != nullptr && workspace_bytes >= need), SA_ERR_WORKSPACE,
               "sa_moe_dispatch: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    return dispatch_launch(logits, T, E, perm, expert_of, counts, gate, workspace, st);
}

// ---- the dispatch for callers that cannot allocate -------------------------------------------------
// Its scratch (the histograms and their scan of the three-step path) is this array instead of a workspace:
// 2 * 4096 workgroups * 8 experts * 4 bytes = 256 KiB, enough for kStaticTokens tokens.  Every GPU the library
// runs on holds its own copy at its own address until the process ends; in host code the name `scratch` is only
// a handle for hipGetSymbolAddress, the kernels get the address that call returns for the current device.
constexpr long kStaticTokens = 1L << 20;
static __device__ __align__(256) int32_t scratch[2 * (kStaticTokens / 256) * 8];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each device, asked for once per device

int static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return sa::fail(SA_ERR_HIP, "sa_moe_dispatch_static: hipGetDevice: %s", hipGetErrorString(e));
    SA_REQUIRE(dev >= 0 && dev < kMaxDevices, SA_ERR_UNSUPPORTED, "sa_moe_dispatch_static: device %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr)
            return sa::fail(SA_ERR_HIP, "sa_moe_dispatch_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SA_OK;
}

}  // namespace

extern "C" long sa_moe_dispatch_static_max_tokens(void) { return kStaticTokens; }

extern "C" int sa_moe_dispatch_static(const float *logits, long T, int E, int32_t *perm, int32_t *expert_of,
                                      int32_t *counts, float *gate, void *stream) {
    sa::clear_error();
    int rc = dispatch_check("sa_moe_dispatch_static", logits, T, E, perm, expert_of, counts, gate);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(T <= kStaticTokens, SA_ERR_UNSUPPORTED,
               "sa_moe_dispatch_static: %ld tokens exceed the %ld the built-in scratch holds; use sa_moe_dispatch with a workspace",
               T, kStaticTokens);
    static_assert(sizeof(scratch) >= 2 * ((kStaticTokens + kTok - 1) / kTok) * kMaxE * sizeof(int32_t), "scratch too small");
    hipStream_t st = sa::as_stream(stream);
    if (T == 0) return sa::launch_zero(counts, ((size_t)E * 4 + 3) / 4 * 4, st);
    void *ws = nullptr;
    if (dispatch_scratch_bytes(T, E) != 0) {
        rc = static_scratch(&ws);
        if (rc != SA_OK) return rc;
    }
    return dispatch_launch(logits, T, E, perm, expert_of, counts, gate, ws, st);
}

extern "C" int sa_gather_rows(const void *src, size_t row_bytes, const sa_rows *rows, void *dst, void *stream) {
    sa::clear_error();
    sa::RowSel sel;
    int rc = sa::validate_rows(rows, &sel);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(row_bytes > 0 && row_bytes % 16 == 0, SA_ERR_SHAPE, "sa_gather_rows: row_bytes must be a positive multiple of 16");
    if (sel.max_rows == 0) return SA_OK;
    SA_REQUIRE(src && dst, SA_ERR_INVALID, "sa_gather_rows: NULL buffer");
    SA_REQUIRE(sa::aligned16(src) && sa::aligned16(dst) && sa::aligned4(sel.rows), SA_ERR_ALIGN,
               "sa_gather_rows: pointers must be 16-byte aligned");
    const int cpr = (int)(row_bytes / 16);
    const long total = sel.max_rows * cpr;
    const long blocks = (total + 255) / 256;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_gather_rows: too large");
    gather_kernel<<<dim3((unsigned)blocks), dim3(256), 0, sa::as_stream(stream)>>>(
        static_cast<const uint4 *>(src), cpr, sel, static_cast<uint4 *>(dst));
    return sa::check_launch("sa_gather_rows");
}

extern "C" int sa_combine_rows(const float *src, const sa_rows *rows, const float *gate_or_null, int E,
                               float *y, void *stream) {
    sa::clear_error();
    sa::RowSel sel;
    int rc = sa::validate_rows(rows, &sel);
    if (rc != SA_OK) return rc;
    SA_REQUIRE(E > 0 && E % 4 == 0, SA_ERR_SHAPE, "sa_combine_rows: E must be a positive multiple of 4");
    if (sel.max_rows == 0) return SA_OK;
    SA_REQUIRE(src && y, SA_ERR_INVALID, "sa_combine_rows: NULL buffer");
    SA_REQUIRE(sa::aligned16(src) && sa::aligned16(y) && sa::aligned16(gate_or_null) && sa::aligned4(sel.rows),
               SA_ERR_ALIGN, "sa_combine_rows: pointers must be 16-byte aligned");
    const long total = sel.max_rows * (E / 4);
    const long blocks = (total + 255) / 256;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_combine_rows: too large");
    combine_kernel<<<dim3((unsigned)blocks), dim3(256), 0, sa::as_stream(stream)>>>(
        reinterpret_cast<const float4 *>(src), E / 4, sel, gate_or_null, reinterpret_cast<float4 *>(y));
    return sa::check_launch("sa_combine_rows");
}

extern "C" size_t sa_moe_balance_loss_workspace_bytes(long T, int E) {
    if (T <= 0 || E < 2 || E > kMaxE) return 0;
    return (size_t)((T + kTok - 1) / kTok) * 2 * kMaxE * sizeof(float);
}

extern "C" int sa_moe_balance_loss(const float *logits, long T, int E, const float *alpha, float noise_std,
                                   float *losses, float *sums_or_null, void *workspace, size_t workspace_bytes,
                                   void *stream) {
    sa::clear_error();
    SA_REQUIRE(T > 0, SA_ERR_INVALID, "sa_moe_balance_loss: T must be positive (the loss of no tokens is 0 / 0)");
    SA_REQUIRE(E >= 2 && E <= kMaxE, SA_ERR_SHAPE, "sa_moe_balance_loss: 2 to 8 experts (got %d)", E);
    SA_REQUIRE(noise_std > 0.0f && noise_std - noise_std == 0.0f, SA_ERR_INVALID,
               "sa_moe_balance_loss: noise_std must be positive and finite");
    SA_REQUIRE(logits && alpha && losses, SA_ERR_INVALID, "sa_moe_balance_loss: NULL buffer");
    SA_REQUIRE(sa::aligned16(logits) && sa::aligned16(alpha) && sa::aligned16(losses) && sa::aligned16(sums_or_null) &&
                   sa::aligned16(workspace),
               SA_ERR_ALIGN, "sa_moe_balance_loss: pointers must be 16-byte aligned");
    const size_t need = sa_moe_balance_loss_workspace_bytes(T, E);
    SA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SA_ERR_WORKSPACE,
               "sa_moe_balance_loss: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    const long n_blocks = (T + kTok - 1) / kTok;
    SA_REQUIRE(n_blocks < (1L << 31), SA_ERR_SHAPE, "sa_moe_balance_loss: T too large");
    hipStream_t st = sa::as_stream(stream);
    float *partial = static_cast<float *>(workspace);
    balance_partial_kernel<<<dim3((unsigned)n_blocks), dim3(kTok), 0, st>>>(logits, T, E, 1.0f / noise_std, partial);
    int rc = sa::check_launch("sa_moe_balance_loss(partial sums)");
    if (rc != SA_OK) return rc;
    balance_final_kernel<<<dim3(1), dim3(64), 0, st>>>(partial, n_blocks, E, alpha, losses, sums_or_null);
    return sa::check_launch("sa_moe_balance_loss(final)");
}

// ---- the MoE form of one Linear layer -----------------------------------------------------------------
// Sec. 4.1 turns the Linear layers of the attention module into Shift layers or into MoEs; this is the MoE:
// top-1 routing between a Mult expert (fp16 weights, fp16 activations) and a Shift expert (4-bit shift weights,
// int8 activations), each a single layer, y[t, :] = gate[t] * E_i(x[t, :]) (Sec. 4.2).  Three launches: the
// routing, then one tiled GEMM per expert over the rows it was given (gathered by row id on the way into LDS,
// scattered with the gate on the way out), plus the decode of the shift weights where the variant needs one.
namespace {

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct MoeLinearLayout {
    size_t perm, expert_of, counts, gate, scratch, planes, total;
};

MoeLinearLayout moe_linear_layout(long T, int K, int N, int variant) {
    MoeLinearLayout L;
    size_t off = 0;
    L.perm = off; off += up256((size_t)T * 4);
    L.expert_of = off; off += up256((size_t)T * 4);
    L.counts = off; off += 256;
    L.gate = off; off += up256((size_t)T * 4);
    L.scratch = off; off += up256(dispatch_scratch_bytes(T, 2));
    L.planes = off; off += up256(sa::shift_linear_rows_workspace_bytes(K, N, variant));
    L.total = off;
    return L;
}

}  // namespace

extern "C" size_t sa_moe_linear_workspace_bytes(long T, int K, int N, int variant) {
    if (T <= 0 || K <= 0 || N <= 0 || K % 32 != 0 || variant < 0 || variant > 3) return 0;
    return moe_linear_layout(T, K, N, variant).total;
}

extern "C" int sa_moe_linear(const int8_t *xq, const void *xh, const float *logits, long T, int K, int N, const uint8_t *w4,
                             const void *w_f16, float out_scale, float *y, int32_t *expert_of_or_null, float *gate_or_null,
                             int variant, void *workspace, size_t workspace_bytes, void *stream) {
    sa::clear_error();
    SA_REQUIRE(T >= 0 && K > 0 && N > 0, SA_ERR_INVALID, "sa_moe_linear: T < 0, or K or N not positive");
    SA_REQUIRE(variant >= 0 && variant <= 3, SA_ERR_INVALID, "sa_moe_linear: unknown variant %d", variant);
    SA_REQUIRE(K % 32 == 0, SA_ERR_SHAPE, "sa_moe_linear: K (%d) must be a multiple of 32", K);
    SA_REQUIRE(K <= 131072, SA_ERR_SHAPE, "sa_moe_linear: K too large for int32 accumulation");
    SA_REQUIRE(T < (1L << 31), SA_ERR_SHAPE, "sa_moe_linear: T >= 2^31");
    if (T == 0) return SA_OK;
    SA_REQUIRE(xq && xh && logits && w4 && w_f16 && y, SA_ERR_INVALID, "sa_moe_linear: NULL buffer");
    SA_REQUIRE(sa::aligned16(xq) && sa::aligned16(xh) && sa::aligned16(logits) && sa::aligned16(w4) && sa::aligned16(w_f16) &&
                   sa::aligned16(y) && sa::aligned16(expert_of_or_null) && sa::aligned16(gate_or_null) &&
                   sa::aligned16(workspace),
               SA_ERR_ALIGN, "sa_moe_linear: pointers must be 16-byte aligned");
    const MoeLinearLayout L = moe_linear_layout(T, K, N, variant);
    SA_REQUIRE(workspace != nullptr && workspace_bytes >= L.total, SA_ERR_WORKSPACE,
               "sa_moe_linear: workspace of %zu bytes needed, %zu given", L.total, workspace_bytes);
    hipStream_t st = sa::as_stream(stream);
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    int32_t *perm = reinterpret_cast<int32_t *>(ws + L.perm);
    int32_t *expert_of = expert_of_or_null ? expert_of_or_null : reinterpret_cast<int32_t *>(ws + L.expert_of);
    int32_t *counts = reinterpret_cast<int32_t *>(ws + L.counts);
    float *gate = gate_or_null ? gate_or_null : reinterpret_cast<float *>(ws + L.gate);
    int rc = dispatch_launch(logits, T, 2, perm, expert_of, counts, gate, ws + L.scratch, st);
    if (rc != SA_OK) return rc;
    // every token belongs to exactly one expert, so the two scatters write every row of y exactly once
    const sa::RowSel mult_rows{perm, counts, 0, T}, shift_rows{perm, counts, 1, T};
    rc = sa::mult_linear_rows(xh, mult_rows, K, N, w_f16, y, gate, st);
    if (rc != SA_OK) return rc;
    return sa::shift_linear_rows(xq, shift_rows, K, N, w4, out_scale, y, gate, variant, ws + L.planes, st);
}
