// K^T V and Q (K^T V) of the additive attention (Eq. 3, O_Add; Sec. 4.1) on the matrix cores.
//
// An Add layer is a contraction with a +-1 operand: KV[bit, c] = sum_n s(n, bit) V[n, c] and
// out[n, c] = scale * sum_bit s(n, bit) KV[bit, c], s = +1 where the code bit is set, else -1.
// +-1 is exact in bf16, and an fp32 value is exactly the sum of three bf16 terms (each rounded to
// nearest from what the previous ones left), so v_mfma_f32_32x32x16_bf16 against the three term
// planes of the fp32 operand adds exactly the values the Add layer adds, in fp32: the same
// arithmetic as sign-select-and-accumulate on the vector ALU, at the matrix cores' rate (the
// plain-VALU rate is 39 T adds/s on this chip; the three-plane bf16 form runs ~20 times faster).
//
//   K^T V   : M = code bits (one 64-bit word = two 32-bit tiles per wavefront), N = dv columns,
//             K = tokens, 16 per MFMA.  The A operand is built in registers from the code words
//             (one bit-field extract per element); V is staged through LDS transposed into its
//             three bf16 planes, 64 tokens per chunk, double-buffered.  Token ranges are split over workgroups;
//             partial sums meet in a second pass in ascending order (no float atomics).
//   Q(K^T V): M = tokens (TM 32-token tiles per wavefront), N = dv columns, K = code bits.  The
//             A operand of a step is the 8 bf16 signs of one code byte, read from a 256-entry
//             table in LDS; K^T V is staged once per workgroup, transposed into its three planes.
#include <type_traits>

#include "common.h"

namespace {

using sa::kWave;

constexpr int kStageBatch = 4;             // staging tasks whose loads a thread keeps in flight together

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

// (a, b) = sum of three bf16 term pairs, exactly: each term is the round-to-nearest bf16 of what the
// previous terms left.  t[p] holds term p of a in its lower and of b in its upper half (one
// v_cvt_pk_bf16_f32 per term pair).
__device__ inline void split3_pair(float a, float b, uint32_t (&t)[3]) {
    v2f r = {a, b};
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        t[p] = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, v2bf));
        if (p < 2) {
            r[0] -= __builtin_bit_cast(float, t[p] << 16);
            r[1] -= __builtin_bit_cast(float, t[p] & 0xFFFF0000u);
        }
    }
}

// Rows r0, r0+1 (pairs) x columns of an fp32 matrix [n_rows, DV] with row stride `row_stride` floats
// -> three transposed bf16 planes plane[p][col * stride + row], rows >= n_valid zero.  One task =
// two consecutive rows x four columns; a thread issues the loads of kStageBatch tasks together.
template <int DV>
__device__ inline void stage_transposed(const float *__restrict__ src, size_t row_stride, int n_valid, int n_pad,
                                        uint16_t *plane0, uint16_t *plane1, uint16_t *plane2, int stride, int tid,
                                        int n_threads) {
    const int n_tasks = (n_pad / 2) * (DV / 4);
    for (int base = 0; base < n_tasks; base += n_threads * kStageBatch) {
        float4 v0[kStageBatch], v1[kStageBatch];
#pragma unroll
        for (int u = 0; u < kStageBatch; ++u) {
            const int t = base + u * n_threads + tid;
            const int c4 = t % (DV / 4), j = 2 * (t / (DV / 4));
            v0[u] = v1[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            const float *p = src + (size_t)j * row_stride + c4 * 4;
            if (t < n_tasks && j < n_valid) v0[u] = *reinterpret_cast<const float4 *>(p);
            if (t < n_tasks && j + 1 < n_valid) v1[u] = *reinterpret_cast<const float4 *>(p + row_stride);
        }
#pragma unroll
        for (int u = 0; u < kStageBatch; ++u) {
            const int t = base + u * n_threads + tid;
            if (t >= n_tasks) continue;
            const int c4 = t % (DV / 4), j = 2 * (t / (DV / 4));
            const float a0[4] = {v0[u].x, v0[u].y, v0[u].z, v0[u].w}, a1[4] = {v1[u].x, v1[u].y, v1[u].z, v1[u].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uint32_t t[3];
                split3_pair(a0[c], a1[c], t);
                const int off = (c4 * 4 + c) * stride + j;             // even: 4-byte aligned
                *reinterpret_cast<uint32_t *>(plane0 + off) = t[0];
                *reinterpret_cast<uint32_t *>(plane1 + off) = t[1];
                *reinterpret_cast<uint32_t *>(plane2 + off) = t[2];
            }
        }
    }
}

// The three transposed K^T V planes, the sign table and some slack must fit the LDS of a CU.
constexpr bool qkv_fits(int dv, int nbits) { return (size_t)3 * dv * (nbits + 8) * 2 + 4096 <= 150 * 1024; }

// Two bf16 code values in one dword: +1.0 (0x3F80) where the bit of `lo` / `hi` at position `pos` is set;
// a clear bit stands for -1.0, or for 0.0 with ZO ({0,1} codes: the Add layer that skips zeros).
template <bool ZO>
__device__ inline uint32_t sign_pair(uint32_t lo, uint32_t hi, int pos) {
    if (ZO) {
        const uint32_t bl = __builtin_amdgcn_ubfe(lo, pos, 1), bh = __builtin_amdgcn_ubfe(hi, pos, 1);
        return (bl * 0x3F80u) | (bh * 0x3F800000u);
    }
    const uint32_t nl = __builtin_amdgcn_ubfe(~lo, pos, 1), nh = __builtin_amdgcn_ubfe(~hi, pos, 1);
    return 0x3F803F80u | (nl << 15) | (nh << 31);
}

// ------------------------------------------------------------------------------ K^T V ----
// Workgroup: one (b, h), one group of up to 4 code words, one token range.  WB words per group
// (1, 2, 3 or 4), PH token phases (wavefronts that share a word take alternate 16-token steps).
// Tokens pass in chunks of 64 through two LDS buffers: the rows of chunk c+1 are loaded into
// registers before chunk c is multiplied and written (split into their planes) after it.
constexpr int kTok = 64;                   // tokens per chunk
constexpr int kTokStride = kTok + 8;       // bf16 elements per transposed row: 144 bytes, conflict-free b128 reads

template <int DV>
struct KtvChunk {
    static constexpr int U = (kTok / 2 * (DV / 4) + 191) / 192;      // staging tasks per thread (>= 192 threads)
    float4 v0[U], v1[U];
    uint64_t code;
};

template <int DV>
__device__ inline void ktv_load(KtvChunk<DV> &c, const uint64_t *__restrict__ k_codes, const float *__restrict__ v,
                                long bh, int b, int h, int H, int Nk, int W, int w0, int wb, int WB, long j0, int n,
                                int tid, int n_threads) {
    // one code word per thread: kTok * WB <= 256 of them, zero past the last token / word
    const int j = tid / WB, wq = tid % WB;
    c.code = (tid < kTok * WB && j < n && wq < wb) ? k_codes[((size_t)bh * Nk + j0 + j) * W + w0 + wq] : 0ull;
    constexpr int n_tasks = kTok / 2 * (DV / 4);
    const float *src = v + (((size_t)b * Nk + j0) * H + h) * DV;
    const size_t row_stride = (size_t)H * DV;
#pragma unroll
    for (int u = 0; u < KtvChunk<DV>::U; ++u) {
        const int t = u * n_threads + tid;
        const int c4 = t % (DV / 4), jr = 2 * (t / (DV / 4));
        c.v0[u] = c.v1[u] = make_float4(0.f, 0.f, 0.f, 0.f);     // rows past the last token add nothing
        const float *p = src + (size_t)jr * row_stride + c4 * 4;
        if (t < n_tasks && jr < n) c.v0[u] = *reinterpret_cast<const float4 *>(p);
        if (t < n_tasks && jr + 1 < n) c.v1[u] = *reinterpret_cast<const float4 *>(p + row_stride);
    }
}

template <int DV>
__device__ inline void ktv_store(const KtvChunk<DV> &c, uint64_t *kc, uint16_t *plane0, uint16_t *plane1, uint16_t *plane2,
                                 int WB, int tid, int n_threads) {
    if (tid < kTok * WB) kc[tid] = c.code;
    constexpr int n_tasks = kTok / 2 * (DV / 4);
#pragma unroll
    for (int u = 0; u < KtvChunk<DV>::U; ++u) {
        const int t = u * n_threads + tid;
        if (t >= n_tasks) continue;
        const int c4 = t % (DV / 4), jr = 2 * (t / (DV / 4));
        const float a0[4] = {c.v0[u].x, c.v0[u].y, c.v0[u].z, c.v0[u].w}, a1[4] = {c.v1[u].x, c.v1[u].y, c.v1[u].z, c.v1[u].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t t3[3];
            split3_pair(a0[q], a1[q], t3);
            const int off = (c4 * 4 + q) * kTokStride + jr;          // even: 4-byte aligned
            *reinterpret_cast<uint32_t *>(plane0 + off) = t3[0];
            *reinterpret_cast<uint32_t *>(plane1 + off) = t3[1];
            *reinterpret_cast<uint32_t *>(plane2 + off) = t3[2];
        }
    }
}

template <int DV, bool ZO>
__global__ __launch_bounds__(256) void ktv_mfma_kernel(const uint64_t *__restrict__ k_codes, const float *__restrict__ v,
                                                       float *__restrict__ dst, int H, int Nk, int W, int WB, int PH,
                                                       int splits, int tokens_per_block) {
    constexpr int JT = DV / 32;
    constexpr int PLANE = DV * kTokStride;
    __shared__ __attribute__((aligned(16))) uint64_t kc_s[2][kTok * 4];
    __shared__ __attribute__((aligned(16))) uint16_t vt_s[2][3 * PLANE];
    static_assert(sizeof(vt_s) >= 4 * 2 * JT * 16 * 64 * 4 / 2, "the phase reduction reuses the V planes");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_threads = blockDim.x;
    const int n_groups = (W + 3) / 4;
    // blockIdx.x = (bh * n_groups + group) * splits + split
    const int split = blockIdx.x % splits;
    const long bhg = blockIdx.x / splits;
    const int group = (int)(bhg % n_groups);
    const long bh = bhg / n_groups;
    const int b = (int)(bh / H), h = (int)(bh % H);
    const int w0 = group * 4;
    const int wb = min(WB, W - w0);               // words of this group
    const int wl = wave % WB, phase = wave / WB;  // this wavefront's word (within the group) and token phase
    const bool active = wl < wb;
    const int m = lane & 31, kg = lane >> 5;

    v16f acc[2][JT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][jt][r] = 0.0f;

    const long first = (long)split * tokens_per_block;
    const long last = min((long)Nk, first + tokens_per_block);
    KtvChunk<DV> regs;
    if (first < last)
        ktv_load<DV>(regs, k_codes, v, bh, b, h, H, Nk, W, w0, wb, WB, first, (int)min((long)kTok, last - first), tid,
                     n_threads);
    int buf = 0;
    for (long j0 = first; j0 < last; j0 += kTok, buf ^= 1) {
        const int n = (int)min((long)kTok, last - j0);
        const int n_pad = (n + 15) & ~15;
        uint16_t *pl = vt_s[buf];
        ktv_store<DV>(regs, kc_s[buf], pl, pl + PLANE, pl + 2 * PLANE, WB, tid, n_threads);
        __syncthreads();                           // this chunk is staged; the other buffer has been consumed
        if (j0 + kTok < last)
            ktv_load<DV>(regs, k_codes, v, bh, b, h, H, Nk, W, w0, wb, WB, j0 + kTok,
                         (int)min((long)kTok, last - j0 - kTok), tid, n_threads);
        if (!active) continue;
        const uint64_t *kc = kc_s[buf];
        for (int k0 = 16 * phase; k0 < n_pad; k0 += 16 * PH) {
            const int kb = k0 + 8 * kg;            // this lane's first token of the step
            uint32_t lo[8], hi[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint64_t wd = kc[(kb + e) * WB + wl];
                lo[e] = (uint32_t)wd;
                hi[e] = (uint32_t)(wd >> 32);
            }
            // A operands: element e of the lane is token kb + e, bit m of the lower / upper half word
            uint32_t a0[4], a1[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                a0[e2] = sign_pair<ZO>(lo[2 * e2], lo[2 * e2 + 1], m);
                a1[e2] = sign_pair<ZO>(hi[2 * e2], hi[2 * e2 + 1], m);
            }
            const v8bf s0 = __builtin_bit_cast(v8bf, make_uint4(a0[0], a0[1], a0[2], a0[3]));
            const v8bf s1 = __builtin_bit_cast(v8bf, make_uint4(a1[0], a1[1], a1[2], a1[3]));
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                const int off = (jt * 32 + m) * kTokStride + kb;
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    const v8bf vp = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(pl + p * PLANE + off));
                    acc[0][jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(s0, vp, acc[0][jt], 0, 0, 0);
                    acc[1][jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(s1, vp, acc[1][jt], 0, 0, 0);
                }
            }
        }
    }

    // token phases of one word meet in LDS, ascending phase order
    if (PH > 1) {
        float *red = reinterpret_cast<float *>(&vt_s[0][0]);     // 2 * JT * 16 * 64 floats per word
        for (int ph = 1; ph < PH; ++ph) {
            __syncthreads();
            if (active && phase == ph) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) red[((wl * 2 * JT + t * JT + jt) * 16 + r) * 64 + lane] = acc[t][jt][r];
            }
            __syncthreads();
            if (active && phase == 0) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[t][jt][r] += red[((wl * 2 * JT + t * JT + jt) * 16 + r) * 64 + lane];
            }
        }
    }
    if (!active || phase != 0) return;
    // dst: [splits][BH][nbits][DV]; accumulator row = bit within the 32-bit tile, column = lane % 32
    const size_t bh_count = (size_t)gridDim.x / splits / n_groups;
    float *o = dst + (((size_t)split * bh_count + bh) * W + w0 + wl) * 64 * DV;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int bit = t * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                o[(size_t)bit * DV + jt * 32 + m] = acc[t][jt][r];
            }
}

// --------------------------------------------------------------------------- Q (K^T V) ----
// Workgroup: one (b, h) and a range of token tiles; kQkvWaves wavefronts, TM 32-token tiles each per pass.
constexpr int kQkvWaves = 8;

// den (optional, {0,1} codes): int32 [B*H, Nq], the row normaliser; the row then leaves as acc / (den + eps)
// instead of scale * acc.
template <int DV, int W, int TM, bool ZO>
__global__ __launch_bounds__(kQkvWaves * 64) void qkv_mfma_kernel(const uint64_t *__restrict__ q_codes, const float *__restrict__ kv,
                                                       float *__restrict__ out, int H, int Nq, int blocks_per_bh,
                                                       int tiles_per_block, float scale, const int32_t *__restrict__ den,
                                                       float eps) {
    constexpr int JT = DV / 32;
    constexpr int NBITS = W * 64;
    constexpr int STRIDE = NBITS + 8;             // bf16 elements per transposed K^T V row
    __shared__ __attribute__((aligned(16))) uint16_t kvt_s[3][DV * STRIDE];
    __shared__ __attribute__((aligned(16))) uint4 sign_s[256];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long bh = blockIdx.x / blocks_per_bh;
    const int part = blockIdx.x % blocks_per_bh;
    const int b = (int)(bh / H), h = (int)(bh % H);
    const int m = lane & 31, kg = lane >> 5;

    // byte -> its 8 bits as bf16 signs, element e = bit e
    if (tid < 256) {
        uint32_t d[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) d[e2] = sign_pair<ZO>((uint32_t)tid, (uint32_t)tid >> 1, 2 * e2);
        sign_s[tid] = make_uint4(d[0], d[1], d[2], d[3]);
    }
    stage_transposed<DV>(kv + (size_t)bh * NBITS * DV, (size_t)DV, NBITS, NBITS, kvt_s[0], kvt_s[1], kvt_s[2], STRIDE, tid,
                         kQkvWaves * 64);
    __syncthreads();

    const int n_tiles = (Nq + 31) / 32;
    const int tile_begin = part * tiles_per_block;
    const int tile_end = min(n_tiles, tile_begin + tiles_per_block);
    for (int tile0 = tile_begin + wave * TM; tile0 < tile_end; tile0 += kQkvWaves * TM) {
        uint32_t code[TM][2 * W];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int n = min((tile0 + tm) * 32 + m, Nq - 1);
            const uint64_t *cp = q_codes + ((size_t)bh * Nq + n) * W;
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const uint64_t wd = cp[w];
                code[tm][2 * w] = (uint32_t)wd;
                code[tm][2 * w + 1] = (uint32_t)(wd >> 32);
            }
        }
        v16f acc[TM][JT];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[tm][jt][r] = 0.0f;

#pragma unroll
        for (int ks = 0; ks < NBITS / 16; ++ks) {
            // bits 16 ks + 8 kg .. + 7 of the code: one byte of half word ks / 2
            v8bf a[TM];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const uint32_t byte = __builtin_amdgcn_ubfe(code[tm][ks >> 1], 16 * (ks & 1) + 8 * kg, 8);
                a[tm] = __builtin_bit_cast(v8bf, sign_s[byte]);
            }
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                const int off = (jt * 32 + m) * STRIDE + 16 * ks + 8 * kg;
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    const v8bf kp = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(kvt_s[p] + off));
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
                        acc[tm][jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], kp, acc[tm][jt], 0, 0, 0);
                }
            }
            // keep the steps apart: hoisting every operand read of the tile to the top costs hundreds of registers
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            if (tile0 + tm >= tile_end) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = (tile0 + tm) * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
                if (n < Nq) {
                    float *o = out + (((size_t)b * Nq + n) * H + h) * DV + m;
                    const float f = den ? 1.0f / ((float)den[(size_t)bh * Nq + n] + eps) : scale;
#pragma unroll
                    for (int jt = 0; jt < JT; ++jt) o[jt * 32] = f * acc[tm][jt][r];
                }
            }
        }
    }
}

template <int DV, int W>
void launch_qkv_w(const uint64_t *q_codes, const float *kv, float *out, long BH, int H, int Nq, float scale, bool zo,
                  const int32_t *den, float eps, hipStream_t st) {
    constexpr int TM = DV == 128 ? 1 : 2;       // accumulators: TM * DV / 32 tiles of 16 registers
    const int n_tiles = (Nq + 31) / 32;
    // enough workgroups to fill the chip, but each stages all of K^T V once: several passes of its wavefronts
    long per_bh = (1024 + BH - 1) / BH;
    const int passes = (size_t)W * 64 * DV * 4 >= 32768 ? 4 : 1;      // a small K^T V is cheap to stage again
    const long max_per_bh = (n_tiles + kQkvWaves * TM * passes - 1) / (kQkvWaves * TM * passes);
    if (per_bh > max_per_bh) per_bh = max_per_bh;
    if (per_bh < 1) per_bh = 1;
    const int tiles_per_block = (int)((n_tiles + per_bh - 1) / per_bh);
    const dim3 grid((unsigned)(BH * per_bh)), block(kQkvWaves * 64);
    if (zo)
        qkv_mfma_kernel<DV, W, TM, true><<<grid, block, 0, st>>>(q_codes, kv, out, H, Nq, (int)per_bh, tiles_per_block, scale, den, eps);
    else
        qkv_mfma_kernel<DV, W, TM, false><<<grid, block, 0, st>>>(q_codes, kv, out, H, Nq, (int)per_bh, tiles_per_block, scale, den, eps);
}

template <int DV>
bool launch_qkv_dv(int W, const uint64_t *q_codes, const float *kv, float *out, long BH, int H, int Nq, float scale, bool zo,
                   const int32_t *den, float eps, hipStream_t st) {
    switch (W) {
        case 1: launch_qkv_w<DV, 1>(q_codes, kv, out, BH, H, Nq, scale, zo, den, eps, st); return true;
        case 2: launch_qkv_w<DV, 2>(q_codes, kv, out, BH, H, Nq, scale, zo, den, eps, st); return true;
        case 4:
            if constexpr (qkv_fits(DV, 256)) {
                launch_qkv_w<DV, 4>(q_codes, kv, out, BH, H, Nq, scale, zo, den, eps, st);
                return true;
            }
            return false;
        default: return false;
    }
}

}  // namespace

namespace sa {

// Shapes the matrix-core kernels take: K^T V any nbits (multiple of 64); Q(K^T V) 64-, 128- or
// 256-bit codes whose three K^T V planes fit the LDS.
bool additive_mfma_ktv_supported(int nbits, int dv) { return nbits % 64 == 0 && (dv == 32 || dv == 64 || dv == 128); }

bool additive_mfma_qkv_supported(int nbits, int dv) {
    if (!(nbits == 64 || nbits == 128 || nbits == 256) || !(dv == 32 || dv == 64 || dv == 128)) return false;
    return qkv_fits(dv, nbits);
}

// Token splits of the K^T V pass: enough workgroups to fill the chip, whole 128-token chunks each.
AdditiveMfmaPlan plan_additive_mfma(int B, int H, int Nk, int nbits) {
    AdditiveMfmaPlan p;
    const int W = nbits / 64;
    p.groups = (W + 3) / 4;
    p.wb = W < 4 ? W : 4;
    p.ph = p.wb == 1 ? 4 : (p.wb == 2 ? 2 : 1);
    const long base = (long)B * H * p.groups;
    long splits = (768 + base - 1) / base;
    const long chunks = ((long)Nk + kTok - 1) / kTok;
    if (splits > chunks) splits = chunks;
    if (splits < 1) splits = 1;
    if (splits > 256) splits = 256;
    const long chunks_per_block = (chunks + splits - 1) / splits;
    p.tokens_per_block = (int)(chunks_per_block * kTok);
    p.splits = (int)((chunks + chunks_per_block - 1) / chunks_per_block);
    return p;
}

int launch_ktv_mfma(const uint64_t *k_codes, const float *v, float *dst, int B, int H, int Nk, int nbits, int dv,
                    const AdditiveMfmaPlan &p, bool zero_one, hipStream_t st) {
    const int W = nbits / 64;
    const long blocks = (long)B * H * p.groups * p.splits;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_additive_attention: grid too large");
    const dim3 grid((unsigned)blocks), block(p.wb * p.ph * kWave);
#define SA_KTV(DV_, ZO_) ktv_mfma_kernel<DV_, ZO_><<<grid, block, 0, st>>>(k_codes, v, dst, H, Nk, W, p.wb, p.ph, p.splits, p.tokens_per_block)
    switch (dv) {
        case 32: if (zero_one) SA_KTV(32, true); else SA_KTV(32, false); break;
        case 64: if (zero_one) SA_KTV(64, true); else SA_KTV(64, false); break;
        default: if (zero_one) SA_KTV(128, true); else SA_KTV(128, false); break;
    }
#undef SA_KTV
    return check_launch("sa_additive_attention(K^T V)");
}

int launch_qkv_mfma(const uint64_t *q_codes, const float *kv, float *out, int B, int H, int Nq, int nbits, int dv,
                    float scale, bool zero_one, const int32_t *den, float eps, hipStream_t st) {
    const long BH = (long)B * H;
    const int W = nbits / 64;
    bool ok;
    switch (dv) {
        case 32: ok = launch_qkv_dv<32>(W, q_codes, kv, out, BH, H, Nq, scale, zero_one, den, eps, st); break;
        case 64: ok = launch_qkv_dv<64>(W, q_codes, kv, out, BH, H, Nq, scale, zero_one, den, eps, st); break;
        default: ok = launch_qkv_dv<128>(W, q_codes, kv, out, BH, H, Nq, scale, zero_one, den, eps, st); break;
    }
    SA_REQUIRE(ok, SA_ERR_UNSUPPORTED, "sa_additive_attention: unsupported code width for the matrix-core path");
    return check_launch("sa_additive_attention(Q(K^T V))");
}

}  // namespace sa
