// Hashing through the matrix cores, still bit-exact (Sec. 4.1, binary quantisation of Q / K).
//
// The code bit is DEFINED as the sign of the fp32 chain acc = fma(x_k, r_kj, acc), k ascending.
// For almost every (row, bit) that sign is decided long before rounding matters, so the kernel
//   1. computes z~ = x . r^_j on the bf16 matrix cores, r^_j = r_j / |r_j|, with a three-product
//      split (x = xh + xl, r^ = rh + rl, z~ = xh rh + xh rl + xl rh: ~2^-15 relative accuracy),
//   2. keeps sign(z~) wherever |z~| > 2^-13 * |x| (|x| |r^_j| is the Cauchy-Schwarz bound of
//      sum |x_k r^_kj|; the split drops at most 3 * 2^-18 of that sum, the fp32 accumulation of the
//      pre-pass and of the defining chain at most (d + 2) * 2^-24 of it each: 2^-15.4 |x| together
//      at d = 64, so the margin is a factor of five over the worst case), and
//   3. re-runs the defining chain, one (row, bit) per lane, for the rest (about 0.08 % of the bits
//      on Gaussian data at d = 64; every bit if the data is degenerate) and flips the stored bit if
//      needed.  These re-runs are the expensive part (80 uncoalesced loads per bit): a quarter of
//      the kernel's time at a margin of 2^-12, hence the tighter one.
// NaN / Inf / denormal-range sums fail the test in step 2 and take step 3, which is the definition.
//
// Tiles are 32 consecutive rows of the flattened [B*N*H, d] input (one contiguous 32*d*4-byte
// read).  The MFMA computes the TRANSPOSED tile (hash bits down, rows across), so that a lane ends
// up with 16 bits of one row per 32-bit group: signs are packed with two integer operations per
// bit, the margin test is one multiply and one compare per bit against a per-lane threshold, and
// the two half-wavefronts exchange their halves with one shuffle per group.  The hash matrix
// lives in LDS as ready-made bf16 MFMA fragments; wavefronts stride over the tiles and park their
// unsettled bits in LDS lists that one wavefront per workgroup works off at the end.
#include "common.h"

namespace sa {

namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kListCap = 192;                 // unsettled bits parked per wavefront
constexpr float kKeepFactor = 1.565e-8f;      // (2^-13)^2 * 1.05: keep = sqrt(kKeepFactor * |x|^2)
constexpr float kKeepFloor = 1e-37f;          // keep >= ~3e-19: below that the relative error model does not hold

struct RowMap {
    int N, H, W;
    __device__ inline size_t word_index(long row, int col) const {
        const long nh = (long)N * H;
        const long b = row / nh, rem = row - b * nh;
        const long n = rem / H, h = rem - n * H;
        return (((size_t)b * H + h) * N + n) * W + (col >> 6);
    }
};

__device__ inline void split_bf16(float f, __bf16 &hi, __bf16 &lo) {
    hi = (__bf16)f;
    lo = (__bf16)(f - (float)hi);
}

typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

// The same split for a pair (a in the lower half of each dword, b in the upper): one packed conversion per term.
__device__ inline void split_bf16_pair(float a, float b, uint32_t &upper, uint32_t &lower) {
    v2f r = {a, b};
    upper = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, v2bf));
    r[0] -= __builtin_bit_cast(float, upper << 16);
    r[1] -= __builtin_bit_cast(float, upper & 0xFFFF0000u);
    lower = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, v2bf));
}

// Re-runs the defining chain for one parked (row, bit) entry and flips the stored bit where the
// pre-pass had it wrong.
// Up to two tensors of the same shape are hashed by one launch (Q and K of a block).
struct Tensors {
    const float *x0, *x1;
    uint64_t *codes0, *codes1;
};

// RND steps of the chain per round trip of loads.
template <int D, int RND>
__device__ inline void settle_entry(uint64_t e, const Tensors &ts, const float *__restrict__ proj, const RowMap &map,
                                    int nbits) {
    const long row = (long)(e & 0xffffffffu);
    const int col = (int)((e >> 32) & 0xffffu);
    const bool prov = (e >> 48) & 1u;
    const bool second = (e >> 49) & 1u;
    const float *x = second ? ts.x1 : ts.x0;
    uint64_t *codes = second ? ts.codes1 : ts.codes0;
    const float *xr = x + (size_t)row * D;
    const float *pc = proj + col;
    float acc = 0.0f;
    // loads first, then the fmas in their defined order
#pragma unroll 1
    for (int k0 = 0; k0 < D; k0 += RND) {
        float xv[RND], rv[RND];
#pragma unroll
        for (int q = 0; q < RND / 4; ++q) {
            const float4 t4 = *reinterpret_cast<const float4 *>(xr + k0 + 4 * q);
            xv[4 * q] = t4.x; xv[4 * q + 1] = t4.y; xv[4 * q + 2] = t4.z; xv[4 * q + 3] = t4.w;
        }
#pragma unroll
        for (int k = 0; k < RND; ++k) rv[k] = pc[(size_t)(k0 + k) * nbits];
#pragma unroll
        for (int k = 0; k < RND; ++k) acc = __builtin_fmaf(xv[k], rv[k], acc);
    }
    const bool exact = acc >= 0.0f;
    if (exact != prov)
        atomicXor(reinterpret_cast<unsigned long long *>(codes + map.word_index(row, col)), 1ull << (col & 63));
}

// One wavefront's list, worked off 64 entries at a time.  Kept out of line: inside the tile loop it is
// the rare path (degenerate data) and must not cost the loop its registers.
template <int D>
__device__ __attribute__((noinline)) void work_off_list(const uint64_t *list, int cnt, Tensors ts,
                                                        const float *__restrict__ proj, RowMap map, int nbits) {
    const int lane = threadIdx.x & 63;
    __builtin_amdgcn_s_waitcnt(0x0F70);      // the words these bits live in have been stored
    for (int t0 = 0; t0 < cnt; t0 += 64)
        if (t0 + lane < cnt) settle_entry<D, 32>(list[t0 + lane], ts, proj, map, nbits);
}

// D: head dim; G: hash columns handled by one workgroup (blockIdx.y selects the group).
template <int D, int G, int CG>
__global__ __launch_bounds__(256, 2) void binarize_mfma_kernel(Tensors ts, const float *__restrict__ proj, long rows,
                                                               RowMap map, int nbits, long n_tiles, long n_total) {
    constexpr int S = D / 16;      // MFMA steps along k
    constexpr int JT = G / 32;     // 32-bit groups of hash columns
    constexpr int HALF = D / 2;    // k values one lane owns (the other half-wavefront owns the rest)
    constexpr int FRAGS = S * JT * 2 * 64;      // fragments of one group of G columns
    __shared__ __attribute__((aligned(16))) uint4 bfr_s[CG * FRAGS];
    __shared__ uint64_t list_s[4][kListCap];
    __shared__ int cnt_s[4];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i_loc = lane & 31, g = lane >> 5;
    const int c_first = blockIdx.y * (G * CG);  // this workgroup hashes CG groups of G columns from here

    // ---- hash matrix -> normalised bf16 fragments in LDS: fragment (s, jt, hi/lo), lane L holds
    //      r^[k = (L/32)*HALF + s*8 + e][c0 + jt*32 + L%32], e = 0..7.
    //      Thread (column c = tid % G, slice q = tid / G) loads the D / TPC consecutive k of its column
    //      (coalesced across c), which are exactly the elements of STEPS whole fragments.
    constexpr int TPC = 256 / G;           // threads per column
    constexpr int KPT = D / TPC;           // k values per thread
    constexpr int STEPS = KPT / 8;         // fragments (per hi / lo) per thread
    static_assert(KPT % 8 == 0 && HALF % KPT == 0, "a thread's k slice must lie inside one half");
    __shared__ float cn2_s[TPC][G];
#pragma unroll 1
    for (int cg = 0; cg < CG; ++cg) {
        const int c0 = c_first + cg * G;
        const int c = tid % G, qs = tid / G;
        const int k_first = qs * KPT;
        const int fg = k_first / HALF, s_first = (k_first % HALF) / 8;
        const int jt = c / 32, L = fg * 32 + (c & 31);
        float rv[KPT];
#pragma unroll
        for (int k = 0; k < KPT; ++k) rv[k] = proj[(size_t)(k_first + k) * nbits + c0 + c];
        float s2 = 0.0f;
#pragma unroll
        for (int k = 0; k < KPT; ++k) s2 += rv[k] * rv[k];
        __syncthreads();                         // the previous group's sums have been read
        cn2_s[qs][c] = s2;
        __syncthreads();
        float n2 = 0.0f;
#pragma unroll
        for (int t = 0; t < TPC; ++t) n2 += cn2_s[t][c];
        // a dead, overflowing or non-finite column gets an all-zero r^: z~ = 0 fails the margin test, so
        // every bit of that column is parked and settled by the defining chain
        const float inv_raw = 1.0f / __builtin_sqrtf(n2);
        const bool usable = inv_raw > 0.0f && inv_raw < __builtin_inff();
        const float inv = usable ? inv_raw : 0.0f;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            v8bf vh, vl;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                __bf16 hi, lo;
                split_bf16(usable ? rv[st * 8 + e] * inv : 0.0f, hi, lo);
                vh[e] = hi;
                vl[e] = lo;
            }
            const int s = s_first + st;
            bfr_s[cg * FRAGS + ((s * JT + jt) * 2 + 0) * 64 + L] = __builtin_bit_cast(uint4, vh);
            bfr_s[cg * FRAGS + ((s * JT + jt) * 2 + 1) * 64 + L] = __builtin_bit_cast(uint4, vl);
        }
    }
    __syncthreads();

    int cnt = 0;                   // parked entries of this wavefront (wave-uniform)
    uint64_t *list = list_s[wave];

    // the next tile's rows are in flight while the current tile is multiplied and packed
    // tiles 0 .. n_tiles-1 belong to the first tensor, the next n_tiles to the second
    auto load_tile = [&](long tile, float (&dst)[HALF]) {
        const bool second = tile >= n_tiles;
        const long row_ld = min((second ? tile - n_tiles : tile) * 32 + i_loc, rows - 1);
        const float *xr = (second ? ts.x1 : ts.x0) + (size_t)row_ld * D + g * HALF;
#pragma unroll
        for (int q = 0; q < HALF / 4; ++q) {
            const float4 t4 = *reinterpret_cast<const float4 *>(xr + 4 * q);
            dst[4 * q] = t4.x; dst[4 * q + 1] = t4.y; dst[4 * q + 2] = t4.z; dst[4 * q + 3] = t4.w;
        }
    };
    const long tile_step = (long)gridDim.x * 4;
    float xn[HALF];
    {
        const long first = (long)blockIdx.x * 4 + wave;
        if (first < n_total) load_tile(first, xn);
    }
    for (long tile = (long)blockIdx.x * 4 + wave; tile < n_total; tile += tile_step) {
        const bool second = tile >= n_tiles;
        const long r0 = (second ? tile - n_tiles : tile) * 32;
        uint64_t *codes = second ? ts.codes1 : ts.codes0;
        float xv[HALF];
#pragma unroll
        for (int k = 0; k < HALF; ++k) xv[k] = xn[k];
        if (tile + tile_step < n_total) load_tile(tile + tile_step, xn);
        float nx2 = 0.0f;
#pragma unroll
        for (int k = 0; k < HALF; ++k) nx2 += xv[k] * xv[k];
        nx2 += __shfl_xor(nx2, 32);                                // |x_row|^2, row = r0 + i_loc
        // keep sign(z~) where |z~| > keep = 2^-13 |x| (floored); a non-finite |x|^2 keeps nothing
        const float keep = nx2 < __builtin_inff() ? __builtin_sqrtf(__builtin_fmaxf(kKeepFactor * nx2, kKeepFloor))
                                                  : __builtin_inff();

        // the two bf16 terms of the row, once for all column groups; two elements per conversion
        v8bf xh[S], xl[S];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            uint32_t up[4], lo[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) split_bf16_pair(xv[s * 8 + 2 * e2], xv[s * 8 + 2 * e2 + 1], up[e2], lo[e2]);
            xh[s] = __builtin_bit_cast(v8bf, make_uint4(up[0], up[1], up[2], up[3]));
            xl[s] = __builtin_bit_cast(v8bf, make_uint4(lo[0], lo[1], lo[2], lo[3]));
        }
        const bool row_ok = (r0 + i_loc) < rows;

#pragma unroll 1
        for (int cg = 0; cg < CG; ++cg) {
        const int c0 = c_first + cg * G;
        const uint4 *frag = bfr_s + cg * FRAGS;
        // z~^T: accumulator (jt, r) of lane (i_loc, g) = hash bit jt*32 + 8*(r/4) + 4*g + r%4 of row i_loc
        v16f acc[JT];
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[jt][r] = 0.0f;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            // all fragments of the step first, then the three products term by term, so that successive
            // MFMAs go to different accumulators and none waits for the one before it
            v8bf rh[JT], rl[JT];
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                rh[jt] = __builtin_bit_cast(v8bf, frag[((s * JT + jt) * 2 + 0) * 64 + lane]);
                rl[jt] = __builtin_bit_cast(v8bf, frag[((s * JT + jt) * 2 + 1) * 64 + lane]);
            }
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh[jt], xh[s], acc[jt], 0, 0, 0);
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rl[jt], xh[s], acc[jt], 0, 0, 0);
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rh[jt], xl[s], acc[jt], 0, 0, 0);
            // keep the steps apart: hoisting every fragment read of the tile to the top costs
            // 128 registers and one wavefront of occupancy
            __builtin_amdgcn_sched_barrier(0);
        }

        // provisional bits (sign of z~; -0 is parked anyway) and the unsettled ones, one mask bit per
        // accumulator register, per 32-bit group.  Signs: 16 funnel shifts collect the sign bits, then
        // the four nibbles move to their byte.  Margin: the smallest |z~| of the 16 decides for all of
        // them at once (99.7 % of the groups); only a group with a doubtful element is tested one by one.
        uint32_t bits[JT], park[JT];
        uint32_t any_park = 0;
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) {
            uint32_t neg = 0;                                                 // bit r = sign of register r
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const float z = acc[jt][15 - q];
                neg = __builtin_amdgcn_alignbit(neg, __builtin_bit_cast(uint32_t, z), 31);
            }
            const uint32_t pos_bits = ~neg;
            const uint32_t spread = (pos_bits & 0xFu) | ((pos_bits & 0xF0u) << 4) | ((pos_bits & 0xF00u) << 8) |
                                    ((pos_bits & 0xF000u) << 12);             // register r -> bit 8*(r/4) + r%4
            bits[jt] = spread << (4 * g);
            float smallest = __builtin_fabsf(acc[jt][0]);
#pragma unroll
            for (int r = 1; r < 16; ++r) smallest = __builtin_fminf(smallest, __builtin_fabsf(acc[jt][r]));
            uint32_t pk = 0;
            if (__builtin_amdgcn_ballot_w64(!(smallest > keep)) != 0) {        // wave-uniform
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    pk |= (uint32_t)(!(__builtin_fabsf(acc[jt][r]) > keep)) << (8 * (r >> 2) + (r & 3));
            }
            park[jt] = row_ok ? (pk << (4 * g)) : 0u;
            any_park |= park[jt];
        }
        // the other half-wavefront holds the other 16 bits of each group of the same row
        uint32_t word[JT];
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) word[jt] = bits[jt] | (uint32_t)__shfl_xor((int)bits[jt], 32);
        if (lane < 32 && row_ok) {
            uint32_t *dst = reinterpret_cast<uint32_t *>(codes + map.word_index(r0 + lane, c0));
            if (JT == 4)
                *reinterpret_cast<uint4 *>(dst) = make_uint4(word[0], word[1], word[2], word[3]);
            else
                *reinterpret_cast<uint2 *>(dst) = make_uint2(word[0], word[JT - 1]);
        }

        // park the unsettled bits.  The list may be worked off at any point from here on: this
        // tile's words are on their way to memory and the accumulators are dead.
        while (__ballot(any_park != 0) != 0) {                    // wave-uniform; rarely more than 2 rounds
            int jt = 0;
#pragma unroll
            for (int t = JT - 1; t >= 0; --t) jt = park[t] ? t : jt;
            const bool parked = any_park != 0;
            uint32_t mine = 0;                                    // this lane's first non-empty group
#pragma unroll
            for (int t = 0; t < JT; ++t) mine = (t == jt) ? park[t] : mine;
            const int pos = parked ? __builtin_ctz(mine) : 0;
            const uint64_t pm = __ballot(parked);
            if (cnt + 64 > kListCap) {
                work_off_list<D>(list, cnt, ts, proj, map, nbits);
                cnt = 0;
            }
            if (parked) {
                const int slot = cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(pm >> 32),
                                                                 __builtin_amdgcn_mbcnt_lo((uint32_t)pm, 0u));
                uint32_t b = 0;
#pragma unroll
                for (int t = 0; t < JT; ++t) b = (t == jt) ? bits[t] : b;
                list[slot] = (uint64_t)(uint32_t)(r0 + i_loc) | ((uint64_t)(c0 + jt * 32 + pos) << 32) |
                             ((uint64_t)((b >> pos) & 1u) << 48) | ((uint64_t)second << 49);
                const uint32_t cleared = mine & (mine - 1u);
#pragma unroll
                for (int t = 0; t < JT; ++t) park[t] = (t == jt) ? cleared : park[t];
                any_park = 0;
#pragma unroll
                for (int t = 0; t < JT; ++t) any_park |= park[t];
            }
            cnt += __builtin_popcountll(pm);
        }
        }   // column groups
    }

    // The four wavefronts' leftovers are pooled and worked off 64 entries per pass, pass p by wavefront
    // p % 4: the cost of a pass is the latency of its uncoalesced loads, so full passes side by side
    // beat both four nearly empty ones and a queue of full ones on one wavefront.
    __builtin_amdgcn_s_waitcnt(0x0F70);          // this wavefront's words have been stored
    if (lane == 0) cnt_s[wave] = cnt;
    __syncthreads();
    {
        const int n0 = cnt_s[0], n1 = n0 + cnt_s[1], n2 = n1 + cnt_s[2], n3 = n2 + cnt_s[3];
        for (int t0 = wave * 64; t0 < n3; t0 += 256) {
            const int t = t0 + lane;
            if (t < n3) {
                const int w = (t >= n0) + (t >= n1) + (t >= n2);
                const int base = w == 0 ? 0 : (w == 1 ? n0 : (w == 2 ? n1 : n2));
                settle_entry<D, (D <= 64 ? D : 32)>(list_s[w][t - base], ts, proj, map, nbits);   // the tile loop's registers are free now
            }
        }
    }
}

}  // namespace

bool binarize_mfma_supported(int d, int nbits) {
    return (d == 32 || d == 64 || d == 128) && nbits % 64 == 0;
}

template <int D, int G, int CG>
int launch_one(const Tensors &ts, int count, const float *proj, long rows, int N, int H, int nbits, hipStream_t st) {
    const long n_tiles = (rows + 31) / 32;
    const long n_total = n_tiles * count;
    // about two workgroups of 4 wavefronts per CU (what the registers allow), every wavefront the
    // same number of tiles
    const long tiles_per_wave = (n_total + 4 * 512 - 1) / (4 * 512);
    const long blocks = (n_total + 4 * tiles_per_wave - 1) / (4 * tiles_per_wave);
    const dim3 grid((unsigned)blocks, (unsigned)(nbits / (G * CG)));
    RowMap map{N, H, nbits / 64};
    binarize_mfma_kernel<D, G, CG><<<grid, dim3(256), 0, st>>>(ts, proj, rows, map, nbits, n_tiles, n_total);
    return check_launch("sa_binarize(mfma)");
}

// x1 / codes1 may be null: one tensor.  Column groups: 128 columns per pass of the matrix cores (64
// for d = 128 or when nbits is not a multiple of 128); when nbits is a multiple of 256 a workgroup
// takes two groups per row tile, so the rows are read and split once for both.
int launch_binarize_mfma(const float *x0, const float *x1, const float *proj, uint64_t *codes0, uint64_t *codes1,
                         long rows, int N, int H, int d, int nbits, hipStream_t st) {
    const Tensors ts{x0, x1, codes0, codes1};
    const int count = x1 ? 2 : 1;
    const bool g128 = (nbits % 128 == 0), two = (nbits % 256 == 0);
    switch (d) {
        case 32:
            return two    ? launch_one<32, 128, 2>(ts, count, proj, rows, N, H, nbits, st)
                   : g128 ? launch_one<32, 128, 1>(ts, count, proj, rows, N, H, nbits, st)
                          : launch_one<32, 64, 1>(ts, count, proj, rows, N, H, nbits, st);
        case 64:
            return two    ? launch_one<64, 128, 2>(ts, count, proj, rows, N, H, nbits, st)
                   : g128 ? launch_one<64, 128, 1>(ts, count, proj, rows, N, H, nbits, st)
                          : launch_one<64, 64, 1>(ts, count, proj, rows, N, H, nbits, st);
        default:
            return g128 ? launch_one<128, 64, 2>(ts, count, proj, rows, N, H, nbits, st)
                        : launch_one<128, 64, 1>(ts, count, proj, rows, N, H, nbits, st);
    }
}

}  // namespace sa
