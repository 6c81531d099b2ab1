// sa_hamming_attention: quadratic attention on binary codes (Eq. 1 with Q K^T
// replaced by the Hamming similarity S = nbits - 2 * popcount(q xor k) of the
// codes; V stays fp32, Sec. 4.1).
//
// The scores are integer work for the vector ALU (XOR + popcount).  A score takes one of
// nbits + 1 values, so the softmax numerators p = exp2(-|c2| * t), t = |dist - dist_ref|,
// come from a table in LDS that is built once per workgroup; each entry holds p in fp32
// (for the row sum) and p split into two bf16 terms, p ~ ph + pl (each rounded to nearest).
// The second MatMul P * V is the dense contraction of this kernel and runs on the bf16
// matrix cores (v_mfma_f32_32x32x16_bf16) as three products with fp32 accumulation,
//     P * V ~ ph * vh + ph * vl + pl * vh,        v ~ vh + vl likewise,
// which drops only terms below 2^-17 of each p * v (the output tolerance is 1e-4).  The products
// are issued transposed, O^T = V^T * P^T: the P operand of one MFMA is 8 numerators per lane -
// query (lane % 32), keys k0 + 8 * (lane / 32) .. + 7 - exactly the pairs whose distances the lane
// has just computed, so P never exists in memory, and the accumulators end up holding, per lane,
// whole 16-byte pieces of that lane's own query row (no transposes, no staging in the epilogue).
// A workgroup owns one (batch, head) and up to 256 queries (one 32-query tile per wavefront); key
// codes and V rows are staged through LDS in chunks of 128 keys, V transposed and split into its
// two bf16 planes, so that a V operand (8 consecutive keys of one column) is one 16-byte read.
// Row sums ride along in the lanes and meet in the epilogue.
//
// softmax(scale*S)_j = exp2(c2 * (dist_j - dist_ref)) / sum, c2 = -2*scale*log2(e),
// dist_ref = the distance of the largest score.  When scale >= 0 and the exponent
// range cannot underflow, dist_ref = 0 (no first pass); otherwise a first pass over
// the key codes finds it per query.
#include <type_traits>

#include "common.h"
#include "gemm_common.h"

namespace {

using sa::kWave;

constexpr int kMaxWaves = 8;       // 32-query tiles per workgroup
constexpr int kKeyChunk = 128;     // keys staged in LDS at a time
constexpr int kStageBatch = 2;     // V staging tasks (8 loads each) whose loads a thread keeps in flight together
constexpr int kVtStride = kKeyChunk + 8;   // bf16 elements per transposed V row: 272 bytes, so that the
                                           // 16-byte reads of 16 consecutive columns hit 16 bank groups

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int W>
__device__ inline int distance(const uint64_t (&q)[W], const uint64_t *k) {
    int dist = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) dist += __builtin_popcountll(q[w] ^ k[w]);
    return dist;
}

// Round-to-nearest-even bf16 of a finite float, as the upper 16 bits.
__device__ inline uint32_t bf16_bits(float f) {
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// f ~ hi + lo, two bf16 terms; returns (hi << 16) | lo.
__device__ inline uint32_t split_bf16(float f) {
    const uint32_t hi = bf16_bits(f);
    const float rest = f - __builtin_bit_cast(float, hi << 16);
    return (hi << 16) | bf16_bits(rest);
}

typedef _Float16 v4h __attribute__((ext_vector_type(4)));

typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

// The two bf16 terms of a pair of values, as the dwords the transposed planes store: upper terms
// (a in the lower half, b in the upper half) and lower terms.  One v_cvt_pk_bf16_f32 per plane.
__device__ inline void split_bf16_pair(float a, float b, uint32_t &upper, uint32_t &lower) {
    v2f r = {a, b};
    upper = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, v2bf));
    r[0] -= __builtin_bit_cast(float, upper << 16);
    r[1] -= __builtin_bit_cast(float, upper & 0xFFFF0000u);
    lower = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, v2bf));
}

// A chunk of V rows -> the two transposed bf16 planes in LDS (keys n .. n_pad-1 are zero in both planes: their
// numerators add nothing).  One task = eight consecutive keys of one column: the loads of a wavefront cover
// whole rows of the head (coalesced), and the eight values of a task leave as 16 bytes per plane, at offsets
// whose bank groups differ from lane to lane.  (Two keys x four columns per task, the shape a float4 load
// suggests, puts 16 lanes of a 4-byte write on two banks.)  The loads of PT tasks are issued together.
template <int DV, int STRIDE, int PT>
struct VStage {
    static_assert(STRIDE % 4 == 0, "8-byte pieces of a transposed row must be aligned");
    float x[PT][8];
    // tasks first, first + n_threads, ... (PT of them) of the chunk at key j0
    __device__ inline void load(const float *__restrict__ v, int b, int H, int h, int Nk, int j0, int n, int n_pad, int first,
                                int n_threads) {
        const int n_tasks = (n_pad / 8) * DV;
        const size_t row = (size_t)H * DV;
#pragma unroll
        for (int u = 0; u < PT; ++u) {
            const int t = first + u * n_threads;
            const int col = t % DV, j = 8 * (t / DV);
            const float *vp = v + (((size_t)b * Nk + j0 + j) * H + h) * DV + col;
#pragma unroll
            for (int e = 0; e < 8; ++e) x[u][e] = (t < n_tasks && j + e < n) ? vp[e * row] : 0.0f;
        }
    }
    __device__ inline void store(int n_pad, uint16_t *vth_s, uint16_t *vtl_s, int first, int n_threads) const {
        const int n_tasks = (n_pad / 8) * DV;
#pragma unroll
        for (int u = 0; u < PT; ++u) {
            const int t = first + u * n_threads;
            if (t >= n_tasks) continue;
            const int col = t % DV, j = 8 * (t / DV);
            uint32_t up[4], lo[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) split_bf16_pair(x[u][2 * e2], x[u][2 * e2 + 1], up[e2], lo[e2]);
            const int off = col * STRIDE + j;
            if constexpr (STRIDE % 8 == 0) {
                *reinterpret_cast<uint4 *>(vth_s + off) = make_uint4(up[0], up[1], up[2], up[3]);
                *reinterpret_cast<uint4 *>(vtl_s + off) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            } else {
                *reinterpret_cast<uint2 *>(vth_s + off) = make_uint2(up[0], up[1]);
                *reinterpret_cast<uint2 *>(vth_s + off + 4) = make_uint2(up[2], up[3]);
                *reinterpret_cast<uint2 *>(vtl_s + off) = make_uint2(lo[0], lo[1]);
                *reinterpret_cast<uint2 *>(vtl_s + off + 4) = make_uint2(lo[2], lo[3]);
            }
        }
    }
};

// The whole chunk, loads and stores back to back (kStageBatch tasks per round trip).
template <int DV, int STRIDE>
__device__ inline void stage_v(const float *__restrict__ v, int b, int H, int h, int Nk, int j0, int n, int n_pad,
                               uint16_t *vth_s, uint16_t *vtl_s, int tid, int n_threads) {
    const int n_tasks = (n_pad / 8) * DV;
    for (int base = 0; base < n_tasks; base += n_threads * kStageBatch) {
        VStage<DV, STRIDE, kStageBatch> st;
        st.load(v, b, H, h, Nk, j0, n, n_pad, base + tid, n_threads);
        st.store(n_pad, vth_s, vtl_s, base + tid, n_threads);
    }
}

struct TableEntry {
    uint32_t hl;      // bf16 terms of p: (hi << 16) | lo
    float p;
};

// Epilogue.  The accumulators hold the TRANSPOSED output tile (the P * V products are issued as V^T * P^T):
// register r of accumulator jt in lane (i, kg) is column jt * 32 + 8 * (r / 4) + 4 * kg + r % 4 of query i, so a
// lane owns 16-byte pieces of its own query's row and the row sum it needs is its own plus its partner's (lane
// i + 32, which summed the other keys).  Stored straight from the registers those pieces would reach memory as
// 16- and 32-byte requests, several times as many as the bytes need (measured: 45-48 us against 39-40 us for the
// DeiT-Base shape).  So the wavefront writes 16 queries at a time into `stage`, an area in LDS of its own (16 rows
// of DV floats, row pitch stage_pitch), and reads them back with consecutive lanes on consecutive columns of a
// row: fp32 rows leave as 16 bytes per lane (DV / 4 lanes cover a head's row piece), the int8 codes of the
// activation quantiser as 16 columns per lane, the fp16 rounding as 8 columns per lane.  Only this wavefront
// touches its `stage`, and the LDS operations of a wavefront execute in order: no barrier inside.
template <int DV>
constexpr int stage_pitch() { return DV * 4 + (DV >= 64 ? 16 : 8); }
template <int DV>
constexpr int stage_bytes_per_wave() { return 16 * stage_pitch<DV>(); }

template <int DV>
__device__ inline void write_outputs(v16f (&acc)[DV / 32], float den, uint8_t *stage, float *__restrict__ out,
                                            int8_t *__restrict__ xq, _Float16 *__restrict__ xh, float act_inv_scale, int b,
                                            int h, int H, int Nq, int chunk, int wave, int lane) {
    constexpr int JT = DV / 32;
    constexpr int PITCH = stage_pitch<DV>();
    const int i_loc = lane & 31, kg = lane >> 5;
    den += __shfl_xor(den, 32);
    const float inv = 1.0f / den;
    const int q_tile0 = chunk * (kMaxWaves * 32) + wave * 32;
    const size_t row_elems = (size_t)H * DV;
    const size_t tile_at = (((size_t)b * Nq + q_tile0) * H + h) * DV;      // element (q_tile0, column 0 of the head)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        if ((i_loc >> 4) == half) {
            uint8_t *row = stage + (i_loc & 15) * PITCH;
#pragma unroll
            for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4 *>(row + (jt * 32 + 8 * g + 4 * kg) * 4) =
                        make_float4(acc[jt][4 * g] * inv, acc[jt][4 * g + 1] * inv, acc[jt][4 * g + 2] * inv,
                                    acc[jt][4 * g + 3] * inv);
        }
        const int q_half0 = q_tile0 + 16 * half;
        if (out) {
            constexpr int LPR = DV / 4;                   // lanes per row, 16 bytes each
            constexpr int RPP = 64 / LPR;                 // rows per pass
#pragma unroll
            for (int p = 0; p < 16 / RPP; ++p) {
                const int r = p * RPP + lane / LPR, c = (lane % LPR) * 4;
                const float4 val = *reinterpret_cast<const float4 *>(stage + r * PITCH + c * 4);
                if (q_half0 + r < Nq) *reinterpret_cast<float4 *>(out + tile_at + (size_t)(16 * half + r) * row_elems + c) = val;
            }
        }
        if (xq) {
            constexpr int LPR = DV / 16;                  // lanes per row, 16 columns each
            constexpr int RPP = 64 / LPR;
#pragma unroll
            for (int p = 0; p < (16 + RPP - 1) / RPP; ++p) {
                const int r = p * RPP + lane / LPR, c = (lane % LPR) * 16;
                if (r < 16) {
                    uint32_t w[4];
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        const float4 val = *reinterpret_cast<const float4 *>(stage + r * PITCH + (c + 4 * e4) * 4);
                        w[e4] = sa::requant_byte(val.x * act_inv_scale) | (sa::requant_byte(val.y * act_inv_scale) << 8) |
                                (sa::requant_byte(val.z * act_inv_scale) << 16) | (sa::requant_byte(val.w * act_inv_scale) << 24);
                    }
                    if (q_half0 + r < Nq)
                        *reinterpret_cast<uint4 *>(xq + tile_at + (size_t)(16 * half + r) * row_elems + c) =
                            make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
        if (xh) {
            constexpr int LPR = DV / 8;                   // lanes per row, 8 columns each
            constexpr int RPP = 64 / LPR;
#pragma unroll
            for (int p = 0; p < (16 + RPP - 1) / RPP; ++p) {
                const int r = p * RPP + lane / LPR, c = (lane % LPR) * 8;
                if (r < 16) {
                    const float4 v0 = *reinterpret_cast<const float4 *>(stage + r * PITCH + c * 4);
                    const float4 v1 = *reinterpret_cast<const float4 *>(stage + r * PITCH + (c + 4) * 4);
                    v4h h0, h1;
                    h0[0] = (_Float16)v0.x; h0[1] = (_Float16)v0.y; h0[2] = (_Float16)v0.z; h0[3] = (_Float16)v0.w;
                    h1[0] = (_Float16)v1.x; h1[1] = (_Float16)v1.y; h1[2] = (_Float16)v1.z; h1[3] = (_Float16)v1.w;
                    const uint2 a2 = __builtin_bit_cast(uint2, h0), b2 = __builtin_bit_cast(uint2, h1);
                    if (q_half0 + r < Nq)
                        *reinterpret_cast<uint4 *>(xh + tile_at + (size_t)(16 * half + r) * row_elems + c) =
                            make_uint4(a2.x, a2.y, b2.x, b2.y);
                }
            }
        }
    }
}

template <int DV, int W, bool ROWREF>
__global__ __launch_bounds__(kMaxWaves *kWave) void hamming_mfma_kernel(
    const uint64_t *__restrict__ q_codes, const uint64_t *__restrict__ k_codes, const float *__restrict__ v,
    float *__restrict__ out, int H, int Nq, int Nk, int q_chunks, float c2, int8_t *__restrict__ xq,
    _Float16 *__restrict__ xh, float act_inv_scale) {
    constexpr int JT = DV / 32;
    constexpr int NBITS = W * 64;
    __shared__ __attribute__((aligned(16))) uint64_t kc_s[kKeyChunk * W];
    __shared__ __attribute__((aligned(16))) uint16_t vt_s[2][DV * kVtStride];  // V^T, upper and lower bf16 term; the
    uint16_t *vth_s = vt_s[0], *vtl_s = vt_s[1];                                // epilogue stages the outputs here
    static_assert(sizeof(vt_s) >= kMaxWaves * stage_bytes_per_wave<DV>(), "the planes hold every wavefront's staging rows");
    __shared__ __attribute__((aligned(8))) TableEntry tab_s[NBITS + 1];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_threads = blockDim.x;
    const long bh = blockIdx.x / q_chunks;
    const int chunk = blockIdx.x % q_chunks;
    const int b = (int)(bh / H), h = (int)(bh % H);
    const int i_loc = lane & 31, kg = lane >> 5;
    const int qi = chunk * (kMaxWaves * 32) + wave * 32 + i_loc;      // this lane's query
    const int qi_ld = min(qi, Nq - 1);

    uint64_t q[W];
#pragma unroll
    for (int w = 0; w < W; ++w) q[w] = q_codes[((size_t)bh * Nq + qi_ld) * W + w];
    const uint64_t *kc_g = k_codes + (size_t)bh * Nk * W;

    // numerators by t = |dist - dist_ref|: the exponent is c2 * (dist - dist_ref) = -|c2| * t
    const float c2n = c2 <= 0.0f ? c2 : -c2;
    for (int t = tid; t <= NBITS; t += n_threads) {
        const float pt = __builtin_amdgcn_exp2f(c2n * (float)t);
        tab_s[t].hl = split_bf16(pt);
        tab_s[t].p = pt;
    }

    int dref = 0;
    if (ROWREF) {
        // the distance whose score scale*S is largest: the smallest if scale >= 0 (c2 <= 0)
        int dmin = 1 << 30, dmax = -1;
        for (int j0 = 0; j0 < Nk; j0 += kKeyChunk) {
            const int n = min(kKeyChunk, Nk - j0);
            __syncthreads();
            for (int t = tid; t < n * W; t += n_threads) kc_s[t] = kc_g[(size_t)j0 * W + t];
            __syncthreads();
            for (int j = 0; j < n; ++j) {
                const int dist = distance<W>(q, kc_s + j * W);
                dmin = min(dmin, dist);
                dmax = max(dmax, dist);
            }
        }
        dref = (c2 <= 0.0f) ? dmin : dmax;
    }

    v16f acc[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[jt][r] = 0.0f;
    float den = 0.0f;

    // One step: 16 keys from k0 (8 per half-wavefront).  MASK: keys from n on do not count.
    auto step = [&](int k0, int n, auto mask_c) {
        constexpr bool MASK = decltype(mask_c)::value;
        const int kb = k0 + 8 * kg;                       // this lane's first key
        uint32_t hl[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int t = distance<W>(q, kc_s + (kb + e) * W);
            if (ROWREF) {
                t = (c2 <= 0.0f) ? t - dref : dref - t;
                if (MASK) t = min(max(t, 0), NBITS);       // a padding key may lie beyond the reference
            }
            const TableEntry te = tab_s[t];
            hl[e] = te.hl;
            den += (!MASK || kb + e < n) ? te.p : 0.0f;
        }
        // A operands: element e of the lane is key kb + e
        uint32_t ah[4], al[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            ah[e2] = __builtin_amdgcn_perm(hl[2 * e2 + 1], hl[2 * e2], 0x07060302u);   // upper halves
            al[e2] = __builtin_amdgcn_perm(hl[2 * e2 + 1], hl[2 * e2], 0x05040100u);   // lower halves
        }
        const v8bf ph = __builtin_bit_cast(v8bf, make_uint4(ah[0], ah[1], ah[2], ah[3]));
        const v8bf pl = __builtin_bit_cast(v8bf, make_uint4(al[0], al[1], al[2], al[3]));
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) {
            const int off = (jt * 32 + i_loc) * kVtStride + kb;
            const v8bf vh = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(vth_s + off));
            const v8bf vl = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(vtl_s + off));
            acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vh, ph, acc[jt], 0, 0, 0);
            acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vl, ph, acc[jt], 0, 0, 0);
            acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vh, pl, acc[jt], 0, 0, 0);
        }
    };

    for (int j0 = 0; j0 < Nk; j0 += kKeyChunk) {
        const int n = min(kKeyChunk, Nk - j0);
        const int n_pad = (n + 15) & ~15;
        __syncthreads();                           // the previous chunk has been consumed (and the table is there)
        for (int t = tid; t < n_pad * W; t += n_threads) kc_s[t] = (t < n * W) ? kc_g[(size_t)j0 * W + t] : 0ull;
        stage_v<DV, kVtStride>(v, b, H, h, Nk, j0, n, n_pad, vth_s, vtl_s, tid, n_threads);
        __syncthreads();
        const int n_full = n & ~15;                // whole steps first, then at most one masked step
        for (int k0 = 0; k0 < n_full; k0 += 16) step(k0, n, std::false_type{});
        if (n_full < n) step(n_full, n, std::true_type{});
    }

    __syncthreads();                               // every wavefront is through its steps: the planes become staging rows
    write_outputs<DV>(acc, den, reinterpret_cast<uint8_t *>(&vt_s[0][0]) + wave * stage_bytes_per_wave<DV>(), out, xq, xh,
                             act_inv_scale, b, h, H, Nq, chunk, wave, lane);
}

// ---- the same kernel as a pipeline over several (batch, head, query chunk) units per workgroup ------------
// The kernel above runs its phases one after the other: load V, split it, multiply, store.  With every workgroup
// of a launch resident at once (768 at the DeiT-Base shape, three per CU) the whole chip loads, then computes,
// then stores.  Here a launch has only as many workgroups as fit the chip; each walks over its units
// (u = blockIdx.x, + gridDim.x, ...) and over their 128-key chunks, and the NEXT chunk's V rows and key codes are
// already on their way while the current chunk is multiplied: they arrive through direct global -> LDS loads
// (no registers, no waiting wavefront) as raw fp32 rows, and are split into the two bf16 planes LDS -> LDS at the
// chunk switch.  The output stores of a unit drain while the next unit is computed.  Same arithmetic, same
// order, bit-identical results.  Row reference distances (ROWREF in the kernel above) need all key codes of a
// unit before its first step and keep the kernel above.
//
// One wavefront-wide direct load: lane l's 16 (4) bytes at `src` land at LDS byte lds_base + 16 (4) * l.
__device__ inline void async_load_16(const void *src, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, off\n\t"
        :
        : "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(src)
        : "memory");
}
__device__ inline void async_load_4(const void *src, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dword %1, off\n\t"
        :
        : "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(src)
        : "memory");
}

template <int DV, int W>
__global__ __launch_bounds__(kMaxWaves *kWave, 4) void hamming_pipe_kernel(
    const uint64_t *__restrict__ q_codes, const uint64_t *__restrict__ k_codes, const float *__restrict__ v,
    float *__restrict__ out, int H, int Nq, int Nk, int q_chunks, float c2, int8_t *__restrict__ xq,
    _Float16 *__restrict__ xh, float act_inv_scale, long n_units) {
    constexpr int JT = DV / 32;
    constexpr int NBITS = W * 64;
    constexpr int RPI = 1024 / (DV * 4);           // V rows one wavefront-wide 16-byte load brings
    constexpr int L4 = DV / 4;                     // lanes per V row
    __shared__ __attribute__((aligned(1024))) float raw_s[kKeyChunk * DV];          // the next chunk's V rows as loaded
    __shared__ __attribute__((aligned(1024))) uint64_t kc_s[2][kKeyChunk * W];      // key codes, this chunk's and the next's
    __shared__ __attribute__((aligned(16))) uint16_t vt_s[2][DV * kVtStride];  // V^T, upper and lower bf16 term; the
    uint16_t *vth_s = vt_s[0], *vtl_s = vt_s[1];                                // epilogue stages the outputs here
    static_assert(sizeof(vt_s) >= kMaxWaves * stage_bytes_per_wave<DV>(), "the planes hold every wavefront's staging rows");
    __shared__ __attribute__((aligned(8))) TableEntry tab_s[NBITS + 1];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_threads = blockDim.x, n_waves = n_threads >> 6;
    const int i_loc = lane & 31, kg = lane >> 5;
    const uint32_t raw_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float *)raw_s;
    const uint32_t kc_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint64_t *)&kc_s[0][0];

    // Chunk at key j of unit u -> raw_s and kc_s[buf].  Rows and code bytes past the last key are re-reads of
    // the last valid ones (never used: the conversion zeroes those V rows, the last step masks those keys).
    auto issue_chunk = [&](long u, int j, int buf) {
        const long bh = u / q_chunks;
        const int b = (int)(bh / H), h = (int)(bh % H);
        const int n = min(kKeyChunk, Nk - j);
        const int n_pad = (n + 15) & ~15;
        const int v_instr = (n_pad + RPI - 1) / RPI;
        for (int k = wave; k < v_instr; k += n_waves) {
            const int key = min(k * RPI + lane / L4, n - 1);
            const float *src = v + (((size_t)b * Nk + j + key) * H + h) * DV + (lane % L4) * 4;
            async_load_16(src, raw_base + k * 1024);
        }
        const int code_bytes = n * W * 8, code_instr = (n_pad * W * 8 + 255) / 256;
        const char *cg = reinterpret_cast<const char *>(k_codes + ((size_t)bh * Nk + j) * W);
        for (int k = wave; k < code_instr; k += n_waves) {
            const int off = min(k * 256 + lane * 4, code_bytes - 4);
            async_load_4(cg + off, kc_base + buf * (kKeyChunk * W * 8) + k * 256);
        }
    };
    auto load_query = [&](long u, uint64_t (&dst)[W]) {
        const long bh = u / q_chunks;
        const int chunk = (int)(u % q_chunks);
        const int qi = min(chunk * (kMaxWaves * 32) + wave * 32 + i_loc, Nq - 1);
#pragma unroll
        for (int w = 0; w < W; ++w) dst[w] = q_codes[((size_t)bh * Nq + qi) * W + w];
    };

    long u = blockIdx.x;
    if (u >= n_units) return;
    issue_chunk(u, 0, 0);
    uint64_t q[W], qn[W];
    load_query(u, qn);

    // numerators by distance: the exponent is c2 * dist (no row reference here)
    const float c2n = c2 <= 0.0f ? c2 : -c2;
    for (int t = tid; t <= NBITS; t += n_threads) {
        const float pt = __builtin_amdgcn_exp2f(c2n * (float)t);
        tab_s[t].hl = split_bf16(pt);
        tab_s[t].p = pt;
    }

    v16f acc[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[jt][r] = 0.0f;
    float den = 0.0f;

    // One step: 16 keys from k0 (8 per half-wavefront).  MASK: keys from n on do not count.
    auto step = [&](const uint64_t *kc, int k0, int n, auto mask_c) {
        constexpr bool MASK = decltype(mask_c)::value;
        const int kb = k0 + 8 * kg;                       // this lane's first key
        uint32_t hl[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int t = distance<W>(q, kc + (kb + e) * W);      // padding keys hold arbitrary code bytes: still 0 .. NBITS
            const TableEntry te = tab_s[t];
            hl[e] = te.hl;
            den += (!MASK || kb + e < n) ? te.p : 0.0f;
        }
        uint32_t ah[4], al[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            ah[e2] = __builtin_amdgcn_perm(hl[2 * e2 + 1], hl[2 * e2], 0x07060302u);   // upper halves
            al[e2] = __builtin_amdgcn_perm(hl[2 * e2 + 1], hl[2 * e2], 0x05040100u);   // lower halves
        }
        const v8bf ph = __builtin_bit_cast(v8bf, make_uint4(ah[0], ah[1], ah[2], ah[3]));
        const v8bf pl = __builtin_bit_cast(v8bf, make_uint4(al[0], al[1], al[2], al[3]));
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) {
            const int off = (jt * 32 + i_loc) * kVtStride + kb;
            const v8bf vh = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(vth_s + off));
            const v8bf vl = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(vtl_s + off));
            acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vh, ph, acc[jt], 0, 0, 0);
            acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vl, ph, acc[jt], 0, 0, 0);
            acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vh, pl, acc[jt], 0, 0, 0);
        }
    };

    int j0 = 0, buf = 0;
    for (;;) {
        if (j0 == 0) {
#pragma unroll
            for (int w = 0; w < W; ++w) q[w] = qn[w];
        }
        const int n = min(kKeyChunk, Nk - j0);
        const int n_pad = (n + 15) & ~15;
        __builtin_amdgcn_s_waitcnt(0x0F70);          // this wavefront's direct loads of the chunk have landed
        __syncthreads();                             // ... everyone's; the planes of the previous chunk have been consumed
        // raw rows -> the two transposed bf16 planes; one task = eight consecutive keys of one column (a wavefront
        // reads 64 consecutive floats of a row per instruction, and writes 16 bytes per lane and plane)
        {
            const int n_tasks = (n_pad / 8) * DV;
            for (int t = tid; t < n_tasks; t += n_threads) {
                const int col = t % DV, j = 8 * (t / DV);
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = (j + e < n) ? raw_s[(j + e) * DV + col] : 0.0f;
                uint32_t up[4], lo[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) split_bf16_pair(x[2 * e2], x[2 * e2 + 1], up[e2], lo[e2]);
                const int off = col * kVtStride + j;
                *reinterpret_cast<uint4 *>(vth_s + off) = make_uint4(up[0], up[1], up[2], up[3]);
                *reinterpret_cast<uint4 *>(vtl_s + off) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            }
        }
        __syncthreads();                             // planes ready; raw_s is free again
        long u2 = u;
        int j2 = j0 + kKeyChunk;
        if (j2 >= Nk) {
            u2 = u + gridDim.x;
            j2 = 0;
        }
        const bool has_next = u2 < n_units;
        if (has_next) {
            issue_chunk(u2, j2, buf ^ 1);
            if (j2 == 0) load_query(u2, qn);
        }
        const uint64_t *kc = kc_s[buf];
        const int n_full = n & ~15;                  // whole steps first, then at most one masked step
        for (int k0 = 0; k0 < n_full; k0 += 16) step(kc, k0, n, std::false_type{});
        if (n_full < n) step(kc, n_full, n, std::true_type{});
        if (j2 == 0) {                               // last chunk of the unit
            const long bh = u / q_chunks;
            __syncthreads();                         // every wavefront is through its steps: the planes become staging rows
            write_outputs<DV>(acc, den, reinterpret_cast<uint8_t *>(&vt_s[0][0]) + wave * stage_bytes_per_wave<DV>(), out,
                                     xq, xh, act_inv_scale, (int)(bh / H), (int)(bh % H), H, Nq, (int)(u % q_chunks), wave,
                                     lane);
#pragma unroll
            for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[jt][r] = 0.0f;
            den = 0.0f;
        }
        if (!has_next) break;
        u = u2;
        j0 = j2;
        buf ^= 1;
    }
}

// ---- the same attention with the scores on the matrix cores as well ------------------------------
// For +-1 codes the Hamming similarity nbits - 2 popcount(q xor k) IS the dot product of the two
// sign vectors, an exact small integer in fp32: v_mfma_f32_32x32x16_bf16 on the codes expanded to
// +-1.0 gives a 32-key x 32-query tile of scores for 8 (nbits = 128) MFMAs, against ~9 vector
// operations per pair for XOR + popcount.  The tile is computed transposed (keys down, queries
// across), so that a lane ends up with 16 scores of ITS query; their table entries are the A operand
// of the P * V products as they stand (the k index of an MFMA may be any fixed permutation of the
// keys as long as the V operand uses the same one: here element e of step t is key
// 16 t + 8 (e / 4) + 4 (lane / 32) + e % 4 of the tile).
template <int DV, int W, bool ROWREF>
__global__ __launch_bounds__(kMaxWaves *kWave) void hamming_mm_kernel(
    const uint64_t *__restrict__ q_codes, const uint64_t *__restrict__ k_codes, const float *__restrict__ v,
    float *__restrict__ out, int H, int Nq, int Nk, int q_chunks, float c2, int8_t *__restrict__ xq,
    _Float16 *__restrict__ xh, float act_inv_scale) {
    constexpr int JT = DV / 32;
    constexpr int NBITS = W * 64;
    constexpr int KS = NBITS / 16;                 // MFMA steps of a score tile
    constexpr int kVtStride8 = kKeyChunk + 4;     // 264-byte V^T rows: the 8-byte operand reads of 32 columns cover the 64 banks once
    constexpr int KSTRIDE = NBITS + 8;             // bf16 elements per key row of signs (16-byte multiple, conflict-free)
    // one pool: the sign rows of the keys, then the two V^T planes; the epilogue stages the outputs from its start
    constexpr int kSignBytes = kKeyChunk * KSTRIDE * 2, kPlaneBytes = DV * kVtStride8 * 2;
    __shared__ __attribute__((aligned(16))) uint8_t pool_s[kSignBytes + 2 * kPlaneBytes];
    uint16_t *ksign_s = reinterpret_cast<uint16_t *>(pool_s);
    uint16_t *vth_s = reinterpret_cast<uint16_t *>(pool_s + kSignBytes);              // V^T, upper bf16 term
    uint16_t *vtl_s = reinterpret_cast<uint16_t *>(pool_s + kSignBytes + kPlaneBytes);   // V^T, lower bf16 term
    static_assert(sizeof(pool_s) >= kMaxWaves * stage_bytes_per_wave<DV>(), "the pool holds every wavefront's staging rows");
    __shared__ __attribute__((aligned(8))) TableEntry tab_s[NBITS + 1];
    __shared__ __attribute__((aligned(16))) uint4 sign_s[256];
    static_assert(kSignBytes >= kKeyChunk * W * 8, "the first pass keeps the raw key codes there");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_threads = blockDim.x;
    const long bh = blockIdx.x / q_chunks;
    const int chunk = blockIdx.x % q_chunks;
    const int b = (int)(bh / H), h = (int)(bh % H);
    const int i_loc = lane & 31, kg = lane >> 5;
    const int qi = chunk * (kMaxWaves * 32) + wave * 32 + i_loc;      // this lane's query
    const int qi_ld = min(qi, Nq - 1);

    uint64_t q[W];
#pragma unroll
    for (int w = 0; w < W; ++w) q[w] = q_codes[((size_t)bh * Nq + qi_ld) * W + w];
    const uint64_t *kc_g = k_codes + (size_t)bh * Nk * W;

    // byte -> its 8 bits as bf16 signs (element e = bit e); numerators by t = |dist - dist_ref|
    for (int t = tid; t < 256; t += n_threads) {
        uint32_t d[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t nl = ((uint32_t)~t >> (2 * e2)) & 1u, nh = ((uint32_t)~t >> (2 * e2 + 1)) & 1u;
            d[e2] = 0x3F803F80u | (nl << 15) | (nh << 31);
        }
        sign_s[t] = make_uint4(d[0], d[1], d[2], d[3]);
    }
    const float c2n = c2 <= 0.0f ? c2 : -c2;
    for (int t = tid; t <= NBITS; t += n_threads) {
        const float pt = __builtin_amdgcn_exp2f(c2n * (float)t);
        tab_s[t].hl = split_bf16(pt);
        tab_s[t].p = pt;
    }

    int dref = 0;
    if (ROWREF) {
        // the distance whose score scale*S is largest: the smallest if scale >= 0 (c2 <= 0)
        uint64_t *kc_s = reinterpret_cast<uint64_t *>(ksign_s);
        int dmin = 1 << 30, dmax = -1;
        for (int j0 = 0; j0 < Nk; j0 += kKeyChunk) {
            const int n = min(kKeyChunk, Nk - j0);
            __syncthreads();
            for (int t = tid; t < n * W; t += n_threads) kc_s[t] = kc_g[(size_t)j0 * W + t];
            __syncthreads();
            for (int j = 0; j < n; ++j) {
                const int dist = distance<W>(q, kc_s + j * W);
                dmin = min(dmin, dist);
                dmax = max(dmax, dist);
            }
        }
        dref = (c2 <= 0.0f) ? dmin : dmax;
    }
    __syncthreads();                               // the sign table is there (and the first pass is over)

    // this lane's query as the B operand of the score tiles: bits 16 ks + 8 kg .. + 7 per step
    v8bf qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const uint64_t wd = q[ks / 4];
        const uint32_t half = (ks & 2) ? (uint32_t)(wd >> 32) : (uint32_t)wd;
        qf[ks] = __builtin_bit_cast(v8bf, sign_s[__builtin_amdgcn_ubfe(half, 16 * (ks & 1) + 8 * kg, 8)]);
    }
    // byte offset into the table from a score S: 8 t, t = |dist - dref|, dist = (NBITS - S) / 2
    const float off_slope = (c2 <= 0.0f) ? -4.0f : 4.0f;
    const float off_base = (c2 <= 0.0f) ? (float)(4 * NBITS - 8 * dref) : (float)(8 * dref - 4 * NBITS);

    v16f acc[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[jt][r] = 0.0f;
    float den = 0.0f;

    // One step: 32 keys from k0.  MASK: keys from n on do not count.
    auto step = [&](int k0, int n, auto mask_c) {
        constexpr bool MASK = decltype(mask_c)::value;
        v16f sc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = 0.0f;
        const uint16_t *kp = ksign_s + (k0 + i_loc) * KSTRIDE + 8 * kg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const v8bf kf = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(kp + 16 * ks));
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sc, 0, 0, 0);
        }
        // register r: key k0 + 8 (r / 4) + 4 kg + r % 4 against this lane's query
        uint32_t hl[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float fo = __builtin_fmaf(sc[r], off_slope, off_base);
            if (MASK) fo = __builtin_fminf(__builtin_fmaxf(fo, 0.0f), (float)(8 * NBITS));   // padding keys
            const TableEntry te = *reinterpret_cast<const TableEntry *>(reinterpret_cast<const char *>(tab_s) + (uint32_t)fo);
            hl[r] = te.hl;
            den += (!MASK || k0 + 8 * (r >> 2) + 4 * kg + (r & 3) < n) ? te.p : 0.0f;
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            uint32_t ah[4], al[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                ah[e2] = __builtin_amdgcn_perm(hl[8 * t + 2 * e2 + 1], hl[8 * t + 2 * e2], 0x07060302u);   // upper halves
                al[e2] = __builtin_amdgcn_perm(hl[8 * t + 2 * e2 + 1], hl[8 * t + 2 * e2], 0x05040100u);   // lower halves
            }
            const v8bf ph = __builtin_bit_cast(v8bf, make_uint4(ah[0], ah[1], ah[2], ah[3]));
            const v8bf pl = __builtin_bit_cast(v8bf, make_uint4(al[0], al[1], al[2], al[3]));
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                // keys 16 t + 4 kg .. + 3 and 16 t + 8 + 4 kg .. + 3 of the tile, column jt * 32 + i_loc
                const int off = (jt * 32 + i_loc) * kVtStride8 + k0 + 16 * t + 4 * kg;
                const uint2 h0 = *reinterpret_cast<const uint2 *>(vth_s + off), h1 = *reinterpret_cast<const uint2 *>(vth_s + off + 8);
                const uint2 l0 = *reinterpret_cast<const uint2 *>(vtl_s + off), l1 = *reinterpret_cast<const uint2 *>(vtl_s + off + 8);
                const v8bf vh = __builtin_bit_cast(v8bf, make_uint4(h0.x, h0.y, h1.x, h1.y));
                const v8bf vl = __builtin_bit_cast(v8bf, make_uint4(l0.x, l0.y, l1.x, l1.y));
                acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vh, ph, acc[jt], 0, 0, 0);
                acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vl, ph, acc[jt], 0, 0, 0);
                acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vh, pl, acc[jt], 0, 0, 0);
            }
        }
    };

    for (int j0 = 0; j0 < Nk; j0 += kKeyChunk) {
        const int n = min(kKeyChunk, Nk - j0);
        const int n_pad = (n + 31) & ~31;
        __syncthreads();                           // the previous chunk has been consumed
        // key codes -> rows of +-1.0: one task = one 64-bit word of one key (zeros past the last key:
        // a score of 0 is a distance inside the table)
        for (int t = tid; t < n_pad * W; t += n_threads) {
            const int j = t / W, w = t % W;
            const uint64_t wd = (j < n) ? kc_g[(size_t)(j0 + j) * W + w] : 0ull;
            uint4 *dst = reinterpret_cast<uint4 *>(ksign_s + j * KSTRIDE + 64 * w);
#pragma unroll
            for (int bi = 0; bi < 8; ++bi) {
                const uint32_t byte = (uint32_t)(wd >> (8 * bi)) & 0xFFu;
                dst[bi] = (j < n) ? sign_s[byte] : make_uint4(0u, 0u, 0u, 0u);
            }
        }
        // V: as in the kernel above, padded to whole 32-key steps
        stage_v<DV, kVtStride8>(v, b, H, h, Nk, j0, n, n_pad, vth_s, vtl_s, tid, n_threads);
        __syncthreads();
        const int n_full = n & ~31;                // whole steps first, then at most one masked step
        for (int k0 = 0; k0 < n_full; k0 += 32) step(k0, n, std::false_type{});
        if (n_full < n) step(n_full, n, std::true_type{});
    }

    __syncthreads();                               // every wavefront is through its tiles: the pool becomes staging rows
    write_outputs<DV>(acc, den, pool_s + wave * stage_bytes_per_wave<DV>(), out, xq, xh, act_inv_scale, b, h, H, Nq, chunk,
                             wave, lane);
}

// Optional dump of the integer scores, one thread per (query, key) pair.
__global__ __launch_bounds__(256) void hamming_scores_kernel(const uint64_t *__restrict__ q_codes,
                                                             const uint64_t *__restrict__ k_codes,
                                                             int16_t *__restrict__ scores, int Nq,
                                                             int Nk, int W, long total) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx % Nk);
    const long t = idx / Nk;
    const int i = (int)(t % Nq);
    const long bh = t / Nq;
    const uint64_t *q = q_codes + ((size_t)bh * Nq + i) * W;
    const uint64_t *k = k_codes + ((size_t)bh * Nk + j) * W;
    int dist = 0;
    for (int w = 0; w < W; ++w) dist += __builtin_popcountll(q[w] ^ k[w]);
    scores[idx] = (int16_t)(W * 64 - 2 * dist);
}

struct Launch {
    dim3 grid, block;
    hipStream_t st;
    const uint64_t *q, *k;
    const float *v;
    float *out;
    int H, Nq, Nk, q_chunks;
    float c2;
    bool rowref;
    bool mm_scores;         // scores as sign dot products on the matrix cores (else XOR + popcount on the vector ALU)
    bool pipeline;          // several units per workgroup, the next chunk in flight (popcount scores, no row reference)
    long n_units;
    int8_t *xq;
    _Float16 *xh;
    float act_inv_scale;
};

// Workgroups of the pipelined kernel that fit the chip at once (what the LDS and the registers allow per CU,
// times the CUs), asked from the runtime once per block size.
template <int DV, int W>
long pipeline_slots(int threads) {
    static int per_cu[kMaxWaves + 1];          // by wavefronts per workgroup; 0 = not asked yet
    static int n_cu = 0;
    const int waves = threads / kWave;
    if (n_cu == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0) {
            (void)hipGetLastError();
            cus = 256;
        }
        n_cu = cus;
    }
    if (per_cu[waves] == 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, hamming_pipe_kernel<DV, W>, threads, 0) != hipSuccess || occ <= 0) {
            (void)hipGetLastError();
            occ = 1;
        }
        per_cu[waves] = occ;
    }
    return (long)per_cu[waves] * n_cu;
}

template <int DV, int W>
void launch_hamming(const Launch &L) {
    if constexpr (DV <= 64 && W <= 4) {
        if (L.pipeline) {
            const long slots = pipeline_slots<DV, W>((int)L.block.x);
            const long wgs = L.n_units < slots ? L.n_units : slots;
            hamming_pipe_kernel<DV, W><<<dim3((unsigned)wgs), L.block, 0, L.st>>>(L.q, L.k, L.v, L.out, L.H, L.Nq, L.Nk, L.q_chunks,
                                                                                 L.c2, L.xq, L.xh, L.act_inv_scale, L.n_units);
            return;
        }
    }
    // scores on the matrix cores on request, for codes up to 256 bits (the query's sign fragments live in registers)
    if constexpr (W <= 4) {
        if (L.mm_scores) {
            if (L.rowref)
                hamming_mm_kernel<DV, W, true><<<L.grid, L.block, 0, L.st>>>(L.q, L.k, L.v, L.out, L.H, L.Nq, L.Nk, L.q_chunks,
                                                                             L.c2, L.xq, L.xh, L.act_inv_scale);
            else
                hamming_mm_kernel<DV, W, false><<<L.grid, L.block, 0, L.st>>>(L.q, L.k, L.v, L.out, L.H, L.Nq, L.Nk, L.q_chunks,
                                                                              L.c2, L.xq, L.xh, L.act_inv_scale);
            return;
        }
    }
    if (L.rowref)
        hamming_mfma_kernel<DV, W, true><<<L.grid, L.block, 0, L.st>>>(L.q, L.k, L.v, L.out, L.H, L.Nq, L.Nk, L.q_chunks, L.c2,
                                                                       L.xq, L.xh, L.act_inv_scale);
    else
        hamming_mfma_kernel<DV, W, false><<<L.grid, L.block, 0, L.st>>>(L.q, L.k, L.v, L.out, L.H, L.Nq, L.Nk, L.q_chunks, L.c2,
                                                                       L.xq, L.xh, L.act_inv_scale);
}

template <int DV>
int dispatch_w(int W, const Launch &L) {
    switch (W) {
        case 1: launch_hamming<DV, 1>(L); break;
        case 2: launch_hamming<DV, 2>(L); break;
        case 4: launch_hamming<DV, 4>(L); break;
        case 8: launch_hamming<DV, 8>(L); break;
        default:
            return sa::fail(SA_ERR_UNSUPPORTED, "sa_hamming_attention: nbits must be 64, 128, 256 or 512");
    }
    return SA_OK;
}

}  // namespace

extern "C" int sa_hamming_attention(const uint64_t *q_codes, const uint64_t *k_codes, const float *v,
                                    float *out, int B, int H, int Nq, int Nk, int nbits, int dv,
                                    float scale, int16_t *scores_or_null, void *stream) {
    sa::clear_error();
    return sa_hamming_attention_fused(q_codes, k_codes, v, out, B, H, Nq, Nk, nbits, dv, scale, scores_or_null,
                                      nullptr, nullptr, 0.0f, SA_VARIANT_AUTO, stream);
}

extern "C" int sa_hamming_attention_fused(const uint64_t *q_codes, const uint64_t *k_codes, const float *v,
                                          float *out, int B, int H, int Nq, int Nk, int nbits, int dv, float scale,
                                          int16_t *scores_or_null, int8_t *xq_or_null, void *xh_or_null,
                                          float act_inv_scale, int variant, void *stream) {
    sa::clear_error();
    SA_REQUIRE(variant >= 0 && variant <= 2, SA_ERR_INVALID, "sa_hamming_attention: unknown variant %d", variant);
    SA_REQUIRE(B >= 0 && H >= 0 && Nq >= 0 && Nk >= 0 && nbits > 0 && dv > 0, SA_ERR_INVALID,
               "sa_hamming_attention: negative size");
    SA_REQUIRE(nbits % 64 == 0, SA_ERR_SHAPE, "sa_hamming_attention: nbits %d is not a multiple of 64", nbits);
    SA_REQUIRE(nbits <= 16320, SA_ERR_SHAPE, "sa_hamming_attention: scores do not fit int16");
    SA_REQUIRE(dv == 32 || dv == 64 || dv == 128, SA_ERR_UNSUPPORTED,
               "sa_hamming_attention: dv must be 32, 64 or 128 (got %d)", dv);
    SA_REQUIRE(scale == scale && scale - scale == 0.0f, SA_ERR_INVALID, "sa_hamming_attention: scale is not finite");
    SA_REQUIRE((long)B * H < (1L << 20), SA_ERR_SHAPE, "sa_hamming_attention: B*H too large");
    if ((long)B * H == 0 || Nq == 0) return SA_OK;
    SA_REQUIRE(Nk > 0, SA_ERR_SHAPE, "sa_hamming_attention: softmax over zero keys is undefined");
    SA_REQUIRE(q_codes && k_codes && v, SA_ERR_INVALID, "sa_hamming_attention: NULL buffer");
    SA_REQUIRE(out || xq_or_null || xh_or_null, SA_ERR_INVALID, "sa_hamming_attention: no output requested");
    SA_REQUIRE(sa::aligned16(q_codes) && sa::aligned16(k_codes) && sa::aligned16(v) && sa::aligned16(out) &&
                   sa::aligned16(scores_or_null) && sa::aligned16(xq_or_null) && sa::aligned16(xh_or_null),
               SA_ERR_ALIGN, "sa_hamming_attention: pointers must be 16-byte aligned");
    hipStream_t st = sa::as_stream(stream);
    const int W = nbits / 64;
    const long BH = (long)B * H;
    const int q_per_block = kMaxWaves * 32;
    const int q_chunks = (Nq + q_per_block - 1) / q_per_block;
    const int waves = Nq >= q_per_block ? kMaxWaves : (Nq + 31) / 32;   // uniform per launch
    const long blocks = BH * q_chunks;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "sa_hamming_attention: grid too large");
    Launch L;
    L.grid = dim3((unsigned)blocks);
    L.block = dim3(q_chunks > 1 ? kMaxWaves * kWave : waves * kWave);
    L.st = st;
    L.q = q_codes; L.k = k_codes; L.v = v; L.out = out;
    L.H = H; L.Nq = Nq; L.Nk = Nk; L.q_chunks = q_chunks;
    L.xq = xq_or_null;
    L.xh = static_cast<_Float16 *>(xh_or_null);
    L.act_inv_scale = act_inv_scale;
    L.c2 = -2.0f * scale * 1.4426950408889634f;
    // exp2 of c2*dist stays a normal float for every possible distance -> no row reference needed
    L.rowref = !(scale >= 0.0f && -L.c2 * (float)nbits <= 100.0f);
    // measured at the DeiT-Base shape: 38 us with popcount scores, 44 us with matrix-core scores (more LDS
    // traffic and MFMA time than the vector work it saves), so AUTO keeps the popcount
    L.mm_scores = (variant == SA_VARIANT_MFMA);
    // AUTO: the pipelined popcount kernel where it is built (dv <= 64, nbits <= 256, no row reference)
    L.pipeline = variant == SA_VARIANT_AUTO && !L.rowref && dv <= 64 && W <= 4;
    L.n_units = blocks;
    SA_REQUIRE(variant != SA_VARIANT_MFMA || W <= 4, SA_ERR_UNSUPPORTED,
               "sa_hamming_attention: scores on the matrix cores need nbits <= 256 (got %d)", nbits);
    int rc;
    switch (dv) {
        case 32: rc = dispatch_w<32>(W, L); break;
        case 64: rc = dispatch_w<64>(W, L); break;
        default: rc = dispatch_w<128>(W, L); break;
    }
    if (rc != SA_OK) return rc;
    rc = sa::check_launch("sa_hamming_attention");
    if (rc != SA_OK) return rc;
    if (scores_or_null != nullptr) {
        const long total = BH * Nq * Nk;
        const long sb = (total + 255) / 256;
        SA_REQUIRE(sb < (1L << 31), SA_ERR_SHAPE, "sa_hamming_attention: score dump too large");
        hamming_scores_kernel<<<dim3((unsigned)sb), dim3(256), 0, st>>>(q_codes, k_codes, scores_or_null,
                                                                         Nq, Nk, W, total);
        return sa::check_launch("sa_hamming_attention(scores)");
    }
    return SA_OK;
}
