// Tiled "NT" matrix-core GEMM shared by the Shift expert (int8 x two int8 weight planes,
// int32 accumulate) and the Mult expert (fp16 x fp16, fp32 accumulate):
//     C[m, n] = sum_p sum_k A[m, k] * B_p[n, k]
//
// Workgroup tile BM x BN, four wavefronts in a 2 x 2 grid, each owning (BM/2) x (BN/2) as
// 32x32 MFMA tiles.  K advances SB bytes (64 or 128) per stage through a ring of NS (2 to 4) LDS
// stage buffers that is filled by direct global->LDS loads (no register staging): while stage s
// is multiplied out of one buffer, the loads of the following stages are in flight into the
// others; one barrier per stage; the LDS fragment reads run one 32-byte step ahead of the MFMAs
// that consume them, and the loads of a stage are spread between the MFMAs of LS steps.  A direct
// load writes 1 KiB of consecutive LDS per wavefront instruction, so LDS rows cannot be padded;
// instead the 16-byte chunks of a row are XOR-swizzled with the row number (the lane chooses
// which global chunk it fetches), which makes the 16-byte fragment reads of any 16 consecutive
// rows hit 16 different bank groups.
//
// The loads are issued from inline assembly: the kernel orders them by hand (one vmcnt wait and
// one barrier per stage), and the compiler must not serialise the reads of the current buffer
// behind the loads in flight into the other ones.  The K loop is written out in five pieces
// (first stage, steady state, the stage after which no load is left to issue, the stages that
// only drain, the last stage) so that the steady state holds no branch around a load and no
// branch join in front of its MFMAs.
//
// Outputs leave through LDS, 64 rows per pass, so that every lane stores 16 bytes of one row
// (a scattered destination row index and its gate are then fetched once per 16 bytes).
#pragma once

#include <type_traits>
#include <utility>

#include "common.h"
#include "gemm_common.h"

namespace sa {

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), unrolled at compile time.
template <int... I, class F>
__device__ inline void static_for_impl(std::integer_sequence<int, I...>, F &&f) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ inline void static_for(F &&f) {
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));
typedef _Float16 v8h_t __attribute__((ext_vector_type(8)));
typedef float v16f_t __attribute__((ext_vector_type(16)));

struct I8Traits {
    typedef v16i_t Acc;
    static constexpr int kPlanes = 2;
    static constexpr int kElemBytes = 1;
    __device__ static inline Acc mma(const uint4 &a, const uint4 &b, Acc c) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(v4i_t, a), __builtin_bit_cast(v4i_t, b), c,
                                                     0, 0, 0);
    }
};

struct F16Traits {
    typedef v16f_t Acc;
    static constexpr int kPlanes = 1;
    static constexpr int kElemBytes = 2;
    __device__ static inline Acc mma(const uint4 &a, const uint4 &b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h_t, a), __builtin_bit_cast(v8h_t, b), c,
                                                      0, 0, 0);
    }
};

// What the kernel needs to know about its operands.
struct GemmArgs {
    const void *a;          // [rows, K] elements, row-major
    const void *b[2];       // planes, each [N, K] elements, row-major
    RowSel sel;             // which rows of A / of the scattered output
    bool gather_a;          // A rows are sel.rows[m] (else compact m)
    int K, N;               // K: extent of the contraction, a whole number of 64-byte stages; row length of the B planes
    int col_groups = 1;     // 1, 2, 4 or 8: set by the launcher
    // A rows may be shorter than K (int8 only, 64-byte stages): a_valid elements, a multiple of 16 bytes, at a row
    // pitch of a_ld elements; 0 = K.  The B planes must then hold zeros from a_valid on: the kernel multiplies
    // those zeros with bytes it re-reads from inside the row, so it never reads past a row's end.
    int a_ld = 0, a_valid = 0;
};

// Physical 16-byte chunk of logical chunk c in LDS row r, for rows of CPR chunks.
template <int CPR>
__device__ inline int swizzle(int r, int c) {
    return c ^ ((r / (16 / CPR)) & (CPR - 1));
}

// One wavefront-wide direct load: lane l's 16 bytes at `src` land at LDS byte lds_base + 16 * l
// (lds_base is the same in every lane).
__device__ inline void load_to_lds_16(const void *src, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, off\n\t"
        :
        : "s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(src)
        : "memory");
}

// A Store type says how accumulators become output rows:
//   static constexpr int  kBytes      : bytes per output element (1, 2 or 4)
//   static constexpr int  kTableBytes : 0, or 256 for a byte table that is copied into LDS
//   static constexpr bool kScatter    : output row of tile row m is sel.rows[m] (else m)
//   uint32_t convert(acc, int n, const uint8_t *lds_table) const : the element's bits for column n
//   void *out : [rows, N] elements;  const void *table;  const float *gate : null, or a factor per
//       destination row that multiplies fp32 outputs (kScatter && kBytes == 4 only);  bool accumulate :
//       (same case) the product is added to what the destination holds, as fma(gate, value, old)
//   static constexpr bool kSignCodes  : tiles left of column code_cols leave as packed sign bits instead
//       (bit = acc >= 0, 64 columns = one word): uint64_t *codes[2] (column block 0 / 1 of width part_width,
//       laid out [batch, head, token, word]), int head_dim (64 or 128), tokens (per batch element), heads
//   static constexpr bool kLinear     : fp32 outputs leave as fma(value, scale, residual[m, n]) into
//       column blocks: float *parts[3], int part_width (a multiple of 4), const float *residual, float scale
// Wait until at most N of this wavefront's vector-memory loads are still in flight (loads
// complete in issue order, so the oldest ones are the ones that have landed).
template <int N>
__device__ inline void wait_loads_in_flight() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

template <class T, int BM, int BN, int SB, int NS, int LS, int OCC, class Store>
__global__ __launch_bounds__(256, OCC) void gemm_nt_kernel(GemmArgs g, Store store) {
    constexpr int kStageBytes = SB;                     // bytes of K per stage and row
    constexpr int kChunksPerRow = SB / 16;              // 16-byte chunks per LDS row
    constexpr int KK = SB / 32;                         // 32-byte MFMA steps per stage
    static_assert(SB == 64 || SB == 128, "stage rows of 64 or 128 bytes");
    constexpr int NP = T::kPlanes;
    constexpr int MI = BM / 64, NJ = BN / 64;           // 32x32 tiles per wavefront
    constexpr int A_BYTES = BM * kStageBytes, B_BYTES = BN * kStageBytes;
    constexpr int STAGE = A_BYTES + NP * B_BYTES;
    constexpr int ROWS_PER_INSTR = 1024 / kStageBytes;  // LDS rows one wavefront load fills
    constexpr int A_INSTR = BM / ROWS_PER_INSTR / 4;    // loads per wavefront and stage
    constexpr int B_INSTR = BN / ROWS_PER_INSTR / 4;
    constexpr int ES = Store::kBytes;
    constexpr int SLAB_BYTES = 64 * BN * ES;            // epilogue staging: one 32-row slab per wavefront row
    constexpr int EPI_BYTES = SLAB_BYTES + Store::kTableBytes;
    constexpr int LOADS = A_INSTR + NP * B_INSTR;       // direct loads per wavefront and stage
    constexpr int LDS_BYTES = NS * STAGE > EPI_BYTES ? NS * STAGE : EPI_BYTES;
    static_assert(NS >= 2 && NS <= 4, "ring of two to four stages");
    static_assert(LDS_BYTES * OCC <= 160 * 1024, "OCC workgroups of this tile do not fit the LDS of a CU");
    __shared__ __attribute__((aligned(1024))) uint8_t lds[LDS_BYTES];

    const int32_t *rows;
    long n_rows;
    resolve_rows(g.sel, rows, n_rows);
    // Workgroups are handed to the 8 XCDs round-robin by their linear id, and each XCD has its own
    // 4 MiB L2.  The 8 XCDs form a (8 / col_groups) x col_groups grid over the output: an XCD owns
    // every (8 / col_groups)-th row tile and every col_groups-th column tile, and walks them row
    // tile by row tile.  Its share of the B planes (chosen by the host to fit the L2) stays
    // resident, and each row tile of A is fetched by col_groups L2s only.
    const int col_tiles = (g.N + BN - 1) / BN;
    const int cg = g.col_groups, rg = 8 / cg;
    const int cols_per_group = (col_tiles + cg - 1) / cg;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const long row_tile = (long)(slot / cols_per_group) * rg + xcd / cg;
    const int col_tile = (slot % cols_per_group) * cg + xcd % cg;
    const long m0 = row_tile * BM;
    if (m0 >= n_rows || col_tile >= col_tiles) return;
    const int n0 = col_tile * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
    const int N = g.N;
    const size_t row_bytes = (size_t)g.K * T::kElemBytes;
    const size_t a_row_bytes = (size_t)(g.a_ld > 0 ? g.a_ld : g.K) * T::kElemBytes;
    const int a_valid_bytes = (g.a_valid > 0 ? g.a_valid : g.K) * T::kElemBytes;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;

    // ---- what each lane fetches.  Wavefront w issues load i for LDS rows
    //      (w * X_INSTR + i) * ROWS_PER_INSTR + lane / kChunksPerRow, physical chunk lane % kChunksPerRow.
    //      Rows past the end are clamped to the last valid row (computed, never stored).
    const uint8_t *a_src[A_INSTR];
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i) {
        const int r = (wave * A_INSTR + i) * ROWS_PER_INSTR + lane / kChunksPerRow;
        const int c = swizzle<kChunksPerRow>(r, lane % kChunksPerRow);
        long m = m0 + r;
        m = m < n_rows ? m : n_rows - 1;
        const long src = (g.gather_a && rows) ? (long)rows[m] : m;
        a_src[i] = static_cast<const uint8_t *>(g.a) + (size_t)src * a_row_bytes + c * 16;
    }
    // The furthest stage offset at which this lane's chunk still lies inside an A row (64-byte stages: every load of
    // a lane has the same physical chunk, rows 16 apart swizzle alike).  Beyond it the lane re-reads the row's last
    // 16 bytes; with whole rows (a_valid == K) no stage offset gets that far.
    int a_klim = 0;
    if constexpr (SB == 64)
        a_klim = a_valid_bytes - 16 - swizzle<kChunksPerRow>(lane / kChunksPerRow, lane % kChunksPerRow) * 16;
    const uint8_t *b_src[NP][B_INSTR];
#pragma unroll
    for (int i = 0; i < B_INSTR; ++i) {
        const int r = (wave * B_INSTR + i) * ROWS_PER_INSTR + lane / kChunksPerRow;
        const int c = swizzle<kChunksPerRow>(r, lane % kChunksPerRow);
        const int n = min(n0 + r, N - 1);
#pragma unroll
        for (int p = 0; p < NP; ++p)
            b_src[p][i] = static_cast<const uint8_t *>(g.b[p]) + (size_t)n * row_bytes + c * 16;
    }

    // Direct load number q (0 .. LOADS-1) of a stage: A rows first, then the B planes.
    auto issue_load = [&](int q, int buf, int kbyte) {
        const uint32_t base = lds_base + buf * STAGE;
        if (q < A_INSTR) {
            load_to_lds_16(a_src[q] + (SB == 64 ? min(kbyte, a_klim) : kbyte), base + (wave * A_INSTR + q) * 1024);
        } else {
            const int p = (q - A_INSTR) / B_INSTR, i = (q - A_INSTR) % B_INSTR;
            load_to_lds_16(b_src[p][i] + kbyte, base + A_BYTES + p * B_BYTES + (wave * B_INSTR + i) * 1024);
        }
    };
    auto issue_stage = [&](int buf, int kbyte) {
#pragma unroll
        for (int q = 0; q < LOADS; ++q) issue_load(q, buf, kbyte);
    };

    typename T::Acc acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // fragment read offsets (bytes inside a tile) for the 32-byte steps of a stage.  The swizzle of a row depends
    // on the row number modulo 16 only, so tile i of a wavefront reads at the offset of its tile 0 plus 32 rows * i.
    const int fr = lane & 31, fg = lane >> 5;
    int a_rd[KK], b_rd[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        a_rd[kk] = (wm + fr) * kStageBytes + swizzle<kChunksPerRow>(wm + fr, 2 * kk + fg) * 16;
        b_rd[kk] = (wn + fr) * kStageBytes + swizzle<kChunksPerRow>(wn + fr, 2 * kk + fg) * 16;
    }

    auto read_frags = [&](const uint8_t *A, int kk, uint4 (&af)[MI], uint4 (&bf)[NP][NJ]) {
        const uint8_t *B = A + A_BYTES;
#pragma unroll
        for (int i = 0; i < MI; ++i) af[i] = *reinterpret_cast<const uint4 *>(A + a_rd[kk] + i * 32 * kStageBytes);
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                bf[p][j] = *reinterpret_cast<const uint4 *>(B + p * B_BYTES + b_rd[kk] + j * 32 * kStageBytes);
    };
    // One 32-byte step of MFMAs.  When phase >= 0, the direct loads [phase * LPS, (phase+1) * LPS)
    // of the stage at byte kbyte are issued into ring slot `slot`, evenly spaced between the MFMAs:
    // a wavefront that issues its loads back to back stalls on the full vector-memory queue
    // (about 1 KiB per 16 cycles and CU) and leaves its matrix core idle meanwhile.
    constexpr int MFMAS = NP * MI * NJ;
    constexpr int LPS = (LOADS + LS - 1) / LS;          // loads per step
    auto multiply = [&](const uint4 (&af)[MI], const uint4 (&bf)[NP][NJ], auto phase_c, auto more_c, bool more, int slot, int kbyte) {
        constexpr int phase = decltype(phase_c)::value;
        constexpr int MORE = decltype(more_c)::value;      // 1: always, 0: never, -1: `more` decides
        static_for<MFMAS>([&](auto m_c) {
            constexpr int m = decltype(m_c)::value;             // MFMAs issued before this one
            constexpr int p = m / (MI * NJ), i = m / NJ % MI, j = m % NJ;
            acc[i][j] = T::mma(af[i], bf[p][j], acc[i][j]);
            // loads [m * LPS / MFMAS, (m + 1) * LPS / MFMAS) of this step's share follow MFMA m
            if constexpr (phase >= 0) {
                constexpr int q0 = m * LPS / MFMAS, q1 = (m + 1) * LPS / MFMAS;
                if constexpr (q1 > q0) {
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<q1 - q0>([&](auto d_c) {
                        constexpr int q = phase * LPS + q0 + decltype(d_c)::value;
                        if constexpr (q < LOADS && MORE != 0) {
                            if constexpr (MORE == 1)
                                issue_load(q, slot, kbyte);
                            else if (more)
                                issue_load(q, slot, kbyte);
                        }
                    });
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        });
    };

    // Software pipeline over a ring of NS stage buffers, all of them loaded ahead.  The LDS
    // fragment reads of one 32-byte step take about half as long as its MFMAs, so they are issued
    // one step ahead and run under the matrix cores.  The barrier that hands over stage s+1 sits
    // before the last step of stage s: by then every fragment of stage s is in registers, so the
    // slot of stage s is free for stage s+NS, whose loads are spread over that last step and the
    // first LS-1 steps of stage s+1; the first fragments of stage s+1 are read under the MFMAs
    // of the last step.
    static_assert(LS >= 1 && LS <= KK, "loads of a stage are spread over at most one stage of steps");
    const int n_stages = (int)(row_bytes / kStageBytes);
    uint4 af[2][MI], bf[2][NP][NJ];
#pragma unroll
    for (int q = 0; q < NS; ++q)
        if (q < n_stages) issue_stage(q, q * kStageBytes);
    // Wait until all but the `later` most recently issued stages of this wavefront's loads have landed.
    auto wait_all_but = [&](int later) {
        if (NS >= 4 && later >= 3)
            wait_loads_in_flight<(NS >= 4 ? 3 : 0) * LOADS>();
        else if (NS >= 3 && later == 2)
            wait_loads_in_flight<(NS >= 3 ? 2 : 0) * LOADS>();
        else if (later == 1)
            wait_loads_in_flight<LOADS>();
        else
            wait_loads_in_flight<0>();
    };
    // this wavefront's loads of stage 0 have landed (later stages may still be in flight)
    wait_all_but((n_stages < NS ? n_stages : NS) - 1);
    __syncthreads();                             // ... and everyone's
    read_frags(lds, 0, af[0], bf[0]);
    int buf = 0, prev = NS - 1;                  // ring slots of stage s and of stage s-1
    // One stage.  What depends on the position in the K loop is passed as a compile-time constant where the caller
    // knows it (1 = yes, 0 = no, -1 = decide at run time), so that the steady state has no branch around a load and
    // no branch join in front of the MFMAs (at a join the compiler must assume the longer of the two wait lists):
    //   next : there is a stage s+1 (hand-over barrier and its first fragment reads)
    //   m0   : stage s+NS exists (its first share of loads goes into the slot this stage leaves)
    //   m1   : stage s-1+NS exists and s >= 1 (its further shares go into the slot of stage s-1)
    auto stage = [&](int s, auto next_c, auto m0_c, auto m1_c) {
        constexpr int NEXT = decltype(next_c)::value, M0 = decltype(m0_c)::value, M1 = decltype(m1_c)::value;
        const bool next = NEXT < 0 ? s + 1 < n_stages : NEXT != 0;
        const bool m0 = M0 < 0 ? s + NS < n_stages : M0 != 0;
        const bool m1 = M1 < 0 ? (s >= 1 && s - 1 + NS < n_stages) : M1 != 0;
        const uint8_t *cur = lds + buf * STAGE;
        const int nxt = buf + 1 == NS ? 0 : buf + 1;
        static_for<KK>([&](auto kk_c) {
            constexpr int kk = decltype(kk_c)::value;
            if constexpr (kk + 1 < KK) {
                read_frags(cur, kk + 1, af[(kk + 1) & 1], bf[(kk + 1) & 1]);
            } else if (next) {
                // stage s+1 has landed (this wavefront's part); stages s+2 .. s+NS-1 may still be in flight
                if constexpr (M0 == 1)
                    wait_all_but(NS - 2);
                else
                    wait_all_but((s + NS - 1 < n_stages ? s + NS - 1 : n_stages - 1) - (s + 1));
                __syncthreads();                 // everyone's has, and everyone holds its last fragments of stage s
                read_frags(lds + nxt * STAGE, 0, af[0], bf[0]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (kk == KK - 1) {
                // first share of stage s+NS, into the slot this stage has just left
                multiply(af[kk & 1], bf[kk & 1], std::integral_constant<int, 0>{}, m0_c, m0, buf, (s + NS) * kStageBytes);
            } else if constexpr (kk + 1 < LS) {
                // further shares of stage s-1+NS, into the slot of stage s-1
                multiply(af[kk & 1], bf[kk & 1], std::integral_constant<int, kk + 1>{}, m1_c, m1, prev, (s - 1 + NS) * kStageBytes);
            } else {
                multiply(af[kk & 1], bf[kk & 1], std::integral_constant<int, -1>{}, std::integral_constant<int, 0>{}, false, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        prev = buf;
        buf = nxt;
    };
    using Yes = std::integral_constant<int, 1>;
    using No = std::integral_constant<int, 0>;
    using Ask = std::integral_constant<int, -1>;
    if (n_stages > NS + 1) {
        int s = 0;
        stage(s++, Yes{}, Yes{}, No{});
        for (; s < n_stages - NS; ++s) stage(s, Yes{}, Yes{}, Yes{});
        stage(s++, Yes{}, No{}, Yes{});
        for (; s < n_stages - 1; ++s) stage(s, Yes{}, No{}, No{});
        stage(s, No{}, No{}, No{});
    } else {
        for (int s = 0; s < n_stages; ++s) stage(s, Ask{}, Ask{}, Ask{});
    }

    // ---- sign codes: a wavefront's 64 columns are one code word of a head; one ballot per accumulator
    //      register gives 32 sign bits of two rows, and lanes 0..15 write the words of the 32 rows of a tile.
    if constexpr (Store::kSignCodes) {
        if (n0 < store.code_cols) {               // uniform per workgroup
            static_assert(NJ == 2, "a wavefront must own 64 columns");
            const int col0 = n0 + wn;
            const int part = col0 / store.part_width;
            const int cin = col0 - part * store.part_width;
            const int head = cin / store.head_dim, w = (cin % store.head_dim) / 64, W = store.head_dim / 64;
            uint64_t *dst = part == 0 ? store.codes[0] : store.codes[1];
            static_for<MI>([&](auto i_c) {
                constexpr int i = decltype(i_c)::value;
                uint64_t mine[2] = {0, 0};
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint64_t lo = __ballot(acc[i][0][r] >= 0), hi = __ballot(acc[i][1][r] >= 0);
                    const uint64_t w0 = (lo & 0xFFFFFFFFull) | (hi << 32);              // rows of lanes 0..31
                    const uint64_t w1 = (lo >> 32) | (hi & 0xFFFFFFFF00000000ull);      // rows of lanes 32..63
                    if (lane == r) { mine[0] = w0; mine[1] = w1; }
                }
                if (lane < 16) {
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        const long m = m0 + wm + i * 32 + 8 * (lane >> 2) + 4 * half + (lane & 3);
                        if (m < n_rows) {
                            const long b = m / store.tokens, n = m % store.tokens;
                            dst[((size_t)(b * store.heads + head) * store.tokens + n) * W + w] = mine[half];
                        }
                    }
                }
            });
            return;
        }
    }

    // ---- epilogue.  Every output leaves through LDS so that a lane stores 16 contiguous bytes of
    //      one row: per pass, each wavefront converts one 32-row slab of its accumulators into a
    //      64 x BN staging tile, then the workgroup writes the 64 rows out.
    constexpr int CPR = BN * ES / 16;             // 16-byte chunks per staged row
    constexpr int PER_THREAD = 64 * CPR / 256;
    static_assert(PER_THREAD >= 1, "a staged slab has at least one chunk per thread");
    uint8_t *tile = lds;
    uint8_t *table = lds + SLAB_BYTES;
    const size_t out_row_bytes = (size_t)N * ES;
    const bool whole_chunks = out_row_bytes % 16 == 0;
    __syncthreads();                              // the last stage has been read
    if (Store::kTableBytes != 0) table[tid] = static_cast<const uint8_t *>(store.table)[tid];
    static_for<MI>([&](auto i_c) {
        constexpr int i = decltype(i_c)::value;
        __syncthreads();                          // the staging tile is free (and the table is there)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int nl = wn + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ml = (wave >> 1) * 32 + mfma32_row(r, lane);
                const uint32_t v = store.convert(acc[i][j][r], min(n0 + nl, N - 1), table);
                if (ES == 1)
                    tile[ml * BN + nl] = (uint8_t)v;
                else if (ES == 2)
                    reinterpret_cast<uint16_t *>(tile)[ml * BN + nl] = (uint16_t)v;
                else
                    reinterpret_cast<uint32_t *>(tile)[ml * BN + nl] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            const int c = tid + 256 * q;
            const int ml = c / CPR, cc = c % CPR;
            const long m = m0 + (ml >> 5) * (BM / 2) + i * 32 + (ml & 31);
            const int n = n0 + cc * (16 / ES);
            if (m < n_rows && n < N) {
                uint4 v = *reinterpret_cast<const uint4 *>(tile + (ml * CPR + cc) * 16);
                const long t = (Store::kScatter && rows) ? (long)rows[m] : m;
                uint8_t *dst = static_cast<uint8_t *>(store.out) + (size_t)t * out_row_bytes + (size_t)n * ES;
                if constexpr (Store::kLinear) {
                    // whole chunks by construction: part_width and N are multiples of 4
                    float4 res = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    if (store.residual) res = *reinterpret_cast<const float4 *>(store.residual + (size_t)t * N + n);
                    v.x = __builtin_bit_cast(uint32_t, __builtin_fmaf(__builtin_bit_cast(float, v.x), store.scale, res.x));
                    v.y = __builtin_bit_cast(uint32_t, __builtin_fmaf(__builtin_bit_cast(float, v.y), store.scale, res.y));
                    v.z = __builtin_bit_cast(uint32_t, __builtin_fmaf(__builtin_bit_cast(float, v.z), store.scale, res.z));
                    v.w = __builtin_bit_cast(uint32_t, __builtin_fmaf(__builtin_bit_cast(float, v.w), store.scale, res.w));
                    const int part = n / store.part_width;
                    float *base = part == 0 ? store.parts[0] : part == 1 ? store.parts[1] : store.parts[2];
                    dst = reinterpret_cast<uint8_t *>(base + (size_t)t * store.part_width + (n - part * store.part_width));
                }
                if constexpr (ES == 4 && Store::kScatter) {
                    const float gt = store.gate ? store.gate[t] : 1.0f;
                    if (store.accumulate) {
                        float old[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                        if (whole_chunks) {
                            const float4 o4 = *reinterpret_cast<const float4 *>(dst);
                            old[0] = o4.x; old[1] = o4.y; old[2] = o4.z; old[3] = o4.w;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (n + e < N) old[e] = reinterpret_cast<const float *>(dst)[e];
                        }
                        v.x = __builtin_bit_cast(uint32_t, __builtin_fmaf(gt, __builtin_bit_cast(float, v.x), old[0]));
                        v.y = __builtin_bit_cast(uint32_t, __builtin_fmaf(gt, __builtin_bit_cast(float, v.y), old[1]));
                        v.z = __builtin_bit_cast(uint32_t, __builtin_fmaf(gt, __builtin_bit_cast(float, v.z), old[2]));
                        v.w = __builtin_bit_cast(uint32_t, __builtin_fmaf(gt, __builtin_bit_cast(float, v.w), old[3]));
                    } else if (store.gate) {
                        v.x = __builtin_bit_cast(uint32_t, gt * __builtin_bit_cast(float, v.x));
                        v.y = __builtin_bit_cast(uint32_t, gt * __builtin_bit_cast(float, v.y));
                        v.z = __builtin_bit_cast(uint32_t, gt * __builtin_bit_cast(float, v.z));
                        v.w = __builtin_bit_cast(uint32_t, gt * __builtin_bit_cast(float, v.w));
                    }
                }
                if (ES < 4 || whole_chunks) {
                    *reinterpret_cast<uint4 *>(dst) = v;
                } else {                          // 32-bit rows that are not a multiple of 16 bytes
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < N) reinterpret_cast<uint32_t *>(dst)[e] = w[e];
                }
            }
        }
    });
}

template <class T, int BM, int BN, int SB, int NS, int LS, int OCC, class Store>
int launch_gemm_tile(const GemmArgs &g, const Store &store, hipStream_t st, const char *what) {
    const long row_tiles = (g.sel.max_rows + BM - 1) / BM;
    const long col_tiles = (g.N + BN - 1) / BN;
    // The fewest column groups whose share of the B planes stays resident in a 4 MiB L2 next to
    // the A rows streaming through it.  (Fewer groups fetch fewer bytes when A is the larger operand,
    // but a B share that is evicted between row tiles costs more time than the extra A traffic.)
    const size_t b_bytes = (size_t)T::kPlanes * g.N * g.K * T::kElemBytes;
    int cg = 1;
    while (cg < 8 && b_bytes / cg > (size_t)(5 << 19)) cg *= 2;     // 2.5 MiB
    const int rg = 8 / cg;
    const long blocks = 8 * ((row_tiles + rg - 1) / rg) * ((col_tiles + cg - 1) / cg);
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "%s: too many tiles for one launch", what);
    const dim3 grid((unsigned)blocks);
    GemmArgs ga = g;
    ga.col_groups = cg;
    gemm_nt_kernel<T, BM, BN, SB, NS, LS, OCC, Store><<<grid, dim3(256), 0, st>>>(ga, store);
    return check_launch(what);
}

// Tile choice, from timings of the expert layers of the DeiT-Base block on one MI355X:
//  * long rows (>= 2 KiB) in whole 128-byte lines: 128-byte stages pay (every request is a
//    whole cache line); int8 takes the 256 x 128 tile, one workgroup per CU; fp16 takes
//    128 x 128 with a ring of three, one per CU (64 x 128, two per CU, when there are few rows);
//  * short rows leave only a few stages per tile: int8 takes 64-byte stages so that two or
//    three workgroups per CU hide each other's prologue and epilogue; fp16 takes 192 x 128 tiles
//    with 128-byte stages, one per CU (128 x 64, two per CU, when there are few rows).
// Narrow (1- and 2-byte) output rows must be whole 16-byte chunks; operand rows must be a
// multiple of 64 bytes long.
template <class T, class Store>
int launch_gemm(const GemmArgs &g, const Store &store, hipStream_t st, const char *what) {
    if (g.sel.max_rows == 0 || g.N == 0) return SA_OK;
    const size_t row_bytes = (size_t)g.K * T::kElemBytes;
    SA_REQUIRE(row_bytes % 64 == 0 && row_bytes > 0, SA_ERR_SHAPE, "%s: rows of %zu bytes are not a multiple of 64", what, row_bytes);
    const bool short_a = g.a_valid > 0 && g.a_valid != g.K;
    SA_REQUIRE(!short_a || (T::kPlanes == 2 && g.a_valid > 0 && g.a_valid < g.K && g.a_valid % 16 == 0), SA_ERR_SHAPE,
               "%s: A rows of %d valid elements in a contraction of %d", what, g.a_valid, g.K);
    SA_REQUIRE(Store::kBytes == 4 || (size_t)g.N * Store::kBytes % 16 == 0, SA_ERR_SHAPE,
               "%s: narrow output rows of %d elements are not whole 16-byte chunks", what, g.N);
    const bool lines = row_bytes % 128 == 0 && !short_a, long_rows = row_bytes >= 2048;
    const long blocks256 = ((g.sel.max_rows + 255) / 256) * ((g.N + 127) / 128);
    if constexpr (T::kPlanes == 2) {
        if (lines && long_rows) return launch_gemm_tile<T, 256, 128, 128, 2, 2, 1, Store>(g, store, st, what);
        if (blocks256 >= 512) return launch_gemm_tile<T, 256, 128, 64, 2, 1, 2, Store>(g, store, st, what);
        return launch_gemm_tile<T, 128, 128, 64, 2, 1, 3, Store>(g, store, st, what);
    } else {
        const bool many_rows = g.sel.max_rows >= 2048;
        if (lines && long_rows)
            return many_rows ? launch_gemm_tile<T, 128, 128, 128, 3, 2, 1, Store>(g, store, st, what)
                             : launch_gemm_tile<T, 64, 128, 128, 3, 2, 2, Store>(g, store, st, what);
        if (lines)
            return many_rows ? launch_gemm_tile<T, 192, 128, 128, 2, 2, 1, Store>(g, store, st, what)
                             : launch_gemm_tile<T, 128, 64, 128, 2, 2, 2, Store>(g, store, st, what);
        return launch_gemm_tile<T, 128, 128, 64, 3, 1, 2, Store>(g, store, st, what);
    }
}

}  // namespace sa
