// Tiled "NT" matrix-core GEMM shared by the Shift expert (int8 x two int8 weight planes,
// int32 accumulate) and the Mult expert (fp16 x fp16, fp32 accumulate):
//     C[m, n] = sum_p sum_k A[m, k] * B_p[n, k]
//
// Workgroup tile BM x BN, four wavefronts in a 2 x 2 grid, each owning (BM/2) x (BN/2) as
// 32x32 MFMA tiles.  K advances 64 bytes per stage through a double-buffered LDS tile that
// is filled by direct global->LDS loads (no register staging): while stage s is multiplied
// out of one buffer, the loads of stage s+1 are in flight into the other; one barrier per
// stage.  A direct load writes 1 KiB of consecutive LDS per wavefront instruction, so LDS
// rows cannot be padded; instead the 16-byte chunks of a row are XOR-swizzled with the row
// number (the lane chooses which global chunk it fetches), which makes the 16-byte fragment
// reads of any 16 consecutive rows hit 16 different bank groups.
//
// The loads are issued from inline assembly: the kernel orders them by hand (one vmcnt(0)
// and one barrier per stage), and the compiler must not serialise the reads of the current
// buffer behind the loads in flight into the other one.
//
// Narrow outputs (int8 / fp16 hidden rows) leave through LDS so that every lane stores 16
// bytes of one row; 32-bit outputs are stored straight from the accumulators (a 32x32 tile
// row is 128 contiguous bytes).
#pragma once

#include "common.h"
#include "gemm_common.h"

namespace sa {

constexpr int kStageBytes = 64;                 // bytes of K per stage and row
constexpr int kChunksPerRow = kStageBytes / 16; // 16-byte chunks per LDS row

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
    int K, N;
};

// Physical 16-byte chunk of logical chunk c in LDS row r.
__device__ inline int swizzle(int r, int c) {
    return c ^ ((r / (16 / kChunksPerRow)) & (kChunksPerRow - 1));
}

// One wavefront-wide direct load: lane l's 16 bytes at `src` land at LDS byte lds_base + 16 * l.
__device__ inline void load_to_lds_16(const void *src, uint32_t lds_base) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, off\n\t"
        :
        : "s"(lds_base), "v"(src)
        : "memory");
}

// A Store type provides
//   static constexpr int kPackedBytes : 0 = 32-bit output stored per element with
//       void direct(long m, int n, acc, const int32_t *rows) const
//     1 or 2 = narrow output [max_rows, N] written through LDS with
//       uint32_t convert(acc, const uint8_t *lds_table) const,  void *out,  const void *table (256 B or null)
template <class T, int BM, int BN, class Store>
__global__ __launch_bounds__(256, 2) void gemm_nt_kernel(GemmArgs g, Store store) {
    constexpr int NP = T::kPlanes;
    constexpr int MI = BM / 64, NJ = BN / 64;           // 32x32 tiles per wavefront
    constexpr int A_BYTES = BM * kStageBytes, B_BYTES = BN * kStageBytes;
    constexpr int STAGE = A_BYTES + NP * B_BYTES;
    constexpr int ROWS_PER_INSTR = 1024 / kStageBytes;  // LDS rows one wavefront load fills
    constexpr int A_INSTR = BM / ROWS_PER_INSTR / 4;    // loads per wavefront and stage
    constexpr int B_INSTR = BN / ROWS_PER_INSTR / 4;
    constexpr int ES = Store::kPackedBytes;
    constexpr int EPI_BYTES = ES ? BM * BN * ES + Store::kTableBytes : 0;
    constexpr int LDS_BYTES = 2 * STAGE > EPI_BYTES ? 2 * STAGE : EPI_BYTES;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[LDS_BYTES];

    const int32_t *rows;
    long n_rows;
    resolve_rows(g.sel, rows, n_rows);
    // Workgroups are handed to the 8 XCDs round-robin by their linear id, and each XCD has its own
    // L2.  All column tiles of one row tile are therefore given ids with the same id % 8: the row
    // tile of A is fetched into one L2 only, and the (small) B planes stay resident in every L2.
    const int col_tiles = (g.N + BN - 1) / BN;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const long m0 = ((long)(slot / col_tiles) * 8 + xcd) * BM;
    if (m0 >= n_rows) return;
    const int n0 = (slot % col_tiles) * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
    const int N = g.N;
    const size_t row_bytes = (size_t)g.K * T::kElemBytes;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;

    // ---- what each lane fetches.  Wavefront w issues load i for LDS rows
    //      (w * X_INSTR + i) * ROWS_PER_INSTR + lane / kChunksPerRow, physical chunk lane % kChunksPerRow.
    //      Rows past the end are clamped to the last valid row (computed, never stored).
    const uint8_t *a_src[A_INSTR];
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i) {
        const int r = (wave * A_INSTR + i) * ROWS_PER_INSTR + lane / kChunksPerRow;
        const int c = swizzle(r, lane % kChunksPerRow);
        long m = m0 + r;
        m = m < n_rows ? m : n_rows - 1;
        const long src = (g.gather_a && rows) ? (long)rows[m] : m;
        a_src[i] = static_cast<const uint8_t *>(g.a) + (size_t)src * row_bytes + c * 16;
    }
    const uint8_t *b_src[NP][B_INSTR];
#pragma unroll
    for (int i = 0; i < B_INSTR; ++i) {
        const int r = (wave * B_INSTR + i) * ROWS_PER_INSTR + lane / kChunksPerRow;
        const int c = swizzle(r, lane % kChunksPerRow);
        const int n = min(n0 + r, N - 1);
#pragma unroll
        for (int p = 0; p < NP; ++p)
            b_src[p][i] = static_cast<const uint8_t *>(g.b[p]) + (size_t)n * row_bytes + c * 16;
    }

    auto issue_stage = [&](int buf, int kbyte) {
        const uint32_t base = lds_base + buf * STAGE;
#pragma unroll
        for (int i = 0; i < A_INSTR; ++i) load_to_lds_16(a_src[i] + kbyte, base + (wave * A_INSTR + i) * 1024);
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int i = 0; i < B_INSTR; ++i)
                load_to_lds_16(b_src[p][i] + kbyte, base + A_BYTES + p * B_BYTES + (wave * B_INSTR + i) * 1024);
    };

    typename T::Acc acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // fragment read offsets (bytes inside a tile) for the two 32-byte halves of a stage
    const int fr = lane & 31, fg = lane >> 5;
    int a_rd[MI][2], b_rd[NJ][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int r = wm + i * 32 + fr;
            a_rd[i][kk] = r * kStageBytes + swizzle(r, 2 * kk + fg) * 16;
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int r = wn + j * 32 + fr;
            b_rd[j][kk] = r * kStageBytes + swizzle(r, 2 * kk + fg) * 16;
        }
    }

    const int n_stages = (int)(row_bytes / kStageBytes);
    issue_stage(0, 0);
    for (int s = 0; s < n_stages; ++s) {
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wavefront's loads of stage s have landed
        __syncthreads();                         // ... everyone's have, and everyone is done with the other buffer
        if (s + 1 < n_stages) issue_stage((s + 1) & 1, (s + 1) * kStageBytes);
        const uint8_t *A = lds + (s & 1) * STAGE;
        const uint8_t *B = A + A_BYTES;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            uint4 af[MI], bf[NP][NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i) af[i] = *reinterpret_cast<const uint4 *>(A + a_rd[i][kk]);
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    bf[p][j] = *reinterpret_cast<const uint4 *>(B + p * B_BYTES + b_rd[j][kk]);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int p = 0; p < NP; ++p) acc[i][j] = T::mma(af[i], bf[p][j], acc[i][j]);
        }
    }

    if constexpr (ES == 0) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int n = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long m = m0 + wm + i * 32 + mfma32_row(r, lane);
                    if (m < n_rows && n < N) store.direct(m, n, acc[i][j][r], rows);
                }
            }
    } else {
        // narrow output: convert, lay the BM x BN tile out row-major in LDS, store 16 B per lane
        uint8_t *tile = lds;
        uint8_t *table = lds + BM * BN * ES;
        __syncthreads();                          // the last stage has been read
        if (Store::kTableBytes != 0) table[tid] = static_cast<const uint8_t *>(store.table)[tid];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int nl = wn + j * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ml = wm + i * 32 + mfma32_row(r, lane);
                    const uint32_t v = store.convert(acc[i][j][r], table);
                    if (ES == 1)
                        tile[ml * BN + nl] = (uint8_t)v;
                    else
                        reinterpret_cast<uint16_t *>(tile)[ml * BN + nl] = (uint16_t)v;
                }
            }
        __syncthreads();
        constexpr int CPR = BN * ES / 16;         // 16-byte chunks per tile row
        constexpr int PER_THREAD = BM * CPR / 256;
        const size_t out_row_bytes = (size_t)N * ES;
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            const int c = tid + 256 * q;
            const int ml = c / CPR, cc = c % CPR;
            const long m = m0 + ml;
            const int n = n0 + cc * (16 / ES);
            if (m < n_rows && n < N)
                *reinterpret_cast<uint4 *>(static_cast<uint8_t *>(store.out) + (size_t)m * out_row_bytes + (size_t)n * ES) =
                    *reinterpret_cast<const uint4 *>(tile + (ml * CPR + cc) * 16);
        }
    }
}

template <class T, int BM, int BN, class Store>
int launch_gemm_tile(const GemmArgs &g, const Store &store, hipStream_t st, const char *what) {
    const long row_tiles = (g.sel.max_rows + BM - 1) / BM;
    const long col_tiles = (g.N + BN - 1) / BN;
    const long blocks = (row_tiles + 7) / 8 * 8 * col_tiles;
    SA_REQUIRE(blocks < (1L << 31), SA_ERR_SHAPE, "%s: too many tiles for one launch", what);
    const dim3 grid((unsigned)blocks);
    gemm_nt_kernel<T, BM, BN, Store><<<grid, dim3(256), 0, st>>>(g, store);
    return check_launch(what);
}

// Tall tiles reuse the B fragments more; small problems need more, smaller workgroups.
// Narrow outputs need N % 16 == 0 (whole 16-byte chunks per row).
template <class T, class Store>
int launch_gemm(const GemmArgs &g, const Store &store, hipStream_t st, const char *what) {
    if (g.sel.max_rows == 0 || g.N == 0) return SA_OK;
    const long col_tiles = (g.N + 127) / 128;
    const long blocks256 = ((g.sel.max_rows + 255) / 256) * col_tiles;
    if (blocks256 >= 512) return launch_gemm_tile<T, 256, 128, Store>(g, store, st, what);
    return launch_gemm_tile<T, 128, 128, Store>(g, store, st, what);
}

}  // namespace sa
