// sa_probe_mfma: a measurement helper, not a step of the path.  It runs a register-only loop of matrix
// instructions (no memory traffic at all) on as many workgroups as asked for, so that a caller can read off what
// the matrix cores of this chip sustain - instruction rate and shader clock - with operands like the ones the
// Shift and Mult experts feed them.  The roofline fractions bench.py reports are priced against the published
// peaks; this loop shows how much of those peaks is reachable before any kernel design enters.
#include "common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// An empty volatile statement that reads and "writes" a register tile: the compiler may move neither the clock
// reads (which have side effects) nor the loop that produces the tile across it.
template <class V>
__device__ inline void pin(V &v) {
    asm volatile("" : "+v"(v));
}

__device__ inline uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// KIND: 0 = v_mfma_i32_32x32x32_i8, 1 = v_mfma_f32_32x32x16_f16, 2 = v_mfma_f32_32x32x16_bf16.
// Operand registers (4 dwords each, four of them per side, rotated so that no two consecutive instructions see
// the same pair): operands 0 = one non-zero element per register (hardly any bit toggles), 1 = random bits,
// 2 (int8 only) = random int8 on one side, on the other side powers of two alternating with a plane that is 7/8
// zeros, as the two weight planes of a Shift layer are.
template <int KIND>
__global__ __launch_bounds__(256) void probe_kernel(int iters, int operands, unsigned long long *out) {
    v4i x[4], y[4];
    for (int q = 0; q < 4; ++q)
        for (int e = 0; e < 4; ++e) {
            const uint32_t h1 = mix(threadIdx.x * 64 + q * 8 + e + blockIdx.x * 7919u), h2 = mix(h1 + 12345u);
            uint32_t a = h1, b = h2;
            if (operands == 0) {
                a = b = (e == 0) ? (KIND == 0 ? 1u : 0x3C00u) : 0u;
            } else if (KIND != 0) {
                // finite halves / bf16 of moderate size: clear the top exponent bits
                a = h1 & 0xB7FFB7FFu;
                b = h2 & 0xB7FFB7FFu;
            } else if (operands == 2) {
                uint32_t w = 0;
                for (int byte = 0; byte < 4; ++byte) {
                    const uint32_t r = (h2 >> (8 * byte)) & 0xFFu;
                    const uint32_t ex = r & 7u, neg = (r >> 3) & 1u;
                    uint32_t val;
                    if (q & 1) val = (ex == 7u) ? 64u : 0u;                 // the sparse plane
                    else val = 1u << (ex < 6u ? ex : 6u);                    // the dense plane
                    if (neg) val = (0u - val) & 0xFFu;
                    w |= val << (8 * byte);
                }
                b = w;
            }
            x[q][e] = (int)a;
            y[q][e] = (int)b;
        }
    long long t0, w0, t1, w1;
    long long sink = 0;
    if constexpr (KIND == 0) {
        v16i acc[8];
        for (int a = 0; a < 8; ++a)
            for (int r = 0; r < 16; ++r) acc[a][r] = 0;
        for (int a = 0; a < 8; ++a) pin(acc[a]);
        t0 = __builtin_readcyclecounter(), w0 = wall_clock64();
        for (int a = 0; a < 8; ++a) pin(acc[a]);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int a = 0; a < 8; ++a) acc[a] = __builtin_amdgcn_mfma_i32_32x32x32_i8(x[a & 3], y[(a + it) & 3], acc[a], 0, 0, 0);
        }
        for (int a = 0; a < 8; ++a) pin(acc[a]);
        t1 = __builtin_readcyclecounter(), w1 = wall_clock64();
        for (int a = 0; a < 8; ++a)
            for (int r = 0; r < 16; ++r) sink += acc[a][r];
    } else {
        v16f acc[8];
        for (int a = 0; a < 8; ++a)
            for (int r = 0; r < 16; ++r) acc[a][r] = 0.0f;
        for (int a = 0; a < 8; ++a) pin(acc[a]);
        t0 = __builtin_readcyclecounter(), w0 = wall_clock64();
        for (int a = 0; a < 8; ++a) pin(acc[a]);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int a = 0; a < 8; ++a) {
                if constexpr (KIND == 1)
                    acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, x[a & 3]), __builtin_bit_cast(v8h, y[(a + it) & 3]),
                                                                    acc[a], 0, 0, 0);
                else
                    acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, x[a & 3]),
                                                                     __builtin_bit_cast(v8bf, y[(a + it) & 3]), acc[a], 0, 0, 0);
            }
        }
        for (int a = 0; a < 8; ++a) pin(acc[a]);
        t1 = __builtin_readcyclecounter(), w1 = wall_clock64();
        for (int a = 0; a < 8; ++a)
            for (int r = 0; r < 16; ++r) sink += (long long)__builtin_bit_cast(int, acc[a][r]);
    }
    if (sink == 0x7fffffff12345678LL) out[2] = (unsigned long long)sink;      // keeps the loop alive; never true in practice
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = (unsigned long long)(t1 - t0);
        out[1] = (unsigned long long)(w1 - w0);
    }
}

}  // namespace

extern "C" int sa_probe_mfma(int kind, int operands, int workgroups, int iters, unsigned long long *out, void *stream) {
    sa::clear_error();
    SA_REQUIRE(kind >= 0 && kind <= 2, SA_ERR_INVALID, "sa_probe_mfma: kind must be 0 (int8), 1 (fp16) or 2 (bf16)");
    SA_REQUIRE(operands >= 0 && operands <= 2 && (operands < 2 || kind == 0), SA_ERR_INVALID,
               "sa_probe_mfma: operands must be 0, 1 or (int8 only) 2");
    SA_REQUIRE(workgroups > 0 && workgroups <= 65536 && iters > 0 && iters <= (1 << 22), SA_ERR_INVALID,
               "sa_probe_mfma: workgroups in [1, 65536], iters in [1, 2^22]");
    SA_REQUIRE(out != nullptr && sa::aligned16(out), SA_ERR_INVALID, "sa_probe_mfma: out must be 16-byte aligned device memory (3 x 8 bytes)");
    hipStream_t st = sa::as_stream(stream);
    if (kind == 0)
        probe_kernel<0><<<dim3(workgroups), dim3(256), 0, st>>>(iters, operands, out);
    else if (kind == 1)
        probe_kernel<1><<<dim3(workgroups), dim3(256), 0, st>>>(iters, operands, out);
    else
        probe_kernel<2><<<dim3(workgroups), dim3(256), 0, st>>>(iters, operands, out);
    return sa::check_launch("sa_probe_mfma");
}
