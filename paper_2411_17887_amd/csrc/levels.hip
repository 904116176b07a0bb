// Algorithm 1 (MatMulScan) executed literally, one kernel launch per round.
//
// This is the paper's schedule without any fusion: k up-sweep rounds that gather the stride-s^t
// subvector starting at s^t - 1, multiply every s x s chunk by L_s and scatter it back, then k-1
// down-sweep rounds that do the same with B_s on the stride-s^(t-1) subvector starting at s^t - 1.
// One chunk is one product on the matrix unit (procedure BatchMatMul: zero-pad, column-major view,
// left-multiply, flatten) in the unit's native shapes: s = 16 (16 x 16 MFMA), s = 4 (sixteen 4 x 4 blocks
// per instruction) and s = 32 (32 x 32 MFMA) -- the fan-in against depth trade-off of the paper's
// comparison table, 2 log_s n - 1 rounds each.  Both constant matrices go through the matrix unit, B_s
// included, so the utilisation remarks of the paper's discussion section can be measured: the kernel
// counts the s x s products it issues (Lemma 1) and its run time is dominated by the strided
// gathers/scatters.
//
// The fused single-pass kernel in tcuscan.hip is the product path; this executor exists to compare
// against it and to check the schedule itself on the device.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tcuscan.h"

namespace {

typedef float f32x4  __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int   i32x4  __attribute__((ext_vector_type(4)));
typedef int   i32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;        // 4 wavefronts

enum { kMatL = 0, kMatB = 1 };

// Entry (row, col) of the constant left operand: L_s is lower-triangular all-ones, B_s is the identity
// with an all-ones first column.
__device__ __forceinline__ bool mat_entry(int which, int row, int col)
{
    return which == kMatL ? (col <= row) : (col == 0 || col == row);
}
// number of ones in a row (the signed-byte planes of the integer path are biased by 128 per summed entry)
__device__ __forceinline__ uint32_t row_ones(int which, int row) { return which == kMatL ? (uint32_t)(row + 1) : (row == 0 ? 1u : 2u); }

template <class T> __device__ __forceinline__ T zero();
template <> __device__ __forceinline__ float zero<float>() { return 0.f; }
template <> __device__ __forceinline__ uint32_t zero<uint32_t>() { return 0u; }

// exact conversion of an input element to the accumulator type
template <int DT> struct In;
template <> struct In<TCUSCAN_I32_I32>  { using acc = uint32_t; static __device__ acc load(const void *p, size_t i) { return ((const uint32_t *)p)[i]; } };
template <> struct In<TCUSCAN_I8_I32>   { using acc = uint32_t; static __device__ acc load(const void *p, size_t i) { return (uint32_t)(int32_t)((const int8_t *)p)[i]; } };
template <> struct In<TCUSCAN_F32_F32>  { using acc = float;    static __device__ acc load(const void *p, size_t i) { return ((const float *)p)[i]; } };
template <> struct In<TCUSCAN_F16_F32>  { using acc = float;    static __device__ acc load(const void *p, size_t i) { return (float)((const _Float16 *)p)[i]; } };
template <> struct In<TCUSCAN_BF16_F32> { using acc = float;    static __device__ acc load(const void *p, size_t i) { return __builtin_bit_cast(float, (uint32_t)((const uint16_t *)p)[i] << 16); } };

// byte `p` of four 32-bit words, each as (byte - 128), packed into one word
__device__ __forceinline__ uint32_t plane4(const uint32_t *t, int p)
{
    uint32_t b = 0;
    for (int i = 0; i < 4; ++i) b |= (((t[i] >> (8 * p)) & 0xFFu) ^ 0x80u) << (8 * i);
    return b;
}

// One step of a wavefront for radix S: kChunks chunks of S x S gathered entries, kE entries per lane.
// in_index / out_index give the position (inside the step's S*S*kChunks entries) of the lane's i-th operand
// entry and i-th result entry; product() is W = A * T on the MFMA unit for all chunks of the step.
template <int S, class A> struct Radix;

// ---- s = 16: one chunk per step.  Lane (j, c) = (lane / 16, lane % 16) holds T[4j .. 4j+3][c] and receives
// W[4j .. 4j+3][c]  (f32: four K = 4 products; i32: four signed-byte planes through the K = 32 i8 product).
template <class A> struct Radix<16, A> {
    static constexpr int kChunks = 1, kE = 4;
    static __device__ __forceinline__ int in_index(int lane, int i)  { return 16 * (lane & 15) + 4 * (lane >> 4) + i; }
    static __device__ __forceinline__ int out_index(int lane, int i) { return in_index(lane, i); }
    static __device__ __forceinline__ void product(int which, int lane, const float (&t)[4], float (&w)[4])
    {
        const int m = lane & 15, j = lane >> 4;
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < 4; ++p)          // K = 4 per instruction; slot (j, p) carries column-position 4j + p
            d = __builtin_amdgcn_mfma_f32_16x16x4f32(mat_entry(which, m, 4 * j + p) ? 1.0f : 0.0f, t[p], d, 0, 0, 0);
        for (int r = 0; r < 4; ++r) w[r] = d[r];
    }
    static __device__ __forceinline__ void product(int which, int lane, const uint32_t (&t)[4], uint32_t (&w)[4])
    {
        const int m = lane & 15, j = lane >> 4;
        uint32_t a_lo = 0;
        for (int i = 0; i < 4; ++i) a_lo |= (mat_entry(which, m, 4 * j + i) ? 1u : 0u) << (8 * i);
        const i32x4 z = {0, 0, 0, 0};
        i32x4 pl[4];
        for (int p = 0; p < 4; ++p)
            pl[p] = __builtin_amdgcn_mfma_i32_16x16x32_i8((long)(uint64_t)a_lo, (long)(uint64_t)plane4(t, p), z, 0, 0, 0);
        for (int r = 0; r < 4; ++r)
            w[r] = (uint32_t)pl[0][r] + ((uint32_t)pl[1][r] << 8) + ((uint32_t)pl[2][r] << 16) + ((uint32_t)pl[3][r] << 24)
                   + row_ones(which, 4 * j + r) * 0x80808080u;
    }
};

// ---- s = 4: sixteen chunks per step, one per 4 x 4 block of the instruction.  Lane 4b + j holds column j of
// chunk b (4 consecutive gathered entries) and receives the same column of the result.
template <class A> struct Radix<4, A> {
    static constexpr int kChunks = 16, kE = 4;
    static __device__ __forceinline__ int in_index(int lane, int i)  { return 4 * lane + i; }
    static __device__ __forceinline__ int out_index(int lane, int i) { return 4 * lane + i; }
    static __device__ __forceinline__ void product(int which, int lane, const float (&t)[4], float (&w)[4])
    {
        const int row = lane & 3;            // A operand: lane 4b + i supplies A[i][k] of block b
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < 4; ++p)          // K = 1 per instruction
            d = __builtin_amdgcn_mfma_f32_4x4x1f32(mat_entry(which, row, p) ? 1.0f : 0.0f, t[p], d, 0, 0, 0);
        for (int r = 0; r < 4; ++r) w[r] = d[r];
    }
    static __device__ __forceinline__ void product(int which, int lane, const uint32_t (&t)[4], uint32_t (&w)[4])
    {
        const int row = lane & 3;
        uint32_t a = 0;
        for (int k = 0; k < 4; ++k) a |= (mat_entry(which, row, k) ? 1u : 0u) << (8 * k);
        const i32x4 z = {0, 0, 0, 0};
        i32x4 pl[4];
        for (int p = 0; p < 4; ++p)          // K = 4 per instruction: the whole column at once
            pl[p] = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a, (int)plane4(t, p), z, 0, 0, 0);
        for (int r = 0; r < 4; ++r)
            w[r] = (uint32_t)pl[0][r] + ((uint32_t)pl[1][r] << 8) + ((uint32_t)pl[2][r] << 16) + ((uint32_t)pl[3][r] << 24)
                   + row_ones(which, r) * 0x80808080u;
    }
};

// ---- s = 32: one chunk of 1024 entries per step, 16 per lane.  Result register r of lane l is
// W[8 (r / 4) + 4 (l / 32) + r % 4][l % 32].
template <> struct Radix<32, float> {
    static constexpr int kChunks = 1, kE = 16;
    // K = 2 per instruction: lane (h, j) = (lane / 32, lane % 32) supplies T[2p + h][j] to product p
    static __device__ __forceinline__ int in_index(int lane, int i)  { return 32 * (lane & 31) + 2 * i + (lane >> 5); }
    static __device__ __forceinline__ int out_index(int lane, int r) { return 32 * (lane & 31) + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
    static __device__ __forceinline__ void product(int which, int lane, const float (&t)[16], float (&w)[16])
    {
        const int row = lane & 31, h = lane >> 5;
        f32x16 d;
        for (int r = 0; r < 16; ++r) d[r] = 0.f;
        for (int p = 0; p < 16; ++p)
            d = __builtin_amdgcn_mfma_f32_32x32x2f32(mat_entry(which, row, 2 * p + h) ? 1.0f : 0.0f, t[p], d, 0, 0, 0);
        for (int r = 0; r < 16; ++r) w[r] = d[r];
    }
};
template <> struct Radix<32, uint32_t> {
    static constexpr int kChunks = 1, kE = 16;
    // K = 16 per instruction, 8 bytes per lane: lane (h, j) supplies T[16q + 8h .. 16q + 8h + 7][j] to product q
    static __device__ __forceinline__ int in_index(int lane, int i)  { return 32 * (lane & 31) + 16 * (i >> 3) + 8 * (lane >> 5) + (i & 7); }
    static __device__ __forceinline__ int out_index(int lane, int r) { return Radix<32, float>::out_index(lane, r); }
    static __device__ __forceinline__ void product(int which, int lane, const uint32_t (&t)[16], uint32_t (&w)[16])
    {
        const int row = lane & 31, h = lane >> 5;
        i32x16 pl[4];
        for (int p = 0; p < 4; ++p) {
            for (int r = 0; r < 16; ++r) pl[p][r] = 0;
            for (int q = 0; q < 2; ++q) {
                uint64_t a = 0;
                for (int k = 0; k < 8; ++k) a |= (uint64_t)(mat_entry(which, row, 16 * q + 8 * h + k) ? 1u : 0u) << (8 * k);
                const uint64_t b = (uint64_t)plane4(t + 8 * q, p) | ((uint64_t)plane4(t + 8 * q + 4, p) << 32);
                pl[p] = __builtin_amdgcn_mfma_i32_32x32x16_i8((long)a, (long)b, pl[p], 0, 0, 0);
            }
        }
        for (int r = 0; r < 16; ++r) {
            const int out_row = 8 * (r >> 2) + 4 * h + (r & 3);
            w[r] = (uint32_t)pl[0][r] + ((uint32_t)pl[1][r] << 8) + ((uint32_t)pl[2][r] << 16) + ((uint32_t)pl[3][r] << 24)
                   + row_ones(which, out_row) * 0x80808080u;
        }
    }
};

// One round: z = BatchMatMul(y, A) on y = x[start :: step] (m entries), scattered back to the same places.
// Round 0 of the up-sweep reads the input array (any supported type); every later round works in place on
// the output array, which holds accumulator-typed values.
template <int DT, int S>
__global__ __launch_bounds__(kThreads) void round_kernel(const void *src, typename In<DT>::acc *dst, bool from_input,
                                                         size_t start, size_t step, size_t m, int which,
                                                         unsigned long long *matmuls)
{
    using A = typename In<DT>::acc;
    using R = Radix<S, A>;
    constexpr size_t kStep = (size_t)S * S * R::kChunks;              // gathered entries per wavefront step
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t chunks = (m + (size_t)S * S - 1) / ((size_t)S * S);  // zero-pad to a multiple of s^2
    const size_t steps = (chunks + R::kChunks - 1) / R::kChunks;
    unsigned long long mine = 0;
    for (size_t b = (size_t)blockIdx.x * 4 + wave; b < steps; b += (size_t)gridDim.x * 4) {
        A t[R::kE], w[R::kE];
        for (int i = 0; i < R::kE; ++i) {
            const size_t g = b * kStep + (size_t)R::in_index(lane, i);
            t[i] = zero<A>();
            if (g < m) t[i] = from_input ? In<DT>::load(src, start + g * step) : dst[start + g * step];
        }
        R::product(which, lane, t, w);
        for (int i = 0; i < R::kE; ++i) {
            const size_t g = b * kStep + (size_t)R::out_index(lane, i);
            if (g < m) dst[start + g * step] = w[i];                   // drop the padding
        }
        const size_t left = chunks - b * R::kChunks;                   // chunks of this step that are not all padding
        mine += left < (size_t)R::kChunks ? left : (size_t)R::kChunks;
    }
    if (matmuls && lane == 0 && mine) atomicAdd(matmuls, mine);
}

template <int DT, int S>
hipError_t run_levels(const void *d_in, void *d_out, size_t n, int k, int rounds, unsigned long long *d_matmuls, hipStream_t s)
{
    using A = typename In<DT>::acc;
    constexpr size_t kPerBlock = 4 * (size_t)Radix<S, A>::kChunks;      // chunks per workgroup step
    int done = 0;
    auto launch = [&](bool from_input, size_t start, size_t step, int which) -> hipError_t {
        const size_t m = (n - 1 - start) / step + 1;
        const size_t chunks = (m + (size_t)S * S - 1) / ((size_t)S * S);
        const size_t wgs = (chunks + kPerBlock - 1) / kPerBlock;
        const unsigned grid = (unsigned)(wgs < 4096 ? wgs : 4096);
        const void *src = d_in; A *dst = (A *)d_out; size_t mm = m; bool fi = from_input; int wh = which;
        unsigned long long *cnt = d_matmuls;
        void *args[] = {&src, &dst, &fi, &start, &step, &mm, &wh, &cnt};
        return hipLaunchKernel((const void *)round_kernel<DT, S>, dim3(grid), dim3(kThreads), args, 0, s);
    };
    size_t p = 1;                                                       // s^t
    for (int t = 0; t < k; ++t, p *= S) {                               // first phase (up-sweep)
        if (rounds >= 0 && done >= rounds) return hipSuccess;
        hipError_t e = launch(t == 0, p - 1, p, kMatL);
        if (e != hipSuccess) return e;
        ++done;
    }
    p /= S;                                                             // s^(k-1)
    for (int t = k - 1; t >= 1; --t, p /= S) {                          // second phase (down-sweep)
        if (rounds >= 0 && done >= rounds) return hipSuccess;
        hipError_t e = launch(false, p - 1, p / S, kMatB);
        if (e != hipSuccess) return e;
        ++done;
    }
    return hipSuccess;
}

template <int S>
hipError_t run_levels_dt(const void *d_in, void *d_out, size_t n, int dt, int k, int rounds, unsigned long long *d_matmuls, hipStream_t s)
{
    switch (dt) {
    case TCUSCAN_I32_I32:  return run_levels<TCUSCAN_I32_I32, S>(d_in, d_out, n, k, rounds, d_matmuls, s);
    case TCUSCAN_F16_F32:  return run_levels<TCUSCAN_F16_F32, S>(d_in, d_out, n, k, rounds, d_matmuls, s);
    case TCUSCAN_I8_I32:   return run_levels<TCUSCAN_I8_I32, S>(d_in, d_out, n, k, rounds, d_matmuls, s);
    case TCUSCAN_F32_F32:  return run_levels<TCUSCAN_F32_F32, S>(d_in, d_out, n, k, rounds, d_matmuls, s);
    default:               return run_levels<TCUSCAN_BF16_F32, S>(d_in, d_out, n, k, rounds, d_matmuls, s);
    }
}

}  // namespace

extern "C" tcuscan_status_t tcuscan_matmulscan_levels_radix(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt, int s,
                                                            int rounds, unsigned long long *d_matmuls, tcuscan_stream_t stream)
{
    if ((int)dt < 0 || (int)dt > 4) return TCUSCAN_ERR_UNSUPPORTED;
    if (s != 4 && s != 16 && s != 32) return TCUSCAN_ERR_UNSUPPORTED;
    int k = 0;
    size_t p = 1;
    while (p < n) { p *= (size_t)s; ++k; }
    if (n == 0 || p != n || k < 1) return TCUSCAN_ERR_UNSUPPORTED;      // Algorithm 1 proper: n = s^k
    if (!d_in || !d_out) return TCUSCAN_ERR_INVALID_ARG;
    const size_t isz = dt == TCUSCAN_I8_I32 ? 1 : (dt == TCUSCAN_F16_F32 || dt == TCUSCAN_BF16_F32) ? 2 : 4;
    if (((uintptr_t)d_in % isz) != 0 || ((uintptr_t)d_out % 4) != 0) return TCUSCAN_ERR_INVALID_ARG;
    if (d_in == d_out && isz != 4) return TCUSCAN_ERR_INVALID_ARG;
    if (d_matmuls && ((uintptr_t)d_matmuls % 8) != 0) return TCUSCAN_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    if (s == 4)       e = run_levels_dt<4>(d_in, d_out, n, (int)dt, k, rounds, d_matmuls, st);
    else if (s == 16) e = run_levels_dt<16>(d_in, d_out, n, (int)dt, k, rounds, d_matmuls, st);
    else              e = run_levels_dt<32>(d_in, d_out, n, (int)dt, k, rounds, d_matmuls, st);
    return e == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

extern "C" tcuscan_status_t tcuscan_matmulscan_levels(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt,
                                                      int rounds, unsigned long long *d_matmuls, tcuscan_stream_t stream)
{
    return tcuscan_matmulscan_levels_radix(d_in, d_out, n, dt, 16, rounds, d_matmuls, stream);
}
