// Two applications built on the scan, the ones the paper's introduction names as its motivation for
// putting prefix sums on the matrix unit: stream compaction (the "split" / "pack" primitive) and, through
// Blelloch's reduction of radix sort to prefix sums, sorting ("can TCU sort?").
//
// Both are thin: the only non-trivial step is the exclusive scan of a 0/1 byte mask, which is the
// library's int8 -> int32 MFMA scan; the kernels here only build the mask and move the elements.
//
//   compaction : pos = exclusive_scan(mask);  out[pos[i]] = values[i] where mask[i] != 0
//                (without a positions buffer the scatter is fused into the scan kernel: tcuscan.hip, compact_store)
//   split(b)   : f[i] = (bit b of key[i] == 0);  pos = exclusive_scan(f);  Z = pos[n-1] + f[n-1]
//                key i goes to  pos[i]            if f[i]      (zeros keep their order, in front)
//                          to  Z + (i - pos[i])   otherwise   (ones keep their order, behind)
//   radix sort : split(0), split(1), ..., split(bits-1)   -- least significant bit first, stable

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/tcuscan.h"

extern "C" tcuscan_status_t tcuscan_internal_compact_fused(const void *d_values, const void *d_mask, void *d_out, size_t n, unsigned *d_count,
                                                           void *d_ws, size_t ws_bytes, tcuscan_stream_t stream);   // tcuscan.hip
extern "C" tcuscan_status_t tcuscan_internal_bit_zero_counts(const void *d_keys, size_t n, unsigned *d_counts32, tcuscan_stream_t stream);
extern "C" tcuscan_status_t tcuscan_internal_split_pass(const void *d_keys, const void *d_vals, void *d_keys_out, void *d_vals_out, size_t n,
                                                        int bit, const unsigned *d_zeros_total, void *d_ws, size_t ws_bytes,
                                                        tcuscan_stream_t stream);

extern "C" tcuscan_status_t tcuscan_internal_digit_counts(const void *d_keys, size_t n, unsigned *d_counts64, tcuscan_stream_t stream);
extern "C" tcuscan_status_t tcuscan_internal_split4_pass(const void *d_keys, const void *d_vals, void *d_keys_out, void *d_vals_out, size_t n,
                                                         int bit, const unsigned *d_hist4, void *d_ws, size_t ws_bytes,
                                                         tcuscan_stream_t stream);

namespace {

constexpr int kThreads = 256;

// Four elements per thread: 16-byte loads of values and positions, one 4-byte load of the mask; the kept
// elements of a wavefront land in one contiguous run, so the scattered 4-byte stores coalesce.
__global__ __launch_bounds__(kThreads) void pack_kernel(const uint32_t *__restrict__ values, const int8_t *__restrict__ mask,
                                                        const int32_t *__restrict__ pos, uint32_t *__restrict__ out,
                                                        size_t n, uint32_t *count, bool vec)
{
    const size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t i0 = g * 4;
    if (i0 >= n) return;
    if (vec && i0 + 4 <= n) {
        const uint4 v = ((const uint4 *)values)[g];
        const uint4 p = ((const uint4 *)pos)[g];
        const uint32_t m = ((const uint32_t *)mask)[g];
        if (m & 0x000000FFu) out[p.x] = v.x;
        if (m & 0x0000FF00u) out[p.y] = v.y;
        if (m & 0x00FF0000u) out[p.z] = v.z;
        if (m & 0xFF000000u) out[p.w] = v.w;
    } else {
        for (size_t i = i0; i < n && i < i0 + 4; ++i)
            if (mask[i] != 0) out[(uint32_t)pos[i]] = values[i];
    }
    if (count && i0 + 4 >= n) *count = (uint32_t)pos[n - 1] + (mask[n - 1] != 0 ? 1u : 0u);
}

__global__ __launch_bounds__(kThreads) void bit_is_zero_kernel(const uint32_t *__restrict__ keys, int8_t *__restrict__ flags,
                                                               size_t n, int bit)
{
    // 16 keys per thread: one 16-byte store of flags
    const size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const size_t i0 = g * 16;
    if (i0 + 16 <= n) {
        uint32_t w[4];
        for (int q = 0; q < 4; ++q) {
            const uint4 k = ((const uint4 *)keys)[g * 4 + q];
            w[q] = (((k.x >> bit) & 1u) ^ 1u) | ((((k.y >> bit) & 1u) ^ 1u) << 8) | ((((k.z >> bit) & 1u) ^ 1u) << 16) |
                   ((((k.w >> bit) & 1u) ^ 1u) << 24);
        }
        ((uint4 *)flags)[g] = make_uint4(w[0], w[1], w[2], w[3]);
    } else {
        for (size_t i = i0; i < n; ++i) flags[i] = (int8_t)(((keys[i] >> bit) & 1u) ^ 1u);
    }
}

__global__ __launch_bounds__(kThreads) void split_scatter_kernel(const uint32_t *__restrict__ keys, const uint32_t *__restrict__ vals,
                                                                 const int8_t *__restrict__ flags, const int32_t *__restrict__ pos,
                                                                 uint32_t *__restrict__ keys_out, uint32_t *__restrict__ vals_out, size_t n)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const uint32_t zeros = (uint32_t)pos[n - 1] + (uint32_t)flags[n - 1];       // total number of keys whose bit is 0
    const uint32_t p = (uint32_t)pos[i];
    const uint32_t dst = flags[i] ? p : zeros + ((uint32_t)i - p);
    keys_out[dst] = keys[i];
    if (vals) vals_out[dst] = vals[i];
}

__global__ __launch_bounds__(kThreads) void copy_u32_kernel(const uint32_t *__restrict__ src, uint32_t *__restrict__ dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

unsigned blocks_for(size_t items) { return (unsigned)((items + kThreads - 1) / kThreads); }

// measurement / test knob, see tcuscan_set_sort_fusion: 1 fused passes on two bits, 2 fused passes on one bit, 0 three
// kernels per bit.  One atomic word, read once at the top of a sort, so that a change made by another thread while a
// sort is being enqueued cannot mix the forms (or their count tables) within that sort.
std::atomic<int> g_sort_form{1};

}  // namespace

extern "C" {

tcuscan_status_t tcuscan_compact_u32(const void *d_values, const void *d_mask, void *d_out, size_t n,
                                     void *d_positions, unsigned *d_count,
                                     void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    if (n == 0) return TCUSCAN_OK;
    if (n > 0xFFFFFFFFull) return TCUSCAN_ERR_UNSUPPORTED;                       // positions are 32-bit
    if (!d_values || !d_mask || !d_out) return TCUSCAN_ERR_INVALID_ARG;
    if (!d_positions) {                                                          // nobody wants the positions: one fused pass
        if (((uintptr_t)d_values % 4) || ((uintptr_t)d_out % 4) || ((uintptr_t)d_count % 4)) return TCUSCAN_ERR_INVALID_ARG;
        return tcuscan_internal_compact_fused(d_values, d_mask, d_out, n, d_count, d_ws, ws_bytes, stream);
    }
    if (((uintptr_t)d_values % 4) || ((uintptr_t)d_out % 4) || ((uintptr_t)d_positions % 4) || ((uintptr_t)d_count % 4))
        return TCUSCAN_ERR_INVALID_ARG;
    tcuscan_status_t st = tcuscan_exclusive(d_mask, d_positions, n, TCUSCAN_I8_I32, d_ws, ws_bytes, stream);
    if (st != TCUSCAN_OK) return st;
    const uint32_t *v = (const uint32_t *)d_values; const int8_t *m = (const int8_t *)d_mask;
    const int32_t *p = (const int32_t *)d_positions; uint32_t *o = (uint32_t *)d_out; uint32_t *c = d_count;
    bool vec = ((uintptr_t)d_values % 16) == 0 && ((uintptr_t)d_positions % 16) == 0 && ((uintptr_t)d_mask % 4) == 0;
    void *args[] = {&v, &m, &p, &o, &n, &c, &vec};
    hipError_t e = hipLaunchKernel((const void *)pack_kernel, dim3(blocks_for((n + 3) / 4)), dim3(kThreads), args, 0, (hipStream_t)stream);
    return e == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

tcuscan_status_t tcuscan_split_radix_sort_u32(void *d_keys, void *d_vals, size_t n, int bits,
                                              void *d_keys_tmp, void *d_vals_tmp, void *d_flags, void *d_positions,
                                              void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    if (bits < 0 || bits > 32) return TCUSCAN_ERR_INVALID_ARG;
    if (n <= 1 || bits == 0) return TCUSCAN_OK;
    if (n > 0xFFFFFFFFull) return TCUSCAN_ERR_UNSUPPORTED;
    if (!d_keys || !d_keys_tmp || !d_flags || !d_positions || (d_vals && !d_vals_tmp)) return TCUSCAN_ERR_INVALID_ARG;
    if (((uintptr_t)d_keys % 16) || ((uintptr_t)d_keys_tmp % 16) || ((uintptr_t)d_flags % 16) || ((uintptr_t)d_positions % 4) ||
        ((uintptr_t)d_vals % 4) || ((uintptr_t)d_vals_tmp % 4))
        return TCUSCAN_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    uint32_t *src_k = (uint32_t *)d_keys, *dst_k = (uint32_t *)d_keys_tmp;
    uint32_t *src_v = (uint32_t *)d_vals, *dst_v = (uint32_t *)d_vals_tmp;
    int8_t *flags = (int8_t *)d_flags;
    int32_t *pos = (int32_t *)d_positions;
    // Fused passes (the default): the mask and the positions are never written; the split kernel builds the flags from
    // the keys, scans them and scatters in one go -- two bits (four buckets) per pass, and one more pass on a single bit
    // when `bits` is odd.  How many keys have which digit at each position does not change when the keys are permuted:
    // it is counted once, up front, into the first 96 words of d_positions (64 digit counts, 32 zero-bit counts).  The
    // unfused form below (mask kernel, tcuscan_exclusive, scatter kernel, one bit per pass) remains for n < 96 and as
    // the plain statement of the reduction.
    const int form = g_sort_form.load(std::memory_order_relaxed);
    const bool fused = n >= 96 && form != 0;
    const int digit_bits = form == 2 ? 1 : 2;                                   // fused passes: bits per pass
    if (fused) {
        unsigned *hist = (unsigned *)d_positions, *zeros = hist + 64;
        tcuscan_status_t st = digit_bits == 2 ? tcuscan_internal_digit_counts(d_keys, n, hist, stream) : TCUSCAN_OK;
        if (st == TCUSCAN_OK && (digit_bits != 2 || (bits & 1))) st = tcuscan_internal_bit_zero_counts(d_keys, n, zeros, stream);
        if (st != TCUSCAN_OK) return st;
        for (int bit = 0; bit < bits;) {
            const int step = digit_bits == 2 && bits - bit >= 2 ? 2 : 1;
            st = step == 2 ? tcuscan_internal_split4_pass(src_k, src_v, dst_k, dst_v, n, bit, hist + 4 * (bit / 2), d_ws, ws_bytes, stream)
                           : tcuscan_internal_split_pass(src_k, src_v, dst_k, dst_v, n, bit, zeros + bit, d_ws, ws_bytes, stream);
            if (st != TCUSCAN_OK) return st;
            uint32_t *t = src_k; src_k = dst_k; dst_k = t;
            t = src_v; src_v = dst_v; dst_v = t;
            bit += step;
        }
    }
    for (int bit = 0; !fused && bit < bits; ++bit) {
        {
            const uint32_t *k = src_k; void *args[] = {&k, &flags, &n, &bit};
            if (hipLaunchKernel((const void *)bit_is_zero_kernel, dim3(blocks_for((n + 15) / 16)), dim3(kThreads), args, 0, s) != hipSuccess)
                return TCUSCAN_ERR_HIP;
        }
        tcuscan_status_t st = tcuscan_exclusive(flags, pos, n, TCUSCAN_I8_I32, d_ws, ws_bytes, stream);
        if (st != TCUSCAN_OK) return st;
        {
            const uint32_t *k = src_k, *v = src_v; const int8_t *f = flags; const int32_t *p = pos;
            void *args[] = {&k, &v, &f, &p, &dst_k, &dst_v, &n};
            if (hipLaunchKernel((const void *)split_scatter_kernel, dim3(blocks_for(n)), dim3(kThreads), args, 0, s) != hipSuccess)
                return TCUSCAN_ERR_HIP;
        }
        uint32_t *t = src_k; src_k = dst_k; dst_k = t;
        t = src_v; src_v = dst_v; dst_v = t;
    }
    if (src_k != (uint32_t *)d_keys) {                                          // odd number of passes: bring the result home
        const uint32_t *a = src_k; uint32_t *b = (uint32_t *)d_keys;
        void *args[] = {&a, &b, &n};
        if (hipLaunchKernel((const void *)copy_u32_kernel, dim3(blocks_for(n)), dim3(kThreads), args, 0, s) != hipSuccess) return TCUSCAN_ERR_HIP;
        if (d_vals) {
            const uint32_t *av = src_v; uint32_t *bv = (uint32_t *)d_vals;
            void *args2[] = {&av, &bv, &n};
            if (hipLaunchKernel((const void *)copy_u32_kernel, dim3(blocks_for(n)), dim3(kThreads), args2, 0, s) != hipSuccess) return TCUSCAN_ERR_HIP;
        }
    }
    return TCUSCAN_OK;
}

}  // extern "C"

extern "C" tcuscan_status_t tcuscan_set_sort_fusion(int fused)
{
    if (fused < 0 || fused > 2) return TCUSCAN_ERR_INVALID_ARG;
    g_sort_form.store(fused, std::memory_order_relaxed);
    return TCUSCAN_OK;
}
