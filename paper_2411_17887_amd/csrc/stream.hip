// Measurement only: streaming kernels with a scan's memory traffic and none of its work.
//
// A scan reads every input once and writes every output once, so the best it can do is what the memory system
// gives a kernel that does nothing else with the same read : write mix -- 1 : 4 bytes for 8-bit inputs (32-bit
// outputs), 2 : 4 for 16-bit inputs, 4 : 4 for 32-bit inputs; write-only is the limit of wider and wider outputs.
// These kernels are that yardstick: every lane loads whole 16-byte granules and stores 16-byte groups, a wavefront's
// load or store instruction covers 1 KiB of consecutive memory, stores are non-temporal, nothing waits for anything
// but its own loads -- or, in the variants with a pause, a fixed number of cycles more once they have arrived (a scan
// computes between its loads and its stores; a streaming kernel that stores the moment its loads land is not the
// fastest one: 512 to 2048 cycles of pause lift the 2 : 4 mix from 6.1 to 6.5 TB/s).  The benchmark times them next to each scan configuration and reports the scan's bandwidth as a
// fraction of the best variant's; nothing else calls them.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tcuscan.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One workgroup = 256 lanes x U input granules; input granule i becomes output granules R * i .. R * i + R - 1,
// laid out so that the k-th store of a wavefront writes the k-th KiB of the wavefront's R KiB of output.
// R = 0: write-only (no input), U output granules per lane.
// RUNS: false -- the u-th load of the workgroup's four wavefronts covers 4 KiB of consecutive input (wavefronts
// interleaved); true -- every wavefront owns U KiB of consecutive input (what a scan tile looks like).
// The grid may be smaller than the number of chunks: a workgroup then walks over chunks grid-stride.
// PAUSE: s_sleep argument (units of 64 cycles) between the arrival of a chunk's loads and its stores; 0: none.
template <int U, int R, bool NTL, bool RUNS, int PAUSE = 0>
__global__ __launch_bounds__(256) void stream_kernel(const u32x4 *__restrict__ in, u32x4 *__restrict__ out, size_t n_in, size_t n_out,
                                                     size_t chunks)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (size_t chunk = blockIdx.x; chunk < chunks; chunk += gridDim.x) {
        const size_t base = chunk * 256 * U + (RUNS ? (size_t)wave * 64 * U + lane : threadIdx.x);
        constexpr size_t step = RUNS ? 64 : 256;
        if constexpr (R == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t i = base + (size_t)u * step;
                if (i < n_out) __builtin_nontemporal_store(u32x4{1u, 2u, 3u, (unsigned)i}, out + i);
            }
        } else {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t i = base + (size_t)u * step;
                v[u] = u32x4{0u, 0u, 0u, 0u};
                if (i < n_in) v[u] = NTL ? __builtin_nontemporal_load(in + i) : in[i];
            }
            if constexpr (PAUSE != 0) {
                __builtin_amdgcn_s_waitcnt(0);                  // every counter at zero: the loads have arrived
                __builtin_amdgcn_s_sleep(PAUSE);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t i = base + (size_t)u * step;
                const size_t wave_out = (i & ~(size_t)63) * R;
#pragma unroll
                for (int k = 0; k < R; ++k) {
                    const size_t o = wave_out + 64 * k + (i & 63);
                    if (i < n_in && o < n_out) __builtin_nontemporal_store(v[u] + (unsigned)k, out + o);
                }
            }
        }
    }
}

template <int U, int R, int PAUSE = 0> const void *stream_fn(bool ntl, bool runs)
{
    if (runs) return ntl ? (const void *)stream_kernel<U, R, true, true, PAUSE> : (const void *)stream_kernel<U, R, false, true, PAUSE>;
    return ntl ? (const void *)stream_kernel<U, R, true, false, PAUSE> : (const void *)stream_kernel<U, R, false, false, PAUSE>;
}
template <int R> const void *stream_fn_u(int log2u, bool ntl, bool runs, int pause)
{
    if (pause == 1) return log2u == 0 ? stream_fn<1, R, 8>(ntl, runs) : stream_fn<2, R, 8>(ntl, runs);
    if (pause == 2) return log2u == 0 ? stream_fn<1, R, 32>(ntl, runs) : stream_fn<2, R, 32>(ntl, runs);
    switch (log2u) {
    case 0:  return stream_fn<1, R>(ntl, runs);
    case 1:  return stream_fn<2, R>(ntl, runs);
    case 2:  return stream_fn<4, R>(ntl, runs);
    case 3:  return stream_fn<8, R>(ntl, runs);
    case 4:  return stream_fn<16, R>(ntl, runs);
    default: return stream_fn<32, R>(ntl, runs);
    }
}

}  // namespace

extern "C" tcuscan_status_t tcuscan_measure_stream(const void *d_in, void *d_out, size_t out_bytes, int in_bytes_per_out_word,
                                                   unsigned variant, tcuscan_stream_t stream)
{
    const int b = in_bytes_per_out_word;
    const int pause = (int)((variant >> 11) & 3u);         // 0: none, 1: 512 cycles, 2: 2048 cycles (1 or 2 loads per lane, with input only)
    if ((b != 0 && b != 1 && b != 2 && b != 4) || (variant & ~0x1F07u) || (variant & 7u) > 5u) return TCUSCAN_ERR_INVALID_ARG;
    if (pause == 3 || (pause != 0 && ((variant & 7u) > 1u || b == 0))) return TCUSCAN_ERR_INVALID_ARG;
    if (out_bytes == 0) return TCUSCAN_OK;
    if (!d_out || (b && !d_in) || ((uintptr_t)d_out % 16) || ((uintptr_t)d_in % 16) || (out_bytes % 64)) return TCUSCAN_ERR_INVALID_ARG;
    const int log2u = (int)(variant & 7u);
    const bool ntl = (variant & 0x100u) != 0, runs = (variant & 0x200u) != 0, resident = (variant & 0x400u) != 0;
    const int R = b ? 4 / b : 0;
    size_t n_out = out_bytes / 16, n_in = R ? n_out / R : 0;
    const size_t lanes = R ? n_in : n_out, per_wg = (size_t)256 << log2u;
    size_t chunks = (lanes + per_wg - 1) / per_wg;
    const size_t grid = resident && chunks > 2048 ? 2048 : chunks;         // resident: 8 workgroups per compute unit walk over the chunks
    if (grid > 0x7FFFFFFFull) return TCUSCAN_ERR_UNSUPPORTED;
    const void *fn = R == 4 ? stream_fn_u<4>(log2u, ntl, runs, pause) : R == 2 ? stream_fn_u<2>(log2u, ntl, runs, pause)
                   : R == 1 ? stream_fn_u<1>(log2u, ntl, runs, pause) : stream_fn_u<0>(log2u, false, runs, 0);
    const u32x4 *in = (const u32x4 *)d_in; u32x4 *out = (u32x4 *)d_out;
    void *args[] = {&in, &out, &n_in, &n_out, &chunks};
    return hipLaunchKernel(fn, dim3((unsigned)grid), dim3(256), args, 0, (hipStream_t)stream) == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}
