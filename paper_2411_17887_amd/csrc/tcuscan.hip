// tcuscan: prefix sums as triangular-matrix products on the gfx950 MFMA units.
//
// One kernel does the whole scan in a single pass over HBM (read every input once,
// write every output once).  Per workgroup tile:
//
//   level 0  (Algorithm 1, up-sweep t = 0; BatchMatMul with L_s)
//            A 1 KiB run of input is viewed column-major as 16 columns of S consecutive
//            elements (S = 16 / 32 / 64 for 4 / 2 / 1-byte inputs).  Each column is
//            replaced by its local prefix sums by an MFMA  D = L * T  whose constant left
//            operand holds rows of the all-ones lower-triangular matrix (strictly lower
//            for the exclusive scan).  Data reach the MFMA operand layout through LDS:
//            global loads are 128-bit and fully coalesced, the LDS read-back gives lane
//            (j, c) the j-th quarter of column c.
//   level 1  (up-sweep t = 1 and its down-sweep)   the 16 column totals of a tile sit in
//            one 16-lane DPP row; a row_shr scan turns them into per-column carries.
//   level 2  tile totals inside a wavefront, wavefront totals through LDS.
//   level 3+ (remaining up-/down-sweep rounds; Section 2.2 steps 2-4 for lengths that are
//            not powers of s)  one 64-bit status word per workgroup tile, published with
//            relaxed agent-scope atomics and resolved by a decoupled look-back.
//   down-sweep  (B_s: broadcast-add of a carry)  is a vector add, as the paper's
//            discussion section recommends, fused before the store.
//   store    results go back through LDS so that every lane writes 16 contiguous bytes.
//
// The C entry points at the bottom validate arguments on the host and launch this kernel.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tcuscan.h"

namespace {

typedef float        f32x4  __attribute__((ext_vector_type(4)));
typedef int          i32x4  __attribute__((ext_vector_type(4)));
typedef _Float16     f16x8  __attribute__((ext_vector_type(8)));
typedef __bf16       bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4  __attribute__((ext_vector_type(4)));   // one 16-byte granule

constexpr int kWaves   = 4;           // wavefronts per workgroup
constexpr int kThreads = 64 * kWaves;

// Workspace header (256 bytes), followed by one 64-bit status word per tile.
struct WsHeader {
    uint32_t epoch;    // number of completed calls (mod 2^30 - 1); tags the status words
    uint32_t fault;    // sticky: a look-back wait hit its spin bound
    uint32_t pad[62];
};
static_assert(sizeof(WsHeader) == 256, "header size");

constexpr uint32_t kStateAggregate = 1u;   // value = total of this tile only
constexpr uint32_t kStatePrefix    = 2u;   // value = total of this tile and all before it in the row
constexpr uint32_t kEpochMod       = (1u << 30) - 1u;
constexpr uint32_t kSpinLimit      = 1u << 24;   // look-back polls before giving up (seconds of waiting)

struct Params {
    const void *in;
    void       *out;
    uint64_t    rows, cols;
    uint32_t    tiles_per_row, num_tiles;
    WsHeader   *ws;          // null when tiles_per_row == 1
};

// ---------------------------------------------------------------- small helpers

template <class To, class From> __device__ __forceinline__ To bits(From v) { return __builtin_bit_cast(To, v); }

template <int CTRL> __device__ __forceinline__ uint32_t dpp0(uint32_t v)
{   // lanes whose DPP source does not exist receive 0
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
constexpr int kRowShr = 0x110;   // DPP control: shift right by n lanes inside each row of 16

__device__ __forceinline__ float    acc_add(float a, float b)       { return a + b; }
__device__ __forceinline__ uint32_t acc_add(uint32_t a, uint32_t b) { return a + b; }
__device__ __forceinline__ uint32_t acc_bits(float a)    { return bits<uint32_t>(a); }
__device__ __forceinline__ uint32_t acc_bits(uint32_t a) { return a; }
template <class A> __device__ __forceinline__ A acc_from_bits(uint32_t b);
template <> __device__ __forceinline__ float    acc_from_bits<float>(uint32_t b)    { return bits<float>(b); }
template <> __device__ __forceinline__ uint32_t acc_from_bits<uint32_t>(uint32_t b) { return b; }

template <class A, int CTRL> __device__ __forceinline__ A dpp_shr(A v) { return acc_from_bits<A>(dpp0<CTRL>(acc_bits(v))); }

template <class A> __device__ __forceinline__ A wave_sum(A v)
{
    for (int m = 32; m >= 1; m >>= 1) {
        uint32_t o = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((__lane_id()) ^ m) << 2), (int)acc_bits(v));
        v = acc_add(v, acc_from_bits<A>(o));
    }
    return v;
}

template <class A> __device__ __forceinline__ A lane_value(A v, int src_lane)
{   // every lane receives v of lane src_lane (per-lane selectable source)
    return acc_from_bits<A>((uint32_t)__builtin_amdgcn_ds_bpermute(src_lane << 2, (int)acc_bits(v)));
}

template <class A> __device__ __forceinline__ A uniform_from_lane(A v, int lane)
{   // wave-uniform copy of one lane's value
    return acc_from_bits<A>((uint32_t)__builtin_amdgcn_readlane((int)acc_bits(v), lane));
}

// ------------------------------------------------------------------- dtype traits
//
// A tile is 64 granules of 16 bytes.  Lane (j, c) = (lane / 16, lane % 16) feeds the MFMA
// with granule 4c + j, i.e. the j-th quarter of column c; the K slot of element i of that
// granule pairs with the same (j, i) slot of the constant operand, so the constant is
// built as  A[row][slot(j, i)] = [pos(j, i) <= row]  (or < for the exclusive scan) with
// pos = position of the element inside its column.  Output block p holds rows
// 16p .. 16p+15; lane (q, c) register r of block p is row 16p + 4q + r of column c.

template <int DT> struct Tr;

template <> struct Tr<TCUSCAN_F16_F32> {
    using acc = float; using acc4 = f32x4;
    static constexpr int kEsz = 2, kG = 8, kBlocks = 2;
    struct AConst { f16x8 a[kBlocks]; };
    static __device__ AConst make(int lane, bool excl)
    {
        AConst A; int m = lane & 15, j = lane >> 4;
        for (int p = 0; p < kBlocks; ++p)
            for (int i = 0; i < kG; ++i) {
                int pos = kG * j + i, row = 16 * p + m;
                A.a[p][i] = (_Float16)((excl ? pos < row : pos <= row) ? 1.0f : 0.0f);
            }
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int, bool, acc4 (&d)[kBlocks])
    {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        f16x8 bv = bits<f16x8>(b);
        for (int p = 0; p < kBlocks; ++p) d[p] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A.a[p], bv, z, 0, 0, 0);
    }
    static __device__ __forceinline__ acc last(u32x4 b) { return (float)bits<f16x8>(b)[kG - 1]; }
};

template <> struct Tr<TCUSCAN_BF16_F32> {
    using acc = float; using acc4 = f32x4;
    static constexpr int kEsz = 2, kG = 8, kBlocks = 2;
    struct AConst { bf16x8 a[kBlocks]; };
    static __device__ AConst make(int lane, bool excl)
    {
        AConst A; int m = lane & 15, j = lane >> 4;
        u32x4 w[kBlocks];
        for (int p = 0; p < kBlocks; ++p) {
            w[p] = u32x4{0u, 0u, 0u, 0u};
            for (int i = 0; i < kG; ++i) {
                int pos = kG * j + i, row = 16 * p + m;
                uint32_t one = (excl ? pos < row : pos <= row) ? 0x3F80u : 0u;     // bf16 1.0
                w[p][i >> 1] |= one << (16 * (i & 1));
            }
            A.a[p] = bits<bf16x8>(w[p]);
        }
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int, bool, acc4 (&d)[kBlocks])
    {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        bf16x8 bv = bits<bf16x8>(b);
        for (int p = 0; p < kBlocks; ++p) d[p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A.a[p], bv, z, 0, 0, 0);
    }
    static __device__ __forceinline__ acc last(u32x4 b) { return bits<float>(b[3] & 0xFFFF0000u); }
};

template <> struct Tr<TCUSCAN_I8_I32> {
    using acc = uint32_t; using acc4 = i32x4;
    static constexpr int kEsz = 1, kG = 16, kBlocks = 4;
    struct AConst { i32x4 a[kBlocks]; };
    static __device__ AConst make(int lane, bool excl)
    {
        AConst A; int m = lane & 15, j = lane >> 4;
        for (int p = 0; p < kBlocks; ++p) {
            A.a[p] = i32x4{0, 0, 0, 0};
            for (int i = 0; i < kG; ++i) {
                int pos = kG * j + i, row = 16 * p + m;
                int one = (excl ? pos < row : pos <= row) ? 1 : 0;
                A.a[p][i >> 2] |= one << (8 * (i & 3));
            }
        }
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int, bool, acc4 (&d)[kBlocks])
    {
        const i32x4 z = {0, 0, 0, 0};
        i32x4 bv = bits<i32x4>(b);
        for (int p = 0; p < kBlocks; ++p) d[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A.a[p], bv, z, 0, 0, 0);
    }
    static __device__ __forceinline__ acc last(u32x4 b) { return (uint32_t)(int32_t)(int8_t)(b[3] >> 24); }
};

template <> struct Tr<TCUSCAN_F32_F32> {
    using acc = float; using acc4 = f32x4;
    static constexpr int kEsz = 4, kG = 4, kBlocks = 1;
    // The K = 4 product p takes element p of every lane's granule: slot (j, p) <-> position 4j + p.
    struct AConst { float a[4]; };
    static __device__ AConst make(int lane, bool excl)
    {
        AConst A; int m = lane & 15, j = lane >> 4;
        for (int p = 0; p < 4; ++p) { int pos = 4 * j + p; A.a[p] = (excl ? pos < m : pos <= m) ? 1.0f : 0.0f; }
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int, bool, acc4 (&d)[kBlocks])
    {
        f32x4 r = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < 4; ++p) r = __builtin_amdgcn_mfma_f32_16x16x4f32(A.a[p], bits<float>(b[p]), r, 0, 0, 0);
        d[0] = r;
    }
    static __device__ __forceinline__ acc last(u32x4 b) { return bits<float>(b[3]); }
};

template <> struct Tr<TCUSCAN_I32_I32> {
    using acc = uint32_t; using acc4 = i32x4;
    static constexpr int kEsz = 4, kG = 4, kBlocks = 1;
    // int32 has no MFMA of its own: x = sum_p 2^(8p) * byte_p(x) (mod 2^32), every byte plane is
    // scanned by an i8 MFMA and the planes are recombined with shifts.  The i8 MFMA is signed, so
    // byte b enters as b - 128 (bit 7 flipped) and 128 * (number of summed elements) is added back.
    struct AConst { long a; };
    static __device__ AConst make(int lane, bool excl)
    {
        int m = lane & 15, j = lane >> 4; uint32_t lo = 0;
        for (int i = 0; i < 4; ++i) { int pos = 4 * j + i; lo |= ((excl ? pos < m : pos <= m) ? 1u : 0u) << (8 * i); }
        AConst A; A.a = (long)(uint64_t)lo;       // K slots 4..7 of every lane are unused (zero on both sides)
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int lane, bool excl, acc4 (&d)[kBlocks])
    {
        const i32x4 z = {0, 0, 0, 0};
        uint32_t x0 = b[0] ^ 0x80808080u, x1 = b[1] ^ 0x80808080u, x2 = b[2] ^ 0x80808080u, x3 = b[3] ^ 0x80808080u;
        i32x4 pl[4];
        for (int p = 0; p < 4; ++p) {
            uint32_t lo = __builtin_amdgcn_perm(x1, x0, 0x0c0c0000u | ((4u + p) << 8) | (uint32_t)p);
            uint32_t hi = __builtin_amdgcn_perm(x3, x2, 0x00000c0cu | ((4u + p) << 24) | ((uint32_t)p << 16));
            pl[p] = __builtin_amdgcn_mfma_i32_16x16x32_i8(A.a, (long)(uint64_t)(lo | hi), z, 0, 0, 0);
        }
        int q = lane >> 4;
        for (int r = 0; r < 4; ++r) {
            uint32_t cnt = (uint32_t)(4 * q + r) + (excl ? 0u : 1u);          // elements summed into row 4q + r
            uint32_t v = (uint32_t)pl[0][r] + ((uint32_t)pl[1][r] << 8) + ((uint32_t)pl[2][r] << 16) + ((uint32_t)pl[3][r] << 24);
            d[0][r] = (int)(v + cnt * 0x80808080u);                           // 128 * cnt on every byte plane
        }
    }
    static __device__ __forceinline__ acc last(u32x4 b) { return b[3]; }
};

// LDS staging positions (in granules).  One pad granule per 2^shift granules keeps both the
// linear (lane l <-> granule l) and the operand-order (lane (j,c) <-> granule 4c + j, or the
// output order) access patterns spread over the banks.
template <int SHIFT> __device__ __forceinline__ int padded(int g) { return g + (g >> SHIFT); }

// ------------------------------------------------------------------------ carry chain

__device__ __forceinline__ uint64_t status_word(uint32_t tag, uint32_t state, uint32_t value_bits)
{
    return ((uint64_t)((tag << 2) | state) << 32) | value_bits;
}

// Exclusive prefix of tile `tr` of its row: sum of the totals of tiles 0 .. tr-1, found by walking
// back over published status words 64 at a time.  Called by all 64 lanes of one wavefront.
template <class A>
__device__ A look_back(const uint64_t *row_status, int tr, uint32_t tag, WsHeader *ws)
{
    const int lane = __lane_id();
    A sum = acc_from_bits<A>(0u);
    for (int base = tr - 1; base >= 0; base -= 64) {
        const int idx = base - lane;
        uint32_t state = kStatePrefix, vbits = 0u;          // lanes before the row start count as "prefix 0"
        if (idx >= 0) {
            uint32_t spins = 0;
            for (;;) {
                uint64_t w = __hip_atomic_load(row_status + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                uint32_t f = (uint32_t)(w >> 32);
                if ((f >> 2) == tag) { state = f & 3u; vbits = (uint32_t)w; break; }
                if (++spins > kSpinLimit) {               // never in correct operation: give up instead of hanging
                    __hip_atomic_store(&ws->fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
        }
        const uint64_t have_prefix = __ballot(state == kStatePrefix);   // never 0 in the last window
        const int first = have_prefix ? __builtin_ctzll(have_prefix) : 63;
        A v = acc_from_bits<A>(lane <= first ? vbits : 0u);
        sum = acc_add(sum, wave_sum(v));
        if (have_prefix) break;
    }
    return sum;
}

// ----------------------------------------------------------------------------- kernel

template <int DT, int EPW, bool EXCL>
__global__ __launch_bounds__(kThreads) void scan_kernel(Params P)
{
    using T = Tr<DT>;
    using A = typename T::acc;
    using A4 = typename T::acc4;
    constexpr int kG = T::kG;                       // elements per input granule
    constexpr int kS = 4 * kG;                      // column length
    constexpr int kTileElems = 64 * kG;             // one MFMA tile = 1 KiB of input
    constexpr int kTPW = EPW / kTileElems;          // MFMA tiles per wavefront
    constexpr int kBlocks = T::kBlocks;
    constexpr int kOutGran = EPW / 4;               // output granules per wavefront
    constexpr int kOutShift = (kS == 64) ? 4 : 3;
    constexpr int kStage = kOutGran + (kOutGran >> kOutShift) + 1;
    static_assert(kTPW >= 1 && kTPW * kTileElems == EPW, "EPW must be a multiple of the MFMA tile");
    constexpr uint32_t kWgElems = EPW * kWaves;

    __shared__ u32x4 stage[kWaves][kStage];
    __shared__ uint32_t s_wave_total[kWaves];
    __shared__ uint32_t s_bcast;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, j = lane >> 4;         // operand order: column, quarter (also output row group q)

    // ---- which tile.  Tiles are taken in workgroup-index order: a tile only ever waits for tiles with
    // a smaller index, which the hardware dispatched earlier (or at the same time), so the lowest
    // unfinished tile is always running and the chain cannot stall.  (A shared ticket counter would
    // guarantee the same without that assumption, but one contended atomic per tile caps the whole
    // kernel at the device's single-address atomic rate.)  Status words carry the call's tag, so
    // words left over from earlier calls read as "not published yet" and need no clearing.
    const bool chained = P.tiles_per_row > 1;
    const uint32_t tile = blockIdx.x;
    const uint32_t tag = chained ? __hip_atomic_load(&P.ws->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u : 0u;
    const uint64_t row = tile / P.tiles_per_row;
    const uint32_t tr = tile - (uint32_t)row * P.tiles_per_row;
    const uint64_t row_base = row * P.cols;                          // first element of the row
    const uint64_t tile_base = (uint64_t)tr * kWgElems;             // first element of the tile inside the row
    const uint64_t wave_base = tile_base + (uint64_t)wave * EPW;    // first element of this wavefront's run

    const char *in_row  = (const char *)P.in + row_base * T::kEsz;
    char       *out_row = (char *)P.out + row_base * 4;
    const bool in_vec  = (((uintptr_t)in_row) & 15) == 0;
    const bool out_vec = (((uintptr_t)out_row) & 15) == 0;

    const typename T::AConst Aop = T::make(lane, EXCL);

    // ---- a1: coalesced 128-bit loads, zero-filled past the end of the row (BatchMatMul's zero-pad)
    u32x4 g[kTPW];
#pragma unroll
    for (int t = 0; t < kTPW; ++t) {
        const uint64_t e0 = wave_base + (uint64_t)t * kTileElems + (uint64_t)lane * kG;
        if (in_vec && e0 + kG <= P.cols) {
            g[t] = *(const u32x4 *)(in_row + e0 * T::kEsz);
        } else {
            uint32_t w[4] = {0u, 0u, 0u, 0u};
            for (int i = 0; i < kG; ++i) {
                if (e0 + i < P.cols) {
                    uint32_t v;
                    if (T::kEsz == 4)      v = ((const uint32_t *)in_row)[e0 + i];
                    else if (T::kEsz == 2) v = ((const uint16_t *)in_row)[e0 + i];
                    else                   v = ((const uint8_t *)in_row)[e0 + i];
                    w[(i * T::kEsz) >> 2] |= v << (8 * ((i * T::kEsz) & 3));
                }
            }
            g[t] = u32x4{w[0], w[1], w[2], w[3]};
        }
    }

    // ---- to operand order through LDS (wave-private region, no workgroup barrier needed)
#pragma unroll
    for (int t = 0; t < kTPW; ++t) stage[wave][padded<3>(64 * t + lane)] = g[t];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    u32x4 b[kTPW];
#pragma unroll
    for (int t = 0; t < kTPW; ++t) b[t] = stage[wave][padded<3>(64 * t + 4 * c + j)];

    // ---- a2: local scans of every column on the MFMA unit;  a3: level 1 on DPP
    A4 d[kTPW][kBlocks];
    A colcarry[kTPW];       // exclusive prefix of the column totals inside the tile, per lane
    A tile_off[kTPW];       // exclusive prefix of the tile totals inside the wavefront (uniform)
    A wave_total = acc_from_bits<A>(0u);
#pragma unroll
    for (int t = 0; t < kTPW; ++t) {
        T::mma(Aop, b[t], lane, EXCL, d[t]);
        // column totals live in row S-1 = lanes 48..63, last register of the last block
        A tot = acc_from_bits<A>((uint32_t)bits<u32x4>(d[t][kBlocks - 1])[3]);
        if (EXCL) tot = acc_add(tot, T::last(b[t]));     // the strictly-lower product leaves the last element out
        A e = dpp_shr<A, kRowShr + 1>(tot);              // shift by one column -> exclusive
        e = acc_add(e, dpp_shr<A, kRowShr + 1>(e));
        e = acc_add(e, dpp_shr<A, kRowShr + 2>(e));
        e = acc_add(e, dpp_shr<A, kRowShr + 4>(e));
        e = acc_add(e, dpp_shr<A, kRowShr + 8>(e));
        const A ttot = uniform_from_lane(acc_add(e, tot), 63);
        colcarry[t] = lane_value(e, 48 + c);             // row 3 -> all four rows
        tile_off[t] = wave_total;
        wave_total = acc_add(wave_total, ttot);
    }

    // ---- level 2: wavefront totals through LDS
    if (lane == 0) s_wave_total[wave] = acc_bits(wave_total);
    __syncthreads();
    A wave_off = acc_from_bits<A>(0u), wg_total = acc_from_bits<A>(0u);
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const A v = acc_from_bits<A>(s_wave_total[w]);
        if (w < wave) wave_off = acc_add(wave_off, v);
        wg_total = acc_add(wg_total, v);
    }

    // ---- a4: carry chain between workgroup tiles of the same row
    A prefix = acc_from_bits<A>(0u);
    if (chained) {
        uint64_t *row_status = (uint64_t *)(P.ws + 1) + row * P.tiles_per_row;
        if (wave == 0) {
            if (tr == 0) {
                if (lane == 0)
                    __hip_atomic_store(row_status, status_word(tag, kStatePrefix, acc_bits(wg_total)),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                if (lane == 0)
                    __hip_atomic_store(row_status + tr, status_word(tag, kStateAggregate, acc_bits(wg_total)),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                prefix = look_back<A>(row_status, (int)tr, tag, P.ws);
                if (lane == 0)
                    __hip_atomic_store(row_status + tr, status_word(tag, kStatePrefix, acc_bits(acc_add(prefix, wg_total))),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (lane == 0) {
                s_bcast = acc_bits(prefix);
                // Single row: once the last tile has resolved its look-back every tile of this call has
                // read the epoch, so it can be advanced here.  Several rows: a trailing kernel does it.
                if (P.rows == 1 && tr == P.tiles_per_row - 1)
                    __hip_atomic_store(&P.ws->epoch, tag % kEpochMod, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
        prefix = acc_from_bits<A>(s_bcast);
    }

    // ---- a5: down-sweep = add the carry of (row prefix, wavefront, tile, column) to the local scans
    const A wave_carry = acc_add(prefix, wave_off);
#pragma unroll
    for (int t = 0; t < kTPW; ++t) {
        const A carry = acc_add(acc_add(wave_carry, tile_off[t]), colcarry[t]);
#pragma unroll
        for (int p = 0; p < kBlocks; ++p) {
            u32x4 v = bits<u32x4>(d[t][p]);
            for (int r = 0; r < 4; ++r) v[r] = acc_bits(acc_add(carry, acc_from_bits<A>(v[r])));
            // a6: stage in output order: rows 16p + 4q .. +3 of column c are 4 consecutive outputs
            const int og = t * (kTileElems / 4) + (kS / 4) * c + 4 * p + j;
            stage[wave][padded<kOutShift>(og)] = v;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int k = 0; k < kOutGran / 64; ++k) {
        const int og = 64 * k + lane;
        const u32x4 v = stage[wave][padded<kOutShift>(og)];
        const uint64_t e0 = wave_base + 4ull * og;
        if (out_vec && e0 + 4 <= P.cols) {
            *(u32x4 *)(out_row + e0 * 4) = v;
        } else {
            for (int r = 0; r < 4; ++r)
                if (e0 + r < P.cols) ((uint32_t *)out_row)[e0 + r] = v[r];
        }
    }

}

// Advances the workspace epoch after a multi-row call (stream-ordered behind the scan kernel).
__global__ void advance_epoch_kernel(WsHeader *ws)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) ws->epoch = (ws->epoch + 1u) % kEpochMod;
}

__global__ void fill_zero_kernel(uint32_t *p, size_t words)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0u;
}

// ------------------------------------------------------------------------ host side

constexpr int kEPW = 2048;                               // elements per wavefront
constexpr size_t kTile = (size_t)kEPW * kWaves;          // elements per workgroup tile

bool valid_dtype(int dt) { return dt >= 0 && dt <= 4; }
size_t in_size(int dt) { return dt == TCUSCAN_I8_I32 ? 1 : (dt == TCUSCAN_F16_F32 || dt == TCUSCAN_BF16_F32) ? 2 : 4; }

template <int DT> hipError_t launch_dt(const Params &P, bool excl, hipStream_t s)
{
    // hipLaunchKernel reports this launch's own status (hipGetLastError could return a stale,
    // unrelated code left behind by another library's polling calls).
    Params p = P;
    void *args[] = {&p};
    const void *fn = excl ? (const void *)scan_kernel<DT, kEPW, true> : (const void *)scan_kernel<DT, kEPW, false>;
    hipError_t e = hipLaunchKernel(fn, dim3(P.num_tiles), dim3(kThreads), args, 0, s);
    if (e == hipSuccess && P.ws && P.rows > 1) {
        WsHeader *ws = P.ws;
        void *a2[] = {&ws};
        e = hipLaunchKernel((const void *)advance_epoch_kernel, dim3(1), dim3(64), a2, 0, s);
    }
    return e;
}

tcuscan_status_t run(const void *d_in, void *d_out, size_t rows, size_t cols, int dt, int exclusive,
                     void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    if (!valid_dtype(dt)) return TCUSCAN_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return TCUSCAN_OK;
    if (!d_in || !d_out) return TCUSCAN_ERR_INVALID_ARG;
    if (((uintptr_t)d_in % in_size(dt)) != 0 || ((uintptr_t)d_out % 4) != 0) return TCUSCAN_ERR_INVALID_ARG;
    if (d_in == d_out && in_size(dt) != 4) return TCUSCAN_ERR_INVALID_ARG;
    const size_t tpr = (cols + kTile - 1) / kTile;
    if (rows > 0x7FFFFFFFull / tpr) return TCUSCAN_ERR_UNSUPPORTED;     // tile index must fit 31 bits
    const size_t need = tcuscan_workspace_bytes(rows, cols, (tcuscan_dtype_t)dt);
    if (need && (!d_ws || ws_bytes < need || ((uintptr_t)d_ws % 8) != 0)) return TCUSCAN_ERR_WORKSPACE;

    Params P;
    P.in = d_in; P.out = d_out; P.rows = rows; P.cols = cols;
    P.tiles_per_row = (uint32_t)tpr; P.num_tiles = (uint32_t)(rows * tpr);
    P.ws = need ? (WsHeader *)d_ws : nullptr;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    switch (dt) {
    case TCUSCAN_I32_I32:  e = launch_dt<TCUSCAN_I32_I32>(P, exclusive != 0, s); break;
    case TCUSCAN_F16_F32:  e = launch_dt<TCUSCAN_F16_F32>(P, exclusive != 0, s); break;
    case TCUSCAN_I8_I32:   e = launch_dt<TCUSCAN_I8_I32>(P, exclusive != 0, s); break;
    case TCUSCAN_F32_F32:  e = launch_dt<TCUSCAN_F32_F32>(P, exclusive != 0, s); break;
    default:               e = launch_dt<TCUSCAN_BF16_F32>(P, exclusive != 0, s); break;
    }
    return e == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

}  // namespace

extern "C" {

size_t tcuscan_tile_elems(tcuscan_dtype_t dt) { return valid_dtype((int)dt) ? kTile : 0; }

size_t tcuscan_workspace_bytes(size_t rows, size_t cols, tcuscan_dtype_t dt)
{
    if (!valid_dtype((int)dt) || rows == 0 || cols == 0) return 0;
    const size_t tpr = (cols + kTile - 1) / kTile;
    if (tpr <= 1) return 0;
    return sizeof(WsHeader) + 8 * rows * tpr;
}

tcuscan_status_t tcuscan_workspace_init(void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    if (ws_bytes == 0) return TCUSCAN_OK;
    if (!d_ws || ((uintptr_t)d_ws % 8) != 0 || (ws_bytes % 4) != 0) return TCUSCAN_ERR_INVALID_ARG;
    size_t words = ws_bytes / 4;
    uint32_t *p = (uint32_t *)d_ws;
    void *args[] = {&p, &words};
    hipError_t e = hipLaunchKernel((const void *)fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256),
                                   args, 0, (hipStream_t)stream);
    return e == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

tcuscan_status_t tcuscan_inclusive(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt,
                                   void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    return run(d_in, d_out, n ? 1 : 0, n, (int)dt, 0, d_ws, ws_bytes, stream);
}

tcuscan_status_t tcuscan_exclusive(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt,
                                   void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    return run(d_in, d_out, n ? 1 : 0, n, (int)dt, 1, d_ws, ws_bytes, stream);
}

tcuscan_status_t tcuscan_batched(const void *d_in, void *d_out, size_t rows, size_t cols,
                                 tcuscan_dtype_t dt, int exclusive,
                                 void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    return run(d_in, d_out, rows, cols, (int)dt, exclusive, d_ws, ws_bytes, stream);
}

tcuscan_status_t tcuscan_workspace_fault(const void *d_ws, tcuscan_stream_t stream, unsigned *h_fault)
{
    if (!d_ws || !h_fault) return TCUSCAN_ERR_INVALID_ARG;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return TCUSCAN_ERR_HIP;
    const WsHeader *h = (const WsHeader *)d_ws;
    if (hipMemcpy(h_fault, &h->fault, sizeof(unsigned), hipMemcpyDeviceToHost) != hipSuccess) return TCUSCAN_ERR_HIP;
    return TCUSCAN_OK;
}

const char *tcuscan_status_string(tcuscan_status_t st)
{
    switch (st) {
    case TCUSCAN_OK:              return "ok";
    case TCUSCAN_ERR_INVALID_ARG: return "invalid argument";
    case TCUSCAN_ERR_UNSUPPORTED: return "unsupported dtype or size";
    case TCUSCAN_ERR_WORKSPACE:   return "workspace missing or too small";
    case TCUSCAN_ERR_HIP:         return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
