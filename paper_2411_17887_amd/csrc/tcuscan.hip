// tcuscan: prefix sums as triangular-matrix products on the gfx950 MFMA units.
//
// One kernel does the whole scan in a single pass over HBM (read every input once,
// write every output once).  Per workgroup tile the order of work is: load, reduce, publish
// the tile total, wait for the carry, scan, store -- the registers that wait for the carry hold
// the (narrow) inputs, not the (wide) outputs, so more elements per compute unit are in flight
// while the carry chain's latency is being paid.
//
//   level 0  (Algorithm 1, up-sweep t = 0; BatchMatMul with L_s)
//            A 1 KiB run of input is 64 granules of 16 bytes, s = 16 / 8 / 4 elements each for
//            1 / 2 / 4-byte inputs, and lane l of the wavefront loads granule l (128-bit, fully
//            coalesced).  Every granule is replaced by its local prefix sums by an MFMA
//            D = (I_4 (x) L_s) * T : the lane's granule is its share of the B operand as it is, the
//            constant left operand holds the rows of the all-ones lower-triangular blocks
//            (strictly lower for the exclusive scan) -- 64 s x s products per instruction group.
//            The tile total that is published early is the product with the all-ones matrix
//            (every row of the result is the row of column totals) for the MFMA-native types,
//            plain vector adds for 32-bit inputs.
//   level 1-2 (up-sweep t = 1, 2 and their down-sweep)   the 64 granule totals of a tile -- a second
//            product with a 0/1 matrix puts each where its carry is needed -- are scanned with DPP
//            row shifts inside 16-lane rows; the four row totals are wave-uniform.
//   level 3  tile totals inside a wavefront (a running carry), wavefront totals through LDS.
//   level 4+ (remaining up-/down-sweep rounds; Section 2.2 steps 2-4 for lengths that are
//            not powers of s)  one 64-bit status word per workgroup tile, published with
//            relaxed agent-scope atomics and resolved by a decoupled look-back.
//   down-sweep  (B_s: broadcast-add of a carry)  is a vector add, as the paper's
//            discussion section recommends, fused before the store.
//   store    straight from the MFMA result registers: the rows of the triangular blocks are dealt
//            to result rows so that each store instruction writes 1 KiB of consecutive outputs
//            (partial lines per instruction measured 30 % slower).  No data pass through LDS.
//
// Variants of the same kernel: reverse scans (suffix sums: upper triangular blocks, granules mirrored, the
// chain runs from the end of the row) and segmented scans (rows of different lengths stored back to back: a
// tile looks up its row in a map the host side builds with two small kernels and this library's own int32
// scan).  The C entry points at the bottom validate arguments on the host and launch these kernels.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "../../include/tcuscan.h"
#include "chain_tags.h"

namespace {

typedef float        f32x4  __attribute__((ext_vector_type(4)));
typedef int          i32x4  __attribute__((ext_vector_type(4)));
typedef _Float16     f16x8  __attribute__((ext_vector_type(8)));
typedef __bf16       bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4  __attribute__((ext_vector_type(4)));   // one 16-byte granule

constexpr int kWaves   = 4;           // wavefronts per workgroup of the short-row kernel (one row each)
constexpr int kThreads = 64 * kWaves;

// Workspace header (256 bytes), followed by one 64-bit status word per tile, each word alone in a
// 64-byte slot: thousands of tiles poll the words of the few hundred tiles in front of them, and with
// the words packed 8 to a line that traffic lands on a handful of memory channels (measured: 5-9 %
// of the whole kernel's run time).
constexpr size_t kStatusStride = 8;    // in 64-bit words
struct WsHeader {
    uint32_t fault;    // sticky: 1 = a look-back wait hit its spin bound, 2 = a segmented scan was given bad offsets
    uint32_t ticket;   // ticket policy only: the next tile index to hand out (cleared in front of every such call)
    uint32_t pad[62];
};
static_assert(sizeof(WsHeader) == 256, "header size");

constexpr uint32_t kStateAggregate = 1u;   // value = total of this tile only
constexpr uint32_t kStatePrefix    = 2u;   // value = total of this tile and all before it in the row
constexpr uint32_t kDefaultSpinLimit = 1u << 24;   // look-back polls before giving up (seconds of waiting)
constexpr uint32_t kNoTile           = 0xFFFFFFFFu;

struct Params {
    const void *in;
    void       *out;
    uint64_t    rows, cols;  // segmented scans: cols = number of elements of the arrays
    uint32_t    tiles_per_row, num_tiles;
    uint32_t    tag;         // this call's tag for the status words (30 bits; see chain_tags.h)
    uint32_t    ticket;      // non-zero: workgroups draw their tile index from the counter in the workspace header
    uint32_t    spin_limit;  // look-back polls per status word before the wait gives up and raises the fault word
    uint32_t    mute_tile;   // test hook: the tile with this index does not publish its status word (kNoTile: none)
    uint32_t    reverse;     // non-zero: suffix sums (every row is scanned from its end)
    WsHeader   *ws;          // null when tiles_per_row == 1
    // segmented scans only: what every tile has to know about its row (built by seg_desc_kernel)
    const struct TileDesc *tile_desc;
};

// One per tile of a segmented scan (32 bytes, read with one scalar load).
struct TileDesc {
    long long off;                 // first element of the tile's row
    unsigned long long len;        // length of the row
    uint32_t first_tile;           // index of the row's first tile
    uint32_t tiles_in_row;         // 0: no such tile (the grid is an upper bound)
    uint32_t pad[2];
};
static_assert(sizeof(TileDesc) == 32, "descriptor size");

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

// Sum over the 64 lanes, returned wave-uniform.  Row-local DPP shifts give every row's total in its
// lane 15; row_bcast15 / row_bcast31 fold the four row totals into lane 63.
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;
template <class A> __device__ __forceinline__ A wave_inclusive_scan(A v)
{   // lane l receives v[0] + ... + v[l]
    v = acc_add(v, dpp_shr<A, kRowShr + 1>(v));
    v = acc_add(v, dpp_shr<A, kRowShr + 2>(v));
    v = acc_add(v, dpp_shr<A, kRowShr + 4>(v));
    v = acc_add(v, dpp_shr<A, kRowShr + 8>(v));
    v = acc_add(v, acc_from_bits<A>((uint32_t)__builtin_amdgcn_update_dpp(0, (int)acc_bits(v), kRowBcast15, 0xa, 0xf, false)));
    v = acc_add(v, acc_from_bits<A>((uint32_t)__builtin_amdgcn_update_dpp(0, (int)acc_bits(v), kRowBcast31, 0xc, 0xf, false)));
    return v;
}
template <class A> __device__ __forceinline__ A wave_sum(A v)
{
    return acc_from_bits<A>((uint32_t)__builtin_amdgcn_readlane((int)acc_bits(wave_inclusive_scan(v)), 63));
}
constexpr int kWaveShr1 = 0x138;   // DPP control: shift right by one lane across the whole wavefront
template <class A> __device__ __forceinline__ A wave_shift_up(A v)
{   // lane l receives v[l - 1], lane 0 receives 0
    return dpp_shr<A, kWaveShr1>(v);
}

template <class A> __device__ __forceinline__ A uniform_from_lane(A v, int lane)
{   // wave-uniform copy of one lane's value
    return acc_from_bits<A>((uint32_t)__builtin_amdgcn_readlane((int)acc_bits(v), lane));
}

// ------------------------------------------------------------------- dtype traits
//
// A tile is 64 granules of 16 bytes (G elements each), and lane l = 16j + c loads granule l.  The MFMA
// takes lane (j, c)'s granule as K slots (j, 0..G-1) of column c of its B operand, so a column holds the
// four granules c, 16+c, 32+c, 48+c.  Level 0 (BatchMatMul with L_s, s = G) scans every granule by
// itself: the constant A operand is block-diagonal, row (j, i) = [same j, slot i' <= i]  (< for the
// exclusive scan) -- I_4 (x) L_G, 64 independent s x s products in one pass over the matrix unit.
//
// The rows are dealt to the MFMA's 16-row result blocks so that one store instruction of the wavefront
// writes 1 KiB of consecutive outputs.  Lane (q, c) register r of block p is result row 4q + r; it is
// made to be element 4 * sub(p, q) + r of granule (jmap(p, q), c):
//      8-bit  (G = 16, 4 blocks)   jmap = p,            sub = q
//     16-bit  (G =  8, 2 blocks)   jmap = 2p + q / 2,   sub = q % 2
//     32-bit  (G =  4, 1 block)    jmap = q,            sub = 0     (every lane keeps its own granule)
// so the four results of a lane in block p are outputs G * (16 jmap + c) + 4 sub .. +3 of the tile.
//
// A second constant operand ("tot") delivers the granule totals where they are needed: result row
// 4q + r of  tot * T  is the total of granule (jmap(r, q), c), i.e. register p of lane (q, c) is the total
// of the granule whose results the lane holds in block p.

template <int DT> struct Tr;

// 64-bit word whose `cnt` lowest slots of `bits_per_slot` bits hold `one` (a slot pattern repeated over
// the whole word is passed in), the rest zero: the part of a row of the triangular operand that falls
// into one half of a lane's granule.
__device__ __forceinline__ uint64_t low_slots(uint64_t ones, int cnt, int slots, int bits_per_slot)
{
    cnt = cnt < 0 ? 0 : (cnt > slots ? slots : cnt);
    return cnt == 0 ? 0ull : ones >> (bits_per_slot * (slots - cnt));
}
// the same with the `cnt` highest slots (rows of the upper triangular blocks of a reverse scan)
__device__ __forceinline__ uint64_t high_slots(uint64_t ones, int cnt, int slots, int bits_per_slot)
{
    cnt = cnt < 0 ? 0 : (cnt > slots ? slots : cnt);
    return cnt == 0 ? 0ull : (ones << (bits_per_slot * (slots - cnt))) & (slots * bits_per_slot == 64 ? ~0ull : ((1ull << (slots * bits_per_slot)) - 1));
}
// Row i of a G x G triangular block as two words of G/2 slots each: slots 0 .. i (forward) or i .. G-1 (reverse);
// the strict forms leave slot i out.
__device__ __forceinline__ void tri_row(uint64_t ones, int i, int G, int bits_per_slot, bool excl, bool rev, bool present,
                                        uint64_t &lo, uint64_t &hi)
{
    const int half = G / 2;
    if (!present) { lo = hi = 0; return; }
    if (!rev) {
        const int cnt = i + (excl ? 0 : 1);
        lo = low_slots(ones, cnt, half, bits_per_slot); hi = low_slots(ones, cnt - half, half, bits_per_slot);
    } else {
        const int cnt = G - i - (excl ? 1 : 0);
        hi = high_slots(ones, cnt, half, bits_per_slot); lo = high_slots(ones, cnt - half, half, bits_per_slot);
    }
}

// Shared by the two 16-bit types: which granule row / which half a result row of block p stands for.
struct Map16 {
    static __device__ __forceinline__ int jmap(int p, int q) { return 2 * p + (q >> 1); }
    static __device__ __forceinline__ int sub(int, int q) { return q & 1; }
};

// Operands of a 16-bit type as raw words; `one` is the 16-bit pattern of 1.0 repeated four times.
struct AWords16 { u32x4 a[2]; u32x4 ones; u32x4 tot; };
__device__ __forceinline__ AWords16 make16(int lane, bool excl, bool rev, uint64_t one)
{
    AWords16 A; const int m = lane & 15, jj = lane >> 4;       // this lane supplies row m, K slots (jj, 0..7)
    const uint32_t o = (uint32_t)one;
    A.ones = u32x4{o, o, o, o};
    for (int p = 0; p < 2; ++p) {
        const int j = Map16::jmap(p, m >> 2), i = 4 * Map16::sub(p, m >> 2) + (m & 3);
        uint64_t lo, hi;
        tri_row(one, i, 8, 16, excl, rev, jj == j, lo, hi);
        A.a[p] = u32x4{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
    }
    const int r = m & 3;
    const uint32_t t = (r < 2 && jj == Map16::jmap(r, m >> 2)) ? o : 0u;
    A.tot = u32x4{t, t, t, t};
    return A;
}

template <> struct Tr<TCUSCAN_F16_F32> {
    using acc = float; using acc4 = f32x4;
    static constexpr int kEsz = 2, kG = 8, kBlocks = 2;
    static constexpr bool kLinear = false;
    using Map = Map16;
    struct AConst { f16x8 a[kBlocks]; f16x8 ones; f16x8 tot; };
    using red = f32x4;
    static __device__ __forceinline__ red red_init() { return f32x4{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ red red_add(const AConst &A, red r, u32x4 b)
    {   // J * T: every row of the product is the row of column totals; accumulated over the tiles
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(A.ones, bits<f16x8>(b), r, 0, 0, 0);
    }
    static __device__ __forceinline__ acc red_lane(red r, int lane) { return lane < 16 ? r[0] : 0.f; }
    static __device__ __forceinline__ red totals(const AConst &A, u32x4 b)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(A.tot, bits<f16x8>(b), red_init(), 0, 0, 0);
    }
    static __device__ AConst make(int lane, bool excl, bool rev)
    {
        const AWords16 w = make16(lane, excl, rev, 0x3C003C003C003C00ull);       // 1.0h
        AConst A; A.a[0] = bits<f16x8>(w.a[0]); A.a[1] = bits<f16x8>(w.a[1]); A.ones = bits<f16x8>(w.ones); A.tot = bits<f16x8>(w.tot);
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int, bool, bool, acc4 (&d)[kBlocks])
    {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        f16x8 bv = bits<f16x8>(b);
        for (int p = 0; p < kBlocks; ++p) d[p] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A.a[p], bv, z, 0, 0, 0);
    }
};

template <> struct Tr<TCUSCAN_BF16_F32> {
    using acc = float; using acc4 = f32x4;
    static constexpr int kEsz = 2, kG = 8, kBlocks = 2;
    static constexpr bool kLinear = false;
    using Map = Map16;
    struct AConst { bf16x8 a[kBlocks]; bf16x8 ones; bf16x8 tot; };
    using red = f32x4;
    static __device__ __forceinline__ red red_init() { return f32x4{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ red red_add(const AConst &A, red r, u32x4 b)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(A.ones, bits<bf16x8>(b), r, 0, 0, 0);
    }
    static __device__ __forceinline__ acc red_lane(red r, int lane) { return lane < 16 ? r[0] : 0.f; }
    static __device__ __forceinline__ red totals(const AConst &A, u32x4 b)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(A.tot, bits<bf16x8>(b), red_init(), 0, 0, 0);
    }
    static __device__ AConst make(int lane, bool excl, bool rev)
    {
        const AWords16 w = make16(lane, excl, rev, 0x3F803F803F803F80ull);       // bf16 1.0
        AConst A; A.a[0] = bits<bf16x8>(w.a[0]); A.a[1] = bits<bf16x8>(w.a[1]); A.ones = bits<bf16x8>(w.ones); A.tot = bits<bf16x8>(w.tot);
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int, bool, bool, acc4 (&d)[kBlocks])
    {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        bf16x8 bv = bits<bf16x8>(b);
        for (int p = 0; p < kBlocks; ++p) d[p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A.a[p], bv, z, 0, 0, 0);
    }
};

template <> struct Tr<TCUSCAN_I8_I32> {
    using acc = uint32_t; using acc4 = i32x4;
    static constexpr int kEsz = 1, kG = 16, kBlocks = 4;
    static constexpr bool kLinear = false;
    struct Map {
        static __device__ __forceinline__ int jmap(int p, int) { return p; }
        static __device__ __forceinline__ int sub(int, int q) { return q; }
    };
    struct AConst { i32x4 a[kBlocks]; i32x4 ones; i32x4 tot; };
    using red = i32x4;
    static __device__ __forceinline__ red red_init() { return i32x4{0, 0, 0, 0}; }
    static __device__ __forceinline__ red red_add(const AConst &A, red r, u32x4 b)
    {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(A.ones, bits<i32x4>(b), r, 0, 0, 0);
    }
    static __device__ __forceinline__ acc red_lane(red r, int lane) { return lane < 16 ? (uint32_t)r[0] : 0u; }
    static __device__ __forceinline__ red totals(const AConst &A, u32x4 b)
    {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(A.tot, bits<i32x4>(b), red_init(), 0, 0, 0);
    }
    static __device__ AConst make(int lane, bool excl, bool rev)
    {
        AConst A; const int m = lane & 15, jj = lane >> 4;     // this lane supplies row m, K slots (jj, 0..15)
        A.ones = i32x4{0x01010101, 0x01010101, 0x01010101, 0x01010101};
        for (int p = 0; p < kBlocks; ++p) {
            uint64_t lo, hi;                                   // row m of block p is element m of granule row p
            tri_row(0x0101010101010101ull, m, 16, 8, excl, rev, jj == p, lo, hi);
            A.a[p] = i32x4{(int)(uint32_t)lo, (int)(uint32_t)(lo >> 32), (int)(uint32_t)hi, (int)(uint32_t)(hi >> 32)};
        }
        const int t = jj == (m & 3) ? 0x01010101 : 0;          // row 4q + r: total of granule row r
        A.tot = i32x4{t, t, t, t};
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int, bool, bool, acc4 (&d)[kBlocks])
    {
        const i32x4 z = {0, 0, 0, 0};
        i32x4 bv = bits<i32x4>(b);
        for (int p = 0; p < kBlocks; ++p) d[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A.a[p], bv, z, 0, 0, 0);
    }
    // Stream compaction of a 0/1 mask: the triangular blocks with 2 below the diagonal and 1 on it.  The product is
    // 2 * (ones before the element) + (the element itself): destination index and keep flag in one result, with no
    // second product and no exchange between the lanes that hold the mask and the lanes that hold the results.
    static __device__ AConst make_compact(int lane)
    {
        AConst A = make(lane, true, false);
        const AConst B = make(lane, false, false);
        for (int p = 0; p < kBlocks; ++p) A.a[p] = A.a[p] + B.a[p];      // bytes: 1 + 1 = 2 strictly below, 0 + 1 = 1 on the diagonal
        return A;
    }
};

template <> struct Tr<TCUSCAN_F32_F32> {
    using acc = float; using acc4 = f32x4;
    static constexpr int kEsz = 4, kG = 4, kBlocks = 1;
    // A granule is 4 elements: level 0 is s = 4, and lane (q, c) holds the four results of the granule it
    // loaded.  The K = 4 product p takes element p of every lane's granule: slot (j, p) <-> element p of
    // the granule of lane group j.
    static constexpr bool kLinear = true;     // lane l keeps granule l from load to store
    struct Map {
        static __device__ __forceinline__ int jmap(int, int q) { return q; }
        static __device__ __forceinline__ int sub(int, int) { return 0; }
    };
    struct AConst { float a[4]; };
    using red = float;      // 32-bit inputs: the tile total is four vector adds per granule
    static __device__ __forceinline__ red red_init() { return 0.f; }
    static __device__ __forceinline__ red red_add(const AConst &, red r, u32x4 b)
    {
        return r + ((bits<float>(b[0]) + bits<float>(b[1])) + (bits<float>(b[2]) + bits<float>(b[3])));
    }
    static __device__ __forceinline__ acc red_lane(red r, int) { return r; }
    static __device__ AConst make(int lane, bool excl, bool rev)
    {
        AConst A; int m = lane & 15, j = lane >> 4;
        for (int p = 0; p < 4; ++p) {
            const bool in = rev ? (excl ? p > (m & 3) : p >= (m & 3)) : (excl ? p < (m & 3) : p <= (m & 3));
            A.a[p] = (j == (m >> 2) && in) ? 1.0f : 0.0f;
        }
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int, bool, bool, acc4 (&d)[kBlocks])
    {
        f32x4 r = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < 4; ++p) r = __builtin_amdgcn_mfma_f32_16x16x4f32(A.a[p], bits<float>(b[p]), r, 0, 0, 0);
        d[0] = r;
    }
};

template <> struct Tr<TCUSCAN_I32_I32> {
    using acc = uint32_t; using acc4 = i32x4;
    static constexpr int kEsz = 4, kG = 4, kBlocks = 1;
    static constexpr bool kLinear = true;    // s = 4, as for fp32
    using Map = Tr<TCUSCAN_F32_F32>::Map;
    // int32 has no MFMA of its own: x = sum_p 2^(8p) * byte_p(x) (mod 2^32), every byte plane is
    // scanned by an i8 MFMA and the planes are recombined with shifts.  The i8 MFMA is signed, so
    // byte b enters as b - 128 (bit 7 flipped) and 128 * (number of summed elements) is added back.
    struct AConst { long a; };
    using red = uint32_t;
    static __device__ __forceinline__ red red_init() { return 0u; }
    static __device__ __forceinline__ red red_add(const AConst &, red r, u32x4 b) { return r + b[0] + b[1] + b[2] + b[3]; }
    static __device__ __forceinline__ acc red_lane(red r, int) { return r; }
    static __device__ AConst make(int lane, bool excl, bool rev)
    {
        int m = lane & 15, j = lane >> 4;
        uint64_t lo = 0;
        if (j == (m >> 2))
            lo = rev ? high_slots(0x01010101ull, 4 - (m & 3) - (excl ? 1 : 0), 4, 8) : low_slots(0x01010101ull, (m & 3) + (excl ? 0 : 1), 4, 8);
        AConst A; A.a = (long)lo;                 // K slots 4..7 of every lane are unused (zero on both sides)
        return A;
    }
    static __device__ __forceinline__ void mma(const AConst &A, u32x4 b, int lane, bool excl, bool rev, acc4 (&d)[kBlocks])
    {
        const i32x4 z = {0, 0, 0, 0};
        uint32_t x0 = b[0] ^ 0x80808080u, x1 = b[1] ^ 0x80808080u, x2 = b[2] ^ 0x80808080u, x3 = b[3] ^ 0x80808080u;
        i32x4 pl[4];
        for (int p = 0; p < 4; ++p) {
            uint32_t lo = __builtin_amdgcn_perm(x1, x0, 0x0c0c0000u | ((4u + p) << 8) | (uint32_t)p);
            uint32_t hi = __builtin_amdgcn_perm(x3, x2, 0x00000c0cu | ((4u + p) << 24) | ((uint32_t)p << 16));
            pl[p] = __builtin_amdgcn_mfma_i32_16x16x32_i8(A.a, (long)(uint64_t)(lo | hi), z, 0, 0, 0);
        }
        for (int r = 0; r < 4; ++r) {
            uint32_t cnt = (uint32_t)(rev ? 3 - r : r) + (excl ? 0u : 1u);    // elements summed into row 4q + r
            uint32_t v = (uint32_t)pl[0][r] + ((uint32_t)pl[1][r] << 8) + ((uint32_t)pl[2][r] << 16) + ((uint32_t)pl[3][r] << 24);
            d[0][r] = (int)(v + cnt * 0x80808080u);                           // 128 * cnt on every byte plane
        }
    }
};

// ------------------------------------------------------------------------ carry chain

__device__ __forceinline__ uint64_t status_word(uint32_t tag, uint32_t state, uint32_t value_bits)
{
    return ((uint64_t)((tag << 2) | state) << 32) | value_bits;
}

// Exclusive prefix of tile `tr` of its row: sum of the totals of tiles 0 .. tr-1, found by walking
// back over published status words, 64 * kDepth at a time.  Called by all 64 lanes of one
// wavefront.  All loads of a window are in flight together.  The window size is a measured compromise:
// a status round trip under full memory load costs microseconds, so a wider window saves round trips,
// but every extra word polled is uncached traffic that competes with the data (512 words per poll cost
// 5 % of the run time against 128, and 1024 and more cost 50 %).
constexpr int kDepth = 2;
template <class A>
__device__ A look_back(const uint64_t *row_status, int tr, uint32_t tag, WsHeader *ws, uint32_t spin_limit)
{
    const int lane = __lane_id();
    A sum = acc_from_bits<A>(0u);
    for (int base = tr - 1; base >= 0; base -= 64 * kDepth) {
        uint64_t w[kDepth];
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int idx = base - 64 * u - lane;
            if (idx >= 0) w[u] = __hip_atomic_load(row_status + (size_t)idx * kStatusStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // Take every total up to and including the nearest published prefix, skip everything behind it.
        bool done = false;
        A part = acc_from_bits<A>(0u);
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int idx = base - 64 * u - lane;
            uint32_t state = kStatePrefix, vbits = 0u;          // lanes before the row start count as "prefix 0"
            if (idx >= 0) {
                uint32_t spins = 0;
                for (;;) {
                    uint32_t f = (uint32_t)(w[u] >> 32);
                    if ((f >> 2) == tag) { state = f & 3u; vbits = (uint32_t)w[u]; break; }
                    if (++spins > spin_limit) {               // never in correct operation: give up instead of hanging
                        __hip_atomic_store(&ws->fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                    w[u] = __hip_atomic_load(row_status + (size_t)idx * kStatusStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            const uint64_t have_prefix = __ballot(state == kStatePrefix);
            const int first = have_prefix ? __builtin_ctzll(have_prefix) : 63;
            if (!done && lane <= first) part = acc_add(part, acc_from_bits<A>(vbits));
            done = done || have_prefix != 0;
        }
        sum = acc_add(sum, wave_sum(part));
        if (done) break;
    }
    return sum;
}

// The same walk in steps that never wait, for a wavefront that has other work to do while its predecessors' totals
// are still on their way: start() puts the loads of the first window in flight, every poll() looks at what has
// arrived -- a window whose words all carry the call's tag is consumed (and the next window requested), otherwise
// only the missing words are asked for again -- and finish() polls until the prefix is known.  All 64 lanes call.
template <class A> struct LookBackPoll {
    const uint64_t *row_status;
    uint32_t tag;
    int base;                    // the window covers tiles base, base - 1, ..., base - 64 * kDepth + 1
    A sum;
    uint64_t w[kDepth];
    bool done;

    __device__ __forceinline__ void request(bool all)
    {
        const int lane = __lane_id();
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int idx = base - 64 * u - lane;
            if (idx >= 0 && (all || (uint32_t)(w[u] >> 34) != tag))
                w[u] = __hip_atomic_load(row_status + (size_t)idx * kStatusStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __device__ __forceinline__ void start(const uint64_t *status, int tr, uint32_t call_tag)
    {
        row_status = status; tag = call_tag; base = tr - 1; sum = acc_from_bits<A>(0u); done = base < 0;
#pragma unroll
        for (int u = 0; u < kDepth; ++u) w[u] = 0u;
        if (!done) request(true);
    }
    __device__ __forceinline__ bool poll()
    {
        if (done) return true;
        const int lane = __lane_id();
        bool missing = false;
#pragma unroll
        for (int u = 0; u < kDepth; ++u) missing = missing || (base - 64 * u - lane >= 0 && (uint32_t)(w[u] >> 34) != tag);
        if (__ballot(missing) != 0) { request(false); return false; }
        bool found = false;
        A part = acc_from_bits<A>(0u);
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int idx = base - 64 * u - lane;
            const uint32_t state = idx >= 0 ? (uint32_t)(w[u] >> 32) & 3u : kStatePrefix;      // before the row start: "prefix 0"
            const uint32_t vbits = idx >= 0 ? (uint32_t)w[u] : 0u;
            const uint64_t have_prefix = __ballot(state == kStatePrefix);
            const int first = have_prefix ? __builtin_ctzll(have_prefix) : 63;
            if (!found && lane <= first) part = acc_add(part, acc_from_bits<A>(vbits));
            found = found || have_prefix != 0;
        }
        sum = acc_add(sum, wave_sum(part));
        base -= 64 * kDepth;
        done = found || base < 0;
        if (!done) request(true);
        return done;
    }
    __device__ __forceinline__ A finish(WsHeader *ws, uint32_t spin_limit)
    {
        uint32_t spins = 0;
        while (!poll()) {
            if (++spins > spin_limit) {                       // never in correct operation: give up instead of hanging
                __hip_atomic_store(&ws->fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        return sum;
    }
};

// Which tile this workgroup scans.  Default: its index in the grid -- a tile then waits only for tiles with a smaller
// workgroup index, and the chain makes progress as long as the hardware starts workgroups in index order (a workgroup
// is never started while one with a smaller index is still waiting for a place on the chip).  Ticket policy: the
// next number of a counter in the workspace header, drawn when the workgroup has started -- every smaller tile number
// was then drawn by a workgroup that is running or done, whatever the dispatch order; the price is one atomic on a
// single address per tile.  `s_slot`: an LDS word of the workgroup (free again when the call returns).
__device__ __forceinline__ uint32_t take_tile(const Params &P, uint32_t *s_slot)
{
    if (!P.ticket) return blockIdx.x;
    if (threadIdx.x == 0) *s_slot = __hip_atomic_fetch_add(&P.ws->ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t t = (uint32_t)__builtin_amdgcn_readfirstlane((int)*s_slot);
    __syncthreads();
    return t;
}

// ------------------------------------------------------------------- per-wavefront steps
//
// A wavefront owns a run of NT consecutive MFMA tiles (1 KiB of input each) of one row.  The three
// steps below are shared by the long-row kernel (workgroup tiles + carry chain) and the short-row
// kernel (one row per wavefront).

template <int DT> struct Geo {
    using T = Tr<DT>;
    static constexpr int kG = T::kG;                       // elements per input granule
    static constexpr int kS = 4 * kG;                      // column length
    static constexpr int kTileElems = 64 * kG;             // one MFMA tile = 1 KiB of input
};

struct Run {
    const char *in;          // first input byte of this wavefront's run
    char *out;               // first output byte of the run
    uint32_t rem;            // elements of the row from the start of the run on (saturated; 0 when the run starts past the end)
    uint32_t lead;           // segmented scans: elements at the start of the run that lie before the row (read as zero, not written)
    uint32_t cap;            // segmented scans: elements from the start of the run to the end of the caller's array (saturated)
    bool in_vec, out_vec;    // run starts are 16-byte aligned
};

// Element offset, inside the run, of granule slot `l` (0 .. 63) of MFMA tile `t` in processing order.  A reverse
// scan mirrors the granules -- tile 0, slot 0 is the last granule of the run -- and leaves the elements inside a
// granule where they are (the triangular blocks are upper triangular instead); a load or store instruction still
// covers 1 KiB of consecutive memory, and everything that scans "the slots before this one" then scans the
// elements after it.  (Written as tile part + lane part so that the tile part folds into the instruction's
// immediate offset.)
template <int DT, int NT, bool REV> __device__ __forceinline__ uint32_t slot_offset(int t, int l)
{
    constexpr int kG = Tr<DT>::kG;
    return REV ? (uint32_t)(NT - 1 - t) * (64 * kG) + (uint32_t)((63 - l) * kG) : (uint32_t)t * (64 * kG) + (uint32_t)(l * kG);
}

// a1: coalesced 128-bit loads, zero-filled past the end of the row (BatchMatMul's zero-pad)
// Keep bytes [lo, hi) of a granule, zero the rest.
__device__ __forceinline__ u32x4 keep_bytes(u32x4 v, int lo, int hi)
{
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        int a = lo - 4 * w, b = hi - 4 * w;
        a = a < 0 ? 0 : (a > 4 ? 4 : a);
        b = b < 0 ? 0 : (b > 4 ? 4 : b);
        const uint32_t m = b > a ? (uint32_t)((((1ull << (8 * b)) - 1) >> (8 * a)) << (8 * a)) : 0u;
        v[w] &= m;
    }
    return v;
}

template <int DT, int NT, bool REV, bool SEG = false>
__device__ __forceinline__ void load_run(const Run &R, int lane, u32x4 (&g)[NT])
{
    using T = Tr<DT>;
    constexpr int kG = Geo<DT>::kG;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const uint32_t e0 = slot_offset<DT, NT, REV>(t, lane);                            // element offset inside the run
        if (R.in_vec && e0 + kG <= R.rem && (!SEG || e0 >= R.lead)) {
            // (measured: non-temporal loads gain 3 % on the 32-bit chains and cost 10 % on the 8- and 16-bit ones)
            if constexpr (T::kEsz == 4) g[t] = __builtin_nontemporal_load((const u32x4 *)(R.in + e0 * T::kEsz));
            else g[t] = *(const u32x4 *)(R.in + e0 * T::kEsz);
        } else if (SEG && R.in_vec && e0 + kG <= R.cap) {
            // Segmented scans: a granule that straddles a row boundary still lies inside the caller's array; it is
            // loaded whole and the neighbouring row's elements are masked out (rows are short there, and an element-wise
            // load of every boundary granule costs more instructions than the rest of the tile).
            g[t] = u32x4{0u, 0u, 0u, 0u};
            if (e0 < R.rem && e0 + kG > R.lead) {
                const int lo = e0 >= R.lead ? 0 : (int)(R.lead - e0), hi = e0 + kG <= R.rem ? kG : (int)(R.rem - e0);
                g[t] = keep_bytes(*(const u32x4 *)(R.in + e0 * T::kEsz), lo * T::kEsz, hi * T::kEsz);
            }
        } else {
            uint32_t w[4] = {0u, 0u, 0u, 0u};
            for (int i = 0; i < kG; ++i) {
                if (e0 + i < R.rem && (!SEG || e0 + i >= R.lead)) {
                    uint32_t v;
                    if (T::kEsz == 4)      v = ((const uint32_t *)R.in)[e0 + i];
                    else if (T::kEsz == 2) v = ((const uint16_t *)R.in)[e0 + i];
                    else                   v = ((const uint8_t *)R.in)[e0 + i];
                    w[(i * T::kEsz) >> 2] |= v << (8 * ((i * T::kEsz) & 3));
                }
            }
            g[t] = u32x4{w[0], w[1], w[2], w[3]};
        }
    }
}

// Total of the run, taken from the granules as loaded: J * T accumulated over the tiles (every row of the
// product with the all-ones matrix is the row of column totals, and the grand total does not depend on
// which column a granule sits in), plain adds for 32-bit inputs.  No LDS traffic: the total is ready to be
// published as soon as the loads have landed.
template <int DT, int NT>
__device__ __forceinline__ typename Tr<DT>::acc reduce_run(int lane, const typename Tr<DT>::AConst &Aop, const u32x4 (&g)[NT])
{
    using T = Tr<DT>;
    typename T::red rsum = T::red_init();
#pragma unroll
    for (int t = 0; t < NT; ++t) rsum = T::red_add(Aop, rsum, g[t]);
    return wave_sum(T::red_lane(rsum, lane));
}

// Exclusive scan inside each 16-lane row (lane (q, c) receives v(q, 0) + ... + v(q, c-1)).
template <class A> __device__ __forceinline__ A row_exclusive_scan(A v)
{
    A e = dpp_shr<A, kRowShr + 1>(v);
    e = acc_add(e, dpp_shr<A, kRowShr + 1>(e));
    e = acc_add(e, dpp_shr<A, kRowShr + 2>(e));
    e = acc_add(e, dpp_shr<A, kRowShr + 4>(e));
    e = acc_add(e, dpp_shr<A, kRowShr + 8>(e));
    return e;
}

// a2 + a3 + a5 + a6 for the run, tile by tile with a running carry (`carry` = everything before the run).
// Nothing passes through LDS: lane l feeds the MFMA with the granule it loaded, and results are stored
// straight from the MFMA's result registers, 1 KiB of consecutive outputs per store instruction.
template <int DT, int NT, bool EXCL, bool REV, bool SEG = false>
__device__ __forceinline__ void scan_and_store(int lane, const typename Tr<DT>::AConst &Aop, const Run &R,
                                               const u32x4 (&g)[NT], typename Tr<DT>::acc carry)
{
    using T = Tr<DT>;
    using A = typename T::acc;
    using A4 = typename T::acc4;
    constexpr int kBlocks = T::kBlocks;
    const int c = lane & 15, q = lane >> 4;         // result layout: column, row group
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        // a2: level 0, the local scans of the 64 granules on the MFMA unit
        A4 d[kBlocks];
        T::mma(Aop, g[t], lane, EXCL, REV, d);
        // a3 (up-sweep rounds t = 1, 2 and their down-sweep, on the vector unit): e[p] = everything in the run
        // before the granule whose results this lane holds in block p
        A e[kBlocks];
        if constexpr (T::kLinear) {
            // the lane's own granule: its total is the last row of its block; scan the 64 totals in lane order
            constexpr int edge = REV ? 0 : 3;                           // the row of the block that sums the whole granule
            A tot = acc_from_bits<A>((uint32_t)bits<u32x4>(d[0])[edge]);
            if (EXCL) tot = acc_add(tot, acc_from_bits<A>(g[t][edge]));  // the strict product leaves that row's own element out
            const A inc = wave_inclusive_scan(tot);
            e[0] = acc_add(carry, wave_shift_up(inc));
            carry = acc_add(carry, uniform_from_lane(inc, 63));
        } else {
            // granule totals from the matrix unit (register p: granule (jmap(p, q), c)), scanned over c inside
            // each 16-lane row; the totals of the four granule rows j are wave-uniform and are added in order
            const u32x4 tt = bits<u32x4>(T::totals(Aop, g[t]));
#pragma unroll
            for (int p = 0; p < kBlocks; ++p) {
                const A tot = acc_from_bits<A>(tt[p]);
                const A ex = row_exclusive_scan(tot);
                const A inc = acc_add(ex, tot);
                if constexpr (T::kG == 16) {                 // block p <-> granule row p, the same in every lane row
                    e[p] = acc_add(carry, ex);
                    carry = acc_add(carry, uniform_from_lane(inc, 15));
                } else {                                     // block p <-> granule rows 2p (lane rows 0, 1) and 2p + 1 (lane rows 2, 3)
                    const A lo = uniform_from_lane(inc, 15), hi = uniform_from_lane(inc, 47);
                    const A mid = acc_add(carry, lo);
                    e[p] = acc_add(q >= 2 ? mid : carry, ex);
                    carry = acc_add(mid, hi);
                }
            }
        }
        // a5: down-sweep = one add per output;  a6: store
#pragma unroll
        for (int p = 0; p < kBlocks; ++p) {
            u32x4 v = bits<u32x4>(d[p]);
            for (int r = 0; r < 4; ++r) v[r] = acc_bits(acc_add(e[p], acc_from_bits<A>(v[r])));
            const uint32_t e0 = slot_offset<DT, NT, REV>(t, 16 * T::Map::jmap(p, q) + c) + 4u * T::Map::sub(p, q);
            if (R.out_vec && e0 + 4 <= R.rem && (!SEG || e0 >= R.lead)) {
                __builtin_nontemporal_store(v, (u32x4 *)(R.out + e0 * 4));   // written once, never read back here
            } else {
                for (int r = 0; r < 4; ++r)
                    if (e0 + r < R.rem && (!SEG || e0 + r >= R.lead)) ((uint32_t *)R.out)[e0 + r] = v[r];
            }
        }
    }
}

template <int DT>
__device__ __forceinline__ Run make_run(const Params &P, uint64_t row, uint64_t base)
{
    // `base` (first element of the run inside the row) is a multiple of an MFMA tile, so run starts are
    // 16-byte aligned exactly when the row start is.  Offsets inside a run fit 32 bits.
    Run R;
    const uint64_t first = row * P.cols + base;
    R.in = (const char *)P.in + first * Tr<DT>::kEsz;
    R.out = (char *)P.out + first * 4;
    const uint64_t left = base < P.cols ? P.cols - base : 0;
    R.rem = left < 0x40000000ull ? (uint32_t)left : 0x40000000u;
    R.lead = 0;
    R.cap = R.rem;
    R.in_vec = (((uintptr_t)R.in) & 15) == 0;
    R.out_vec = (((uintptr_t)R.out) & 15) == 0;
    return R;
}

// Segmented scans: a row starts wherever the previous one ended, so its first byte is usually not 16-byte aligned.
// The row is therefore tiled from the aligned address just below its start: the `lead` elements in front of it
// (fewer than one granule) are read as zero and never written -- BatchMatMul's zero-pad, at the front -- and every
// full granule behind them takes the 128-bit path.  With both base pointers 16-byte aligned the outputs line up too:
// lead = off mod (elements per granule), and (off - lead) outputs are a whole number of 16-byte groups.
template <int DT>
__device__ __forceinline__ uint32_t seg_lead(const Params &P, long long off)
{
    return (uint32_t)((((uintptr_t)P.in + (uint64_t)off * Tr<DT>::kEsz) & 15) / Tr<DT>::kEsz);
}
template <int DT>
__device__ __forceinline__ Run make_seg_run(const Params &P, long long off, uint64_t len, uint32_t lead, uint64_t base)
{
    Run R;
    const long long first = off - (long long)lead + (long long)base;      // element index of the run's first slot
    R.in = (const char *)P.in + first * Tr<DT>::kEsz;
    R.out = (char *)P.out + first * 4;
    const uint64_t vlen = len + lead;
    const uint64_t left = base < vlen ? vlen - base : 0;
    R.rem = left < 0x40000000ull ? (uint32_t)left : 0x40000000u;
    R.lead = base < lead ? lead - (uint32_t)base : 0;
    const long long to_end = (long long)P.cols - first;                   // P.cols holds the number of elements of the arrays
    R.cap = to_end <= 0 ? 0u : to_end < 0x40000000ll ? (uint32_t)to_end : 0x40000000u;
    // (first < 0: a row that starts within the first granule of an array that is itself not 16-byte aligned; the
    // aligned address below it lies before the array, so that run goes element by element)
    R.in_vec = first >= 0 && (((uintptr_t)R.in) & 15) == 0;
    R.out_vec = first >= 0 && (((uintptr_t)R.out) & 15) == 0;
    return R;
}

// ----------------------------------------------------------------------- long-row kernel

// Waves per SIMD the register allocator is asked to make room for (more resident tiles hide more of the
// carry chain's latency); values found by measurement, none of them makes the allocator spill.
template <int DT, int NT> struct MinWaves { static constexpr int value = 1; };
template <> struct MinWaves<TCUSCAN_I8_I32, 8>    { static constexpr int value = 5; };
template <> struct MinWaves<TCUSCAN_F16_F32, 16>  { static constexpr int value = 4; };
template <> struct MinWaves<TCUSCAN_BF16_F32, 16> { static constexpr int value = 4; };

template <int DT, int NT, bool EXCL, bool REV, int W, bool SEG = false>
__global__ __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(MinWaves<DT, NT>::value)))
void scan_kernel(Params P)
{
    using T = Tr<DT>;
    using A = typename T::acc;
    constexpr uint32_t kEPW = NT * Geo<DT>::kTileElems;   // elements per wavefront
    constexpr uint32_t kWgElems = kEPW * W;               // elements per workgroup tile (W wavefronts)

    __shared__ uint32_t s_wave_total[W];
    __shared__ uint32_t s_bcast;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform: keeps tile bookkeeping in SGPRs

    // ---- which tile.  Tiles are taken in workgroup-index order by default: a tile only ever waits for
    // tiles with a smaller index, which the hardware dispatched earlier (or at the same time), so the
    // lowest unfinished tile is always running and the chain cannot stall.  (The ticket policy
    // guarantees the same without that assumption, but one contended atomic per tile caps the whole
    // kernel at the device's single-address atomic rate.)  Status words carry the call's tag, so
    // words left over from earlier calls read as "not published yet" and need no clearing.
    const uint32_t tile = take_tile(P, &s_bcast);
    const uint32_t tag = P.tag;
    uint64_t row;
    uint32_t tr, tiles_in_row, first_tile;        // position in the carry chain of the row, its length, the row's first tile
    Run R;
    if constexpr (SEG) {
        // Rows have their own numbers of tiles; the grid is an upper bound on their sum.  Everything a tile needs to
        // know about its row was put into one descriptor per tile beforehand: looked up here, it would be a chain of
        // four dependent loads at the head of every workgroup.
        if (tile >= P.num_tiles) return;
        long long off;
        uint64_t len;
        row = 0;
        if (P.tile_desc) {
            const TileDesc d = P.tile_desc[tile];
            if (d.tiles_in_row == 0) return;
            first_tile = d.first_tile;
            tiles_in_row = d.tiles_in_row;
            off = d.off;
            len = d.len;
        } else {
            // Equal rows that do not start at 16-byte boundaries (a batched call with an odd row length or an unaligned
            // array): no descriptors, the row follows from the tile index.  P.cols is the length of the arrays here, as
            // for every segmented call; P.tiles_per_row tiles hold a row and the elements in front of it.
            const uint32_t r = tile / P.tiles_per_row;
            first_tile = r * P.tiles_per_row;
            tiles_in_row = P.tiles_per_row;
            len = P.cols / P.rows;
            off = (long long)(r * len);
        }
        tr = tile - first_tile;
        const uint32_t pos = REV ? tiles_in_row - 1 - tr : tr;
        R = make_seg_run<DT>(P, off, len, seg_lead<DT>(P, off), (uint64_t)pos * kWgElems + (uint64_t)wave * kEPW);
    } else {
        row = tile / P.tiles_per_row;
        tiles_in_row = P.tiles_per_row;
        first_tile = (uint32_t)row * P.tiles_per_row;
        tr = tile - first_tile;
        const uint32_t pos = REV ? tiles_in_row - 1 - tr : tr;            // position in the row: a reverse scan starts at the end
        R = make_run<DT>(P, row, (uint64_t)pos * kWgElems + (uint64_t)wave * kEPW);
    }
    const bool chained = tiles_in_row > 1;

    // A workgroup of the big tiles issues its loads at raised wave priority.  It has just taken the place of a
    // workgroup that finished, and the compute unit's other wavefronts are in the middle of their stores: at equal
    // priority the newcomer's load instructions queue up behind theirs, its tile total -- which every later tile of
    // the row is waiting for -- comes late, and the memory system has nothing to read while it drains the stores.
    // Measured (us, 2^28 elements in one row unless noted): f32 358 -> 340, n = 100,000,007 f32 143 -> 136, bf16 on the
    // 32768-element tile 287 -> 264.  The small 16- and 32-bit tiles lose with it (4096 x 65536 bf16 259 -> 273, 16384 x
    // 8192 f32 172 -> 193: with many short-lived workgroups the stores are what must not wait) and keep the default;
    // the small 8-bit tile, which stores four bytes for every byte it loads, gains (32768 x 8192 i8 258 -> 217).
    constexpr bool kLoadsFirst = kWgElems > 8192 || DT == TCUSCAN_I8_I32;
    // The first generation of the huge 32-bit tiles (two workgroups of 8 wavefronts per compute unit: 512 tiles) starts
    // 20 ns apart instead of all at once -- half the interval at which the memory system finishes such tiles (256 KiB
    // at 6.4 TB/s: 41 ns).  Started together, the whole generation only loads for 10 us and the first stores leave
    // when the last loads have landed; spread out, the early tiles store while the late ones load.  Measured (us):
    // n = 100,000,007 f32 136 -> 132, one i32 row of 2^28 359 -> 345; 10 or 30 ns, or half as many tiles, lose the gain,
    // and the 8- and 16-bit tiles (more workgroups per compute unit, less data each) do not gain at any interval.
    // The wait reads the constant-rate wall clock (10 ns per tick) and is bounded.
    if constexpr (T::kEsz == 4 && W == 8 && NT == 16) {
        if (tile < 512u && P.num_tiles >= 1024u) {
            const uint64_t t0 = wall_clock64(), ticks = 2u * tile;
            for (int i = 0; i < 4096 && wall_clock64() - t0 < ticks; ++i) __builtin_amdgcn_s_sleep(2);
        }
    }
    if constexpr (kLoadsFirst) __builtin_amdgcn_s_setprio(3);
    u32x4 g[NT];
    load_run<DT, NT, REV, SEG>(R, lane, g);
    if constexpr (kLoadsFirst) __builtin_amdgcn_s_setprio(0);
    const typename T::AConst Aop = T::make(lane, EXCL, REV);

    // ---- the total of the run (the up-sweep of this tile in one step)
    const A wave_total = reduce_run<DT, NT>(lane, Aop, g);

    // ---- level 2: wavefront totals through LDS
    A wave_off = acc_from_bits<A>(0u), wg_total = wave_total;
    if constexpr (W > 1) {
        if (lane == 0) s_wave_total[wave] = acc_bits(wave_total);
        __syncthreads();
        wg_total = acc_from_bits<A>(0u);
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const A v = acc_from_bits<A>(s_wave_total[w]);
            if (REV ? w > wave : w < wave) wave_off = acc_add(wave_off, v);    // the wavefronts scanned before this one
            wg_total = acc_add(wg_total, v);
        }
    }

    // ---- a4: carry chain between workgroup tiles of the same row
    A prefix = acc_from_bits<A>(0u);
    if (chained) {
        uint64_t *row_status = (uint64_t *)(P.ws + 1) + (uint64_t)first_tile * kStatusStride;
        if (wave == 0) {
            const bool speaks = lane == 0 && tile != P.mute_tile;      // (the test hook silences one tile)
            if (tr == 0) {
                if (speaks)
                    __hip_atomic_store(row_status, status_word(tag, kStatePrefix, acc_bits(wg_total)),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                if (speaks)
                    __hip_atomic_store(row_status + (size_t)tr * kStatusStride, status_word(tag, kStateAggregate, acc_bits(wg_total)),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                prefix = look_back<A>(row_status, (int)tr, tag, P.ws, P.spin_limit);
                if (speaks)
                    __hip_atomic_store(row_status + (size_t)tr * kStatusStride, status_word(tag, kStatePrefix, acc_bits(acc_add(prefix, wg_total))),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (W > 1 && lane == 0) s_bcast = acc_bits(prefix);
        }
        if constexpr (W > 1) {                    // (a one-wavefront tile has the prefix in every lane already)
            __syncthreads();
            prefix = acc_from_bits<A>(s_bcast);
        }
    }

    // ---- local scans, down-sweep add and store, with everything before this wavefront's run as carry
    scan_and_store<DT, NT, EXCL, REV, SEG>(lane, Aop, R, g, acc_add(prefix, wave_off));
}

// ------------------------------------------------------------- fused split and fused stream compaction
//
// Blelloch's split on bit b (one pass of the radix sort): keys whose bit is 0 go to the front, the others behind them,
// both in their old order.  The mask "bit b is 0" is never written and the keys are read once: a lane loads its keys
// where its results will be (16 bytes per result block, every load instruction 1 KiB contiguous), takes the mask bytes
// from them and passes them to the lanes that feed the product (a 4 x 4 transpose between registers and 16-lane rows:
// four lane swaps per MFMA tile).  The scan is the usual one (run totals first, carry chain between workgroups) with
// an operand that returns 2 * (flagged before) + own flag: destination and flag in one product.  The words of a
// wavefront's run, still in registers, are put in order in an LDS slot (zeros, then ones) and leave it as two
// consecutive ranges, 16 bytes per lane.  The number of zeros of the whole array, which the ones' destinations need,
// does not depend on the order of the keys: all 32 counts are taken once, before the first pass.
//
// Stream compaction is the same kernel body with the flags read from the mask array and only the first range stored.

__global__ __launch_bounds__(256) void bit_zero_counts_kernel(const uint32_t *__restrict__ keys, size_t n, uint32_t *counts)
{
    __shared__ uint32_t s_cnt[32];
    if (threadIdx.x < 32) s_cnt[threadIdx.x] = 0u;
    __syncthreads();
    uint32_t cnt[32];
#pragma unroll
    for (int b = 0; b < 32; ++b) cnt[b] = 0u;
    // bits b, b + 8, b + 16, b + 24 are counted together in the four bytes of one word, which is emptied into the
    // 32-bit counters before a byte can overflow (255 keys)
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i0 < n; i0 += 255u * stride) {
        uint32_t packed[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) packed[b] = 0u;
        size_t i = i0;
#pragma unroll 4
        for (int k = 0; k < 255 && i < n; ++k, i += stride) {
            const uint32_t z = ~keys[i];
#pragma unroll
            for (int b = 0; b < 8; ++b) packed[b] += (z >> b) & 0x01010101u;
        }
#pragma unroll
        for (int b = 0; b < 8; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j) cnt[b + 8 * j] += (packed[b] >> (8 * j)) & 0xFFu;
    }
#pragma unroll
    for (int b = 0; b < 32; ++b) {
        const uint32_t w = wave_sum(cnt[b]);
        if ((threadIdx.x & 63) == 0 && w) atomicAdd(&s_cnt[b], w);
    }
    __syncthreads();
    if (threadIdx.x < 32 && s_cnt[threadIdx.x]) atomicAdd(&counts[threadIdx.x], s_cnt[threadIdx.x]);
}

struct SplitArgs {
    const uint32_t *keys, *vals;       // vals may be null
    uint32_t *keys_out, *vals_out;
    const uint32_t *zeros_total;       // number of keys whose bit is 0
    int bit;
};

// g[k] of the lane in row P (row = 16 lanes) becomes w[P] of the lane in row k, same column: the mask words move
// from the lanes that hold the keys (result layout) to the lanes that feed the product (one granule of 16 bytes each).
__device__ __forceinline__ u32x4 rows_transpose(const uint32_t (&w)[4])
{
    const auto x = __builtin_amdgcn_permlane32_swap(w[0], w[2], false, false);    // {rows 0,1 of both, rows 2,3 of both}
    const auto y = __builtin_amdgcn_permlane32_swap(w[1], w[3], false, false);
    const auto lo = __builtin_amdgcn_permlane16_swap(x[0], y[0], false, false);   // {even rows of both, odd rows of both}
    const auto hi = __builtin_amdgcn_permlane16_swap(x[1], y[1], false, false);
    return u32x4{lo[0], lo[1], hi[0], hi[1]};
}

// 16 bytes of a result block for this lane: words e0 .. e0 + 3 of a run of rem words (fill beyond the end).
__device__ __forceinline__ u32x4 load_block_words(const uint32_t *run, bool vec, uint32_t e0, uint32_t rem, uint32_t fill)
{
    u32x4 x = {fill, fill, fill, fill};
    if (vec && e0 + 4 <= rem) {
        x = *(const u32x4 *)(run + e0);
    } else {
        for (int i = 0; i < 4; ++i)
            if (e0 + i < rem) x[i] = run[e0 + i];
    }
    return x;
}

// One ordered range of the slot (cnt words from word q on) to global memory, cnt words from dst on.  The slot was
// filled before the destination was known, so the range lies in it at whatever offset; a lane still moves whole
// aligned 16-byte groups of the destination (four words of the slot at any word offset, one 16-byte store that is
// 1 KiB contiguous over the wavefront), and the two ragged groups at the ends go word by word.
// lim: words from dst on that exist in the destination.
__device__ __forceinline__ void split_store_range(int lane, const uint32_t *slot, uint32_t q, uint32_t cnt, uint32_t *dst, uint32_t lim)
{
    const uint32_t a = (uint32_t)((uintptr_t)dst >> 2) & 3u;             // offset of the range inside a 16-byte group
    const uint32_t end = a + (cnt < lim ? cnt : lim);
    const uint32_t first = (a + 3u) >> 2, past = end >> 2;               // whole groups: first .. past - 1 (group 0 starts at dst - a)
    const uint32_t *sl = slot + q - a;                                   // only words a .. end - 1 of it are touched
    uint32_t *gq = dst - a;
    for (uint32_t j = first + (uint32_t)lane; j < past; j += 64u) {
        const uint32_t *src = sl + 4u * j;
        __builtin_nontemporal_store(u32x4{src[0], src[1], src[2], src[3]}, (u32x4 *)(gq + 4u * j));
    }
    // the ragged group in front (words a .. 3) and the one behind (words 4 past ..): lanes 0 .. 3 and 4 .. 7, a word each
    if (lane < 8) {
        const uint32_t i = lane < 4 ? (uint32_t)lane : 4u * past + (uint32_t)(lane - 4);
        const bool mine = lane < 4 ? (i >= a && i < end && first == 1u) : (i < end && past >= first);
        if (mine) gq[i] = sl[i];
    }
}

// The words x (keys, payloads or values, in result layout) of one wavefront's run put in order in the wavefront's
// LDS slot: those with the flag ("zeros": the split flags a key whose bit is 0) first and, if ONES, the others behind
// them, both in their old order (positions from the product 2 * zeros before + own flag).  Nothing here depends on
// where the ranges go in the destination, so this runs while the tile's predecessors are still publishing: if
// `polling`, the chain is polled once per result block.
template <int NT, uint32_t SLOT, bool ONES, class Chain>
__device__ __forceinline__ void split_order(int lane, const typename Tr<TCUSCAN_I8_I32>::AConst &Aop, const u32x4 (&g)[NT],
                                            const u32x4 (&x)[NT][4], uint32_t zeros_run, uint32_t rem, uint32_t *slot, Chain &chain,
                                            bool polling)
{
    using T = Tr<TCUSCAN_I8_I32>;
    const bool ragged = rem < NT * 1024u;
    const int c = lane & 15, q = lane >> 4;
    const uint32_t in_blk = 16u * c + 4u * q;
    uint32_t before = 0u;                                                    // zeros in the earlier blocks of the run
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        i32x4 d[T::kBlocks];
        T::mma(Aop, g[t], lane, true, false, d);                            // 2 * zeros before + own flag
        const u32x4 tt = bits<u32x4>(T::totals(Aop, g[t]));
#pragma unroll
        for (int p = 0; p < T::kBlocks; ++p) {
            const uint32_t ex = row_exclusive_scan(tt[p]);
            const uint32_t zeros = uniform_from_lane(ex + tt[p], 15);       // zeros in this block
            const uint32_t idx0 = (uint32_t)t * 1024u + 256u * p + in_blk;
            for (int r = 0; r < 4; ++r) {
                const uint32_t w = (uint32_t)d[p][r], zb = before + ex + (w >> 1), idx = idx0 + r;
                uint32_t at = (w & 1u) ? zb : zeros_run + (idx - zb);
                if constexpr (ONES) {                          // every key has a place: no branch around the write;
                    if (ragged && idx >= rem) at = SLOT - 1u;  // keys past the end go to the slot's spare last word,
                    at = at < SLOT - 1u ? at : SLOT - 1u;      // and so would a position beyond the ranges (never)
                    slot[at] = x[t][p][r];
                } else {
                    if (idx < rem && at < SLOT && (w & 1u)) slot[at] = x[t][p][r];
                }
            }
            before += zeros;
            if (polling) chain.poll();
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The ordered run from the slot to the destination: the zeros from dst[zero_at] on and, if ONES, the others (up to
// `valid` words in all) from dst[one_at] on.
template <bool ONES>
__device__ __forceinline__ void split_store(int lane, const uint32_t *slot, uint32_t *dst, uint64_t zero_at, uint64_t one_at, uint32_t zeros_run,
                                            uint32_t valid, uint64_t n)
{
    const uint64_t room0 = zero_at < n ? n - zero_at : 0u, room1 = one_at < n ? n - one_at : 0u;
    split_store_range(lane, slot, 0u, zeros_run, dst + zero_at, (uint32_t)(room0 < 0x40000000ull ? room0 : 0x40000000ull));
    if constexpr (ONES)
        split_store_range(lane, slot, zeros_run, valid - zeros_run, dst + one_at, (uint32_t)(room1 < 0x40000000ull ? room1 : 0x40000000ull));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// From a wavefront's flag count to what lies before its run in the whole array, in two steps with the ordering of the
// run between them.  Setting out: totals of the workgroup's wavefronts through LDS; wavefront 0 publishes the
// workgroup's total and asks for the status words of the tiles before (the carry chain of scan_kernel; one row, tiles
// in workgroup-index order).
template <int W>
__device__ __forceinline__ void flags_set_out(const Params &P, uint32_t tile, int lane, int wave, uint32_t wave_total, uint32_t *s_wave_total,
                                              LookBackPoll<uint32_t> &lb, uint32_t &wave_off, uint32_t &run_total, uint32_t &wg_total)
{
    if (lane == 0) s_wave_total[wave] = wave_total;
    __syncthreads();
    wave_off = 0u; wg_total = 0u;
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const uint32_t v = s_wave_total[w];
        if (w < wave) wave_off += v;
        wg_total += v;
    }
    run_total = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_wave_total[wave]);
    lb.done = true;
    if (P.num_tiles > 1 && wave == 0) {
        uint64_t *row_status = (uint64_t *)(P.ws + 1);
        if (lane == 0)
            __hip_atomic_store(row_status + (size_t)tile * kStatusStride, status_word(P.tag, tile == 0 ? kStatePrefix : kStateAggregate, wg_total),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lb.start(row_status, (int)tile, P.tag);
    }
}

// Arriving: the flags in all tiles before this one, known to every wavefront of the workgroup.
__device__ __forceinline__ uint32_t flags_arrive(const Params &P, uint32_t tile, int lane, int wave, uint32_t wg_total, LookBackPoll<uint32_t> &lb,
                                                 uint32_t *s_bcast)
{
    uint32_t prefix = 0u;
    if (P.num_tiles > 1) {
        if (wave == 0) {
            prefix = lb.finish(P.ws, P.spin_limit);
            if (lane == 0) {
                if (tile != 0)
                    __hip_atomic_store((uint64_t *)(P.ws + 1) + (size_t)tile * kStatusStride, status_word(P.tag, kStatePrefix, prefix + wg_total),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                *s_bcast = prefix;
            }
        }
        __syncthreads();
        prefix = *s_bcast;
    }
    return prefix;
}

// The 16-byte words of a wavefront's run in result layout: block p of MFMA tile t, words 16 c + 4 q .. + 3 of it.
template <int NT>
__device__ __forceinline__ void load_run_words(int lane, const uint32_t *run, uint32_t rem, uint32_t fill, u32x4 (&x)[NT][4])
{
    const uint32_t in_blk = 16u * (lane & 15) + 4u * (lane >> 4);
    const bool vec = (((uintptr_t)run) & 15) == 0;
    if (vec && rem >= NT * 1024u) {                             // a whole run: straight-line loads
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int p = 0; p < 4; ++p) x[t][p] = __builtin_nontemporal_load((const u32x4 *)(run + (uint32_t)t * 1024u + 256u * p + in_blk));
    } else {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int p = 0; p < 4; ++p) x[t][p] = load_block_words(run, vec, (uint32_t)t * 1024u + 256u * p + in_blk, rem, fill);
    }
}

template <int NT, int W, bool VALS>
__global__ __launch_bounds__(64 * W) void split_kernel(Params P, SplitArgs S)
{
    constexpr int DT = TCUSCAN_I8_I32;
    using T = Tr<DT>;
    static_assert(T::kBlocks == 4, "four result blocks of 256 per MFMA tile");
    constexpr uint32_t kEPW = NT * Geo<DT>::kTileElems;
    constexpr uint32_t kSlot = kEPW + 16u;                      // the run in order, and a spare last word
    __shared__ uint32_t s_wave_total[W];
    __shared__ uint32_t s_bcast;
    __shared__ __attribute__((aligned(16))) uint32_t s_pack[W][kSlot];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint64_t n = P.cols;
    const uint32_t tile = take_tile(P, &s_bcast);
    const uint64_t base = ((uint64_t)tile * W + wave) * kEPW;                       // first key of this wavefront's run
    const uint32_t rem = base < n ? (n - base < 0x40000000ull ? (uint32_t)(n - base) : 0x40000000u) : 0u;
    const int bit = S.bit;

    // ---- the keys, and from them the mask granules (keys past the end read as all ones: flag 0)
    u32x4 key[NT][4], g[NT];
    __builtin_amdgcn_s_setprio(3);                  // loads first, as in scan_kernel
    load_run_words<NT>(lane, S.keys + base, rem, ~0u, key);
    __builtin_amdgcn_s_setprio(0);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        uint32_t w[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            w[p] = 0u;
            for (int i = 0; i < 4; ++i) w[p] |= ((~key[t][p][i] >> bit) & 1u) << (8 * i);
        }
        g[t] = rows_transpose(w);
    }
    const typename T::AConst Aop = T::make_compact(lane);
    LookBackPoll<uint32_t> lb;
    uint32_t wave_off, zeros_run, wg_total;
    flags_set_out<W>(P, tile, lane, wave, reduce_run<DT, NT>(lane, Aop, g), s_wave_total, lb, wave_off, zeros_run, wg_total);

    // ---- the run in order in the slot while the chain is on its way, then to its two places
    const uint32_t valid = rem < kEPW ? rem : kEPW;
    split_order<NT, kSlot, true>(lane, Aop, g, key, zeros_run, rem, s_pack[wave], lb, P.num_tiles > 1 && wave == 0);
    const uint32_t zero_at = flags_arrive(P, tile, lane, wave, wg_total, lb, &s_bcast) + wave_off;
    const uint64_t one_at = (uint64_t)*S.zeros_total + (base - zero_at);     // behind all zeros, after the ones before this run
    split_store<true>(lane, s_pack[wave], S.keys_out, zero_at, one_at, zeros_run, valid, n);
    if constexpr (VALS) {
        u32x4 val[NT][4];
        load_run_words<NT>(lane, S.vals + base, rem, 0u, val);
        split_order<NT, kSlot, true>(lane, Aop, g, val, zeros_run, rem, s_pack[wave], lb, false);
        split_store<true>(lane, s_pack[wave], S.vals_out, zero_at, one_at, zeros_run, valid, n);
    }
}

// ---- the split on two bits at once: four buckets per pass, half the passes
//
// The same reduction with a digit of two bits: keys go to four consecutive ranges by digit, old order kept inside
// each.  Four flag vectors ("digit is d") would be four scans; they are one-hot, so two of them share a byte -- flag
// of digit 0 (2) as 1, of digit 1 (3) as 64 -- and one product with the strict triangular blocks returns both counts
// of earlier keys inside the granule (each below 16) in separate bit fields.  Granule totals come from the totals
// operand the same way; from there on (16-lane scans, blocks, runs, workgroup) two counts travel in the halves of one
// 32-bit word.  The carry chain has four values per tile: the four words share the tile's status slot, and the first
// four wavefronts of a workgroup publish and look back for one digit each, at the same time.

struct Split4Args {
    const uint32_t *keys, *vals;       // vals may be null
    uint32_t *keys_out, *vals_out;
    const uint32_t *hist;              // number of keys with digit 0, 1, 2, 3 at this position (whole array)
    int bit;                           // position of the digit's low bit
};

// 16 digit positions x 4 digits: counts[4 j + d] = keys whose bits 2j+1, 2j are d.  Digits 1, 2 and 3 are counted
// (digit 0 is the rest): a key becomes three words with one bit per digit position ("the digit here is d", at the even
// bits), and the bits of such words are added up in fields that widen as they fill: two keys' words in the 2-bit
// fields they come in, the four keys of a load and up to three loads in 4-bit fields (even and odd positions in a
// word each), 63 loads in byte-wide counters -- bits s, s + 8, s + 16, s + 24 in the four bytes of one word, for s = 0,
// 2, 4, 6 -- which are emptied into 32-bit counters before a byte can overflow.  (With every key's words going
// straight into the byte counters the kernel was bound by the vector unit: 46 instructions per key, 99 us for 2^26
// keys.)
__global__ __launch_bounds__(256) void digit_counts_kernel(const uint32_t *__restrict__ keys, size_t n, uint32_t *counts)
{
    __shared__ uint32_t s_cnt[64];
    if (threadIdx.x < 64) s_cnt[threadIdx.x] = 0u;
    __syncthreads();
    uint32_t cnt[3][16];                                      // [digit - 1][position]
#pragma unroll
    for (int d = 0; d < 3; ++d)
#pragma unroll
        for (int j = 0; j < 16; ++j) cnt[d][j] = 0u;
    // four keys per step (one 16-byte load per lane; the array is 16-byte aligned), the last n mod 4 keys by one thread
    const size_t stride = (size_t)gridDim.x * blockDim.x, quads = n / 4;
    const u32x4 *keys4 = (const u32x4 *)keys;
    for (size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i0 < quads + 1; i0 += 63u * stride) {
        uint32_t packed[3][4];                                // [digit - 1][s / 2]: byte b counts position s / 2 + 4 b
#pragma unroll
        for (int d = 0; d < 3; ++d)
#pragma unroll
            for (int k = 0; k < 4; ++k) packed[d][k] = 0u;
        size_t i = i0;
        for (int grp = 0; grp < 21 && i < quads + 1; ++grp) {                 // 21 x 3 loads of 4 keys: a byte counter stays below 256
            uint32_t even[3] = {0u, 0u, 0u}, odd[3] = {0u, 0u, 0u};           // 4-bit fields: positions 0, 2, .. 14 / 1, 3, .. 15
            u32x4 kqs[3];                                                     // 3 x 4 keys: a 4-bit field stays below 16; the loads side by side
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const size_t ik = i + (size_t)k * stride;
                kqs[k] = u32x4{0u, 0u, 0u, 0u};                               // (a key of 0 has digit 0 everywhere: counted by nobody)
                if (ik < quads) kqs[k] = keys4[ik];
                else if (ik == quads) { const uint32_t have = (uint32_t)(n - 4 * quads); for (uint32_t j = 0; j < have; ++j) kqs[k][j] = keys[4 * quads + j]; }
            }
            i += 3 * stride;
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const u32x4 kq = kqs[k];
                uint32_t is[4][3];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t lo = kq[j] & 0x55555555u, hi = (kq[j] >> 1) & 0x55555555u;
                    is[j][0] = lo & ~hi; is[j][1] = hi & ~lo; is[j][2] = lo & hi;
                }
#pragma unroll
                for (int d = 0; d < 3; ++d) {
                    const uint32_t a = is[0][d] + is[1][d], b = is[2][d] + is[3][d];      // 2-bit fields, at most 2 each
                    even[d] += (a & 0x33333333u) + (b & 0x33333333u);
                    odd[d] += ((a >> 2) & 0x33333333u) + ((b >> 2) & 0x33333333u);
                }
            }
#pragma unroll
            for (int d = 0; d < 3; ++d) {
                packed[d][0] += even[d] & 0x0F0F0F0Fu;
                packed[d][2] += (even[d] >> 4) & 0x0F0F0F0Fu;
                packed[d][1] += odd[d] & 0x0F0F0F0Fu;
                packed[d][3] += (odd[d] >> 4) & 0x0F0F0F0Fu;
            }
        }
#pragma unroll
        for (int d = 0; d < 3; ++d)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int b = 0; b < 4; ++b) cnt[d][q + 4 * b] += (packed[d][q] >> (8 * b)) & 0xFFu;
    }
#pragma unroll
    for (int d = 0; d < 3; ++d)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const uint32_t w = wave_sum(cnt[d][j]);
            if ((threadIdx.x & 63) == 0 && w) atomicAdd(&s_cnt[4 * j + d + 1], w);
        }
    __syncthreads();
    if (threadIdx.x < 64 && (threadIdx.x & 3) && s_cnt[threadIdx.x]) atomicAdd(&counts[threadIdx.x], s_cnt[threadIdx.x]);
}

// counts[4 j] = n - counts[4 j + 1] - counts[4 j + 2] - counts[4 j + 3]
__global__ void digit_zero_counts_kernel(uint32_t *counts, size_t n)
{
    const int j = threadIdx.x;
    if (j < 16) counts[4 * j] = (uint32_t)n - counts[4 * j + 1] - counts[4 * j + 2] - counts[4 * j + 3];
}

// The words x of one wavefront's run put in order in the wavefront's slot: digit 0's first, then digit 1's, 2's, 3's,
// each in the old order (cnt[d] of them).  Nothing here depends on where the ranges go in the destination, so this
// runs while the tile's predecessors are still publishing: if `polling`, the chain is polled once per result block.
// `slots` is the workgroup's array of slots and slot0 this wavefront's first word in it: positions are kept as word
// offsets into the array, two to a register (16-bit halves), so that picking the one for a key's digit is one byte
// permute.  Words past the end of a ragged run go to the slot's spare last word.
template <int NT, uint32_t SLOT, class Chain>
__device__ __forceinline__ void split4_order(int lane, const typename Tr<TCUSCAN_I8_I32>::AConst &Aex, const u32x4 (&gA)[NT],
                                             const u32x4 (&gB)[NT], const u32x4 (&key)[NT][4], int bit, const u32x4 (&x)[NT][4],
                                             const uint32_t (&cnt)[4], uint32_t rem, uint32_t *slots, uint32_t slot0, Chain &chain, bool polling)
{
    using T = Tr<TCUSCAN_I8_I32>;
    const bool ragged = rem < NT * 1024u;
    uint32_t runA = slot0 | ((slot0 + cnt[0]) << 16);                 // where the next key of digit 0 / 1 goes (two halves)
    uint32_t runB = (slot0 + cnt[0] + cnt[1]) | ((slot0 + cnt[0] + cnt[1] + cnt[2]) << 16);      // ... of digit 2 / 3
    const uint32_t in_blk = 16u * (lane & 15) + 4u * (lane >> 4);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const u32x4 ttA = bits<u32x4>(T::totals(Aex, gA[t])), ttB = bits<u32x4>(T::totals(Aex, gB[t]));
#pragma unroll
        for (int p = 0; p < T::kBlocks; ++p) {
            const i32x4 z = {0, 0, 0, 0};                            // same-digit keys before this one in its granule:
            const i32x4 dA = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aex.a[p], bits<i32x4>(gA[t]), z, 0, 0, 0);   // result block p
            const i32x4 dB = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aex.a[p], bits<i32x4>(gB[t]), z, 0, 0, 0);
            const uint32_t pairA = (ttA[p] & 63u) | ((ttA[p] >> 6) << 16), pairB = (ttB[p] & 63u) | ((ttB[p] >> 6) << 16);
            const uint32_t exA = row_exclusive_scan(pairA), exB = row_exclusive_scan(pairB);
            const uint32_t blkA = uniform_from_lane(exA + pairA, 15), blkB = uniform_from_lane(exB + pairB, 15);
            const uint32_t baseA = runA + exA, baseB = runB + exB;
            const uint32_t idx0 = (uint32_t)t * 1024u + 256u * p + in_blk;
            uint32_t at[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t d = (key[t][p][r] >> bit) & 3u;
                // half d of {baseB : baseA}: bytes 2 d and 2 d + 1 of the pair, zeros above
                const uint32_t bs = __builtin_amdgcn_perm(baseB, baseA, 0x0c0c0100u + 0x0202u * d);
                // the four 6-bit counts of the two products side by side, field d of them
                const uint32_t ranks = (uint32_t)dA[r] | ((uint32_t)dB[r] << 12);
                at[r] = bs + ((ranks >> (6u * d)) & 63u);
            }
            if (ragged) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (idx0 + r >= rem) at[r] = slot0 + SLOT - 1u;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) slots[at[r]] = x[t][p][r];
            runA += blkA; runB += blkB;
            if (polling) chain.poll();
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The four ordered ranges of the slot to the destination: digit d's from dst[at0[d]] on.
__device__ __forceinline__ void split4_store(int lane, const uint32_t *slot, uint32_t *dst, const uint64_t (&at0)[4], const uint32_t (&cnt)[4],
                                             uint64_t n)
{
    uint32_t q = 0u;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint64_t room = at0[d] < n ? n - at0[d] : 0u;
        split_store_range(lane, slot, q, cnt[d], dst + at0[d], (uint32_t)(room < 0x40000000ull ? room : 0x40000000ull));
        q += cnt[d];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int NT, int W, bool VALS>
__global__ __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(VALS ? 1 : 4))) void split4_kernel(Params P, Split4Args S)
{
    constexpr int DT = TCUSCAN_I8_I32;
    using T = Tr<DT>;
    static_assert(T::kBlocks == 4 && W >= 4, "four result blocks of 256 per MFMA tile; one wavefront per digit for the carry chain");
    constexpr uint32_t kEPW = NT * Geo<DT>::kTileElems;
    constexpr uint32_t kSlot = kEPW + 16u;                      // the run in order, and a spare last word
    static_assert(W * kSlot < 65536u, "positions in the workgroup's slots travel in 16-bit halves");
    __shared__ uint32_t s_cnt[W][2];
    __shared__ uint32_t s_prefix[4];
    __shared__ __attribute__((aligned(16))) uint32_t s_pack[W][kSlot];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t tile = take_tile(P, &s_prefix[0]), tag = P.tag;
    const uint64_t n = P.cols;
    const uint64_t base = ((uint64_t)tile * W + wave) * kEPW;                       // first key of this wavefront's run
    const uint32_t rem = base < n ? (n - base < 0x40000000ull ? (uint32_t)(n - base) : 0x40000000u) : 0u;
    const int bit = S.bit;
    const uint32_t in_blk = 16u * (lane & 15) + 4u * (lane >> 4);
    const bool ragged = rem < kEPW;

    // ---- the keys; their digit flags as bytes for the two products; this lane's keys per digit
    u32x4 key[NT][4], gA[NT], gB[NT];
    __builtin_amdgcn_s_setprio(3);                  // loads first, as in scan_kernel
    load_run_words<NT>(lane, S.keys + base, rem, ~0u, key);
    __builtin_amdgcn_s_setprio(0);
    uint32_t sumA = 0u, sumB = 0u;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        uint32_t wA[4], wB[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            // the four digits in the four bytes of one word, then all four flag bytes at once: 1 or 64 by the digit's
            // low bit, to stream B where its high bit is set and to stream A where it is not
            uint32_t dig = 0u;
            for (int i = 0; i < 4; ++i) dig |= ((key[t][p][i] >> bit) & 3u) << (8 * i);
            uint32_t one = 0x01010101u + 63u * (dig & 0x01010101u);
            if (ragged) {
                const uint32_t idx0 = (uint32_t)t * 1024u + 256u * p + in_blk;            // keys past the end: no flag
                const uint32_t have = idx0 >= rem ? 0u : (rem - idx0 >= 4u ? 4u : rem - idx0);
                one &= have == 4u ? ~0u : ((1u << (8u * have)) - 1u);
            }
            const uint32_t high = ((dig >> 1) & 0x01010101u) * 255u;
            wB[p] = one & high;
            wA[p] = one ^ wB[p];
            sumA = __builtin_amdgcn_udot4(wA[p], 0x01010101u, sumA, false);    // bytes added up: digit 0 (2) counts 1, digit 1 (3) counts 64
            sumB = __builtin_amdgcn_udot4(wB[p], 0x01010101u, sumB, false);
        }
        gA[t] = rows_transpose(wA);
        gB[t] = rows_transpose(wB);
    }
    static_assert(NT * 16 < 64, "a lane's keys per digit stay below 64: the two counts of a byte sum do not mix");
    const uint32_t c01 = (sumA & 63u) | ((sumA >> 6) << 16), c23 = (sumB & 63u) | ((sumB >> 6) << 16);
    const uint32_t run01 = wave_sum(c01), run23 = wave_sum(c23);                    // at most 2048 per half
    if (lane == 0) { s_cnt[wave][0] = run01; s_cnt[wave][1] = run23; }
    __syncthreads();
    uint32_t off01 = 0u, off23 = 0u, wg01 = 0u, wg23 = 0u;
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const uint32_t v01 = s_cnt[w][0], v23 = s_cnt[w][1];
        if (w < wave) { off01 += v01; off23 += v23; }
        wg01 += v01; wg23 += v23;
    }

    // ---- the carry chain sets out: wavefront d < 4 publishes the tile's count of digit d in its word of the tile's
    // status slot and asks for the words of the tiles before
    const bool chained = P.num_tiles > 1 && wave < 4;
    uint64_t *row_status = (uint64_t *)(P.ws + 1) + (wave & 3);
    const uint32_t mine = ((wave & 2 ? wg23 : wg01) >> (16 * (wave & 1))) & 0xFFFFu;
    LookBackPoll<uint32_t> lb;
    lb.done = true;
    if (chained) {
        if (lane == 0)
            __hip_atomic_store(row_status + (size_t)tile * kStatusStride, status_word(tag, tile == 0 ? kStatePrefix : kStateAggregate, mine),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lb.start(row_status, (int)tile, tag);
    }

    // ---- meanwhile the run is put in order in the slot
    uint32_t cnt[4];
#pragma unroll
    for (int d = 0; d < 4; ++d)
        cnt[d] = (uint32_t)__builtin_amdgcn_readfirstlane((int)(((d & 2 ? run23 : run01) >> (16 * (d & 1))) & 0xFFFFu));
    const typename T::AConst Aex = T::make(lane, true, false);
    split4_order<NT, kSlot>(lane, Aex, gA, gB, key, bit, key, cnt, rem, &s_pack[0][0], (uint32_t)wave * kSlot, lb, chained);

    // ---- the chain arrives
    uint32_t prefix[4] = {0u, 0u, 0u, 0u};
    if (P.num_tiles > 1) {
        if (wave < 4) {
            const uint32_t pre = lb.finish(P.ws, P.spin_limit);
            if (lane == 0) {
                if (tile != 0)
                    __hip_atomic_store(row_status + (size_t)tile * kStatusStride, status_word(tag, kStatePrefix, pre + mine),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_prefix[wave] = pre;
            }
        }
        __syncthreads();
#pragma unroll
        for (int d = 0; d < 4; ++d) prefix[d] = s_prefix[d];
    }

    // ---- where this run's keys of each digit go: behind the smaller digits of the whole array, the same digit of the
    // tiles before, of the wavefronts before
    uint64_t at0[4];
    uint64_t bucket = 0u;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t off = ((d & 2 ? off23 : off01) >> (16 * (d & 1))) & 0xFFFFu;
        at0[d] = bucket + prefix[d] + off;
        bucket += S.hist[d];
    }
    split4_store(lane, s_pack[wave], S.keys_out, at0, cnt, n);
    if constexpr (VALS) {
        u32x4 val[NT][4];
        load_run_words<NT>(lane, S.vals + base, rem, 0u, val);
        split4_order<NT, kSlot>(lane, Aex, gA, gB, key, bit, val, cnt, rem, &s_pack[0][0], (uint32_t)wave * kSlot, lb, false);
        split4_store(lane, s_pack[wave], S.vals_out, at0, cnt, n);
    }
}

struct CompactArgs {
    const uint8_t *mask;               // 0 / 1 bytes
    const uint32_t *values;
    uint32_t *out;                     // the kept values, in order
    uint32_t *count;                   // optional: how many
};

template <int NT, int W>
__global__ __launch_bounds__(64 * W) void compact_kernel(Params P, CompactArgs C)
{
    constexpr int DT = TCUSCAN_I8_I32;
    using T = Tr<DT>;
    static_assert(T::kBlocks == 4, "four result blocks of 256 per MFMA tile");
    constexpr uint32_t kEPW = NT * Geo<DT>::kTileElems;
    constexpr uint32_t kSlot = kEPW + 16u;
    __shared__ uint32_t s_wave_total[W];
    __shared__ uint32_t s_bcast;
    __shared__ __attribute__((aligned(16))) uint32_t s_pack[W][kSlot];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint64_t n = P.cols;
    const uint32_t tile = take_tile(P, &s_bcast);
    const uint64_t base = ((uint64_t)tile * W + wave) * kEPW;                       // first element of this wavefront's run
    const uint32_t rem = base < n ? (n - base < 0x40000000ull ? (uint32_t)(n - base) : 0x40000000u) : 0u;

    // ---- the mask granules (lane l: bytes 16 l .. 16 l + 15 of every MFMA tile; nothing beyond the end) and the values
    __builtin_amdgcn_s_setprio(3);                  // loads first, as in scan_kernel
    const uint8_t *m = C.mask + base;
    u32x4 g[NT], val[NT][4];
    if ((((uintptr_t)m) & 15) == 0 && rem >= kEPW) {
#pragma unroll
        for (int t = 0; t < NT; ++t) g[t] = *(const u32x4 *)(m + (uint32_t)t * 1024u + 16u * lane);
    } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint32_t e0 = (uint32_t)t * 1024u + 16u * lane;
            u32x4 x = {0u, 0u, 0u, 0u};
            for (int i = 0; i < 16; ++i)
                if (e0 + i < rem) x[i >> 2] |= (uint32_t)m[e0 + i] << (8 * (i & 3));
            g[t] = x;
        }
    }
    load_run_words<NT>(lane, C.values + base, rem, 0u, val);
    __builtin_amdgcn_s_setprio(0);
    const typename T::AConst Aop = T::make_compact(lane);
    LookBackPoll<uint32_t> lb;
    uint32_t wave_off, kept_run, wg_total;
    flags_set_out<W>(P, tile, lane, wave, reduce_run<DT, NT>(lane, Aop, g), s_wave_total, lb, wave_off, kept_run, wg_total);
    split_order<NT, kSlot, false>(lane, Aop, g, val, kept_run, rem, s_pack[wave], lb, P.num_tiles > 1 && wave == 0);
    const uint32_t kept_before = flags_arrive(P, tile, lane, wave, wg_total, lb, &s_bcast);
    if (C.count && tile == P.num_tiles - 1 && threadIdx.x == 0) *C.count = kept_before + wg_total;
    split_store<false>(lane, s_pack[wave], C.out, kept_before + wave_off, 0u, kept_run, 0u, n);
}

// ------------------------------------------------------------- segmented scans, short rows
//
// Rows of a few hundred elements: a tile is one wavefront's run of kSegShortNT MFMA tiles, a wavefront takes
// kSegUnroll consecutive tiles and a workgroup is kSegPack such wavefronts that share nothing (no LDS, no barrier).
// A wavefront moves little data per tile, and descriptor -> loads -> products -> stores is a chain of waits, so
// the descriptors and loads of all its tiles are issued before anything is waited for; packing makes the grid smaller
// (it is an upper bound, and a workgroup that finds nothing to do still costs a dispatch).  Rows longer than a tile
// are chained through status words like everywhere else; a wavefront finishes its tiles in order, so a tile still
// waits only for tiles that were started no later than itself.
constexpr int kSegShortNT = 2;
constexpr int kSegUnroll = 2;
constexpr int kSegPack = 4;

template <int DT, bool EXCL, bool REV>
__global__ __launch_bounds__(64 * kSegPack) void seg_short_kernel(Params P)
{
    using T = Tr<DT>;
    using A = typename T::acc;
    constexpr int NT = kSegShortNT, U = kSegUnroll;
    constexpr uint32_t kTile = NT * Geo<DT>::kTileElems;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    uint32_t slot = blockIdx.x * kSegPack + (uint32_t)wave;            // which group of U tiles this wavefront takes
    if (P.ticket) {                                                    // ticket policy: one draw per wavefront (they share nothing)
        uint32_t t = 0u;
        if (lane == 0) t = __hip_atomic_fetch_add(&P.ws->ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        slot = (uint32_t)__builtin_amdgcn_readfirstlane((int)t);
    }
    const uint32_t tile0 = slot * U;

    TileDesc d[U];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        live[u] = tile0 + u < P.num_tiles;
        if (live[u]) d[u] = P.tile_desc[tile0 + u];
        live[u] = live[u] && d[u].tiles_in_row != 0;
    }
    if (!live[0]) return;                             // tiles without a row are the last ones of the grid

    Run R[U];
    u32x4 g[U][NT];
    uint32_t tr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!live[u]) continue;
        tr[u] = tile0 + u - d[u].first_tile;
        const uint32_t pos = REV ? d[u].tiles_in_row - 1 - tr[u] : tr[u];
        R[u] = make_seg_run<DT>(P, d[u].off, d[u].len, seg_lead<DT>(P, d[u].off), (uint64_t)pos * kTile);
        load_run<DT, NT, REV, true>(R[u], lane, g[u]);
    }
    const typename T::AConst Aop = T::make(lane, EXCL, REV);

    // totals first, for all tiles: whoever waits for them is not held up by this wavefront's own look-back
    A total[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!live[u]) continue;
        total[u] = reduce_run<DT, NT>(lane, Aop, g[u]);
        if (d[u].tiles_in_row > 1 && lane == 0) {
            uint64_t *row_status = (uint64_t *)(P.ws + 1) + (uint64_t)d[u].first_tile * kStatusStride;
            __hip_atomic_store(row_status + (size_t)tr[u] * kStatusStride,
                               status_word(P.tag, tr[u] == 0 ? kStatePrefix : kStateAggregate, acc_bits(total[u])),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!live[u]) continue;
        A prefix = acc_from_bits<A>(0u);
        if (d[u].tiles_in_row > 1 && tr[u] != 0) {
            uint64_t *row_status = (uint64_t *)(P.ws + 1) + (uint64_t)d[u].first_tile * kStatusStride;
            prefix = look_back<A>(row_status, (int)tr[u], P.tag, P.ws, P.spin_limit);
            if (lane == 0)
                __hip_atomic_store(row_status + (size_t)tr[u] * kStatusStride,
                                   status_word(P.tag, kStatePrefix, acc_bits(acc_add(prefix, total[u]))),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        scan_and_store<DT, NT, EXCL, REV, true>(lane, Aop, R[u], g[u], prefix);
    }
}

// ------------------------------------------------------------- segmented scans, short rows of 32-bit elements
//
// Rows of a few hundred 32-bit elements do not get tiles of their own: the rows lie back to back, so the whole range
// [offsets[0], offsets[rows]) is tiled like one long row -- every load and store instruction full, no descriptor per
// tile -- and the row starts come in as one bit per element (set by seg_heads_kernel from the offsets).  The scan is
// then the segmented one, sums restart at every set bit:
//   level 0   a lane's granule (4 elements): the MFMA product with the triangular blocks as everywhere else; a granule
//             with a row start at its element 1, 2 or 3 is redone by the lane in three dependent adds (the operand is
//             the same for the 16 granules of a product, so it cannot know where one of them is cut -- and subtracting
//             the part before the cut would not be exact in floating point);
//   levels 1, 2   (sum since the last row start, "a row starts here") pairs scanned over the 64 lanes with DPP shifts:
//             a pair that has a start keeps its sum, the others add the incoming one;
//   beyond    the pair of the wavefront's run, of the workgroup, of the tile.  A tile that contains a row start knows
//             what its successors need without asking anybody -- it publishes its pair as a finished prefix at once --
//             so with short rows the carry chain is one hop long, and with long rows it is the usual one.
// The results stay in the registers that held the inputs (one granule in, one granule out) while the tile waits for
// what comes before it; that sum is then added to the elements that no row start precedes within the tile.
// A reverse scan is the same in mirrored order, restarting at row ends.

__global__ void seg_heads_kernel(const long long *offsets, size_t rows, size_t total, uint32_t shift, uint32_t *heads, WsHeader *ws)
{
    const size_t r = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    const long long off = offsets[r], end = offsets[r + 1];
    const bool bad = off < 0 || end < off || (unsigned long long)end > total;
    if (bad) __hip_atomic_store(&ws->fault, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((end > off || bad) && off >= 0 && (unsigned long long)off < total) {   // (a bad row still ends the row before it)
        const uint64_t b = (uint64_t)off + shift;                      // bit of element i: i + shift (granules start at multiples of 4)
        atomicOr(&heads[b >> 5], 1u << (b & 31));
    }
    if (r == rows - 1 && !bad) {                                       // behind the last row: its last element ends a row (reverse scans)
        const uint64_t b = (uint64_t)end + shift;
        atomicOr(&heads[b >> 5], 1u << (b & 31));
    }
}

// (sum since the last row start, a row starts at or before here) of lanes 0 .. l, in lane l
template <class A> __device__ __forceinline__ void seg_wave_inclusive(A &v, uint32_t &h)
{
#define TCUSCAN_SEG_STEP(CTRL)                                                        \
    {                                                                                 \
        const A vu = dpp_shr<A, CTRL>(v);                                             \
        const uint32_t hu = dpp0<CTRL>(h);                                            \
        v = h ? v : acc_add(vu, v);                                                   \
        h |= hu;                                                                      \
    }
    TCUSCAN_SEG_STEP(kRowShr + 1)
    TCUSCAN_SEG_STEP(kRowShr + 2)
    TCUSCAN_SEG_STEP(kRowShr + 4)
    TCUSCAN_SEG_STEP(kRowShr + 8)
#undef TCUSCAN_SEG_STEP
    {   // the row before, into rows 1 and 3
        const A vu = acc_from_bits<A>((uint32_t)__builtin_amdgcn_update_dpp(0, (int)acc_bits(v), kRowBcast15, 0xa, 0xf, false));
        const uint32_t hu = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)h, kRowBcast15, 0xa, 0xf, false);
        v = h ? v : acc_add(vu, v);
        h |= hu;
    }
    {   // rows 0 and 1, into rows 2 and 3
        const A vu = acc_from_bits<A>((uint32_t)__builtin_amdgcn_update_dpp(0, (int)acc_bits(v), kRowBcast31, 0xc, 0xf, false));
        const uint32_t hu = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)h, kRowBcast31, 0xc, 0xf, false);
        v = h ? v : acc_add(vu, v);
        h |= hu;
    }
}

// From the pair of a wavefront's run -- (sum since the last row start, "there is a row start") -- to the sum the open row
// brings to the start of that run: the pairs of the workgroup's wavefronts through LDS, combined in processing order
// (a reverse scan takes the wavefronts from the last to the first), then the carry chain between tiles.  A tile that
// contains a row start publishes its pair as a finished prefix at once: nothing before it matters to the tiles after
// it; the others publish a total, look back, and publish their prefix.
template <class A, int W, bool REV>
__device__ __forceinline__ A seg_open_sum_before_run(const Params &P, uint32_t tile, int lane, int wave, A carry, bool run_open,
                                                     uint32_t *s_sum, uint32_t *s_head, uint32_t *s_bcast)
{
    const uint32_t tag = P.tag;
    if (lane == 0) { s_sum[wave] = acc_bits(carry); s_head[wave] = run_open ? 0u : 1u; }
    __syncthreads();
    A before = acc_from_bits<A>(0u), wg_sum = acc_from_bits<A>(0u);       // of the wavefronts before this one / of all of them
    bool before_head = false, wg_head = false;
#pragma unroll
    for (int k = 0; k < W; ++k) {
        const int w = REV ? W - 1 - k : k;
        const A v = acc_from_bits<A>(s_sum[w]);
        const bool hd = s_head[w] != 0u;
        if (REV ? w > wave : w < wave) { before = hd ? v : acc_add(before, v); before_head = before_head || hd; }
        wg_sum = hd ? v : acc_add(wg_sum, v);
        wg_head = wg_head || hd;
    }
    A prefix = acc_from_bits<A>(0u);
    if (P.num_tiles > 1) {
        uint64_t *row_status = (uint64_t *)(P.ws + 1);
        if (wave == 0) {
            if (tile == 0 || wg_head) {
                if (lane == 0)
                    __hip_atomic_store(row_status + (size_t)tile * kStatusStride, status_word(tag, kStatePrefix, acc_bits(wg_sum)),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (tile != 0) prefix = look_back<A>(row_status, (int)tile, tag, P.ws, P.spin_limit);
            } else {
                if (lane == 0)
                    __hip_atomic_store(row_status + (size_t)tile * kStatusStride, status_word(tag, kStateAggregate, acc_bits(wg_sum)),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                prefix = look_back<A>(row_status, (int)tile, tag, P.ws, P.spin_limit);
                if (lane == 0)
                    __hip_atomic_store(row_status + (size_t)tile * kStatusStride, status_word(tag, kStatePrefix, acc_bits(acc_add(prefix, wg_sum))),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (lane == 0) *s_bcast = acc_bits(prefix);
        }
        __syncthreads();
        prefix = acc_from_bits<A>(*s_bcast);
    }
    return before_head ? before : acc_add(prefix, before);
}

template <int DT, int NT, bool EXCL, bool REV, int W>
__global__ __launch_bounds__(64 * W) void seg_flat_kernel(Params P, const long long *offsets, const uint32_t *heads, uint32_t shift)
{
    using T = Tr<DT>;
    using A = typename T::acc;
    static_assert(T::kLinear && T::kG == 4 && NT <= 8, "32-bit elements: a lane keeps its granule; 4 flag bits per granule in one word");
    constexpr uint32_t kEPW = NT * Geo<DT>::kTileElems;
    constexpr uint32_t kWgElems = kEPW * W;
    __shared__ uint32_t s_sum[W], s_head[W];
    __shared__ uint32_t s_bcast;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t tile = take_tile(P, &s_bcast);

    // the range the rows cover, clamped to the arrays (offsets that leave them have raised the fault word already)
    long long lo = offsets[0], hi = offsets[P.rows];
    const long long total = (long long)P.cols;
    lo = lo < 0 ? 0 : (lo > total ? total : lo);
    hi = hi < lo ? lo : (hi > total ? total : hi);
    const uint32_t lead = seg_lead<DT>(P, lo);
    const uint64_t vlen = (uint64_t)(hi - lo) + lead;
    const uint64_t tiles = (vlen + kWgElems - 1) / kWgElems;
    if (tile >= tiles) return;                                 // the grid is an upper bound
    const uint64_t pos = REV ? tiles - 1 - tile : tile;        // a reverse scan starts at the end of the range
    const uint64_t base = pos * kWgElems + (uint64_t)wave * kEPW;
    const Run R = make_seg_run<DT>(P, lo, (uint64_t)(hi - lo), lead, base);
    // Everything below works in processing order: element i of a granule is its memory element mem(i); a reverse scan
    // mirrors the granules of the run (slot_offset), the elements inside a granule, the wavefronts and the tiles, and
    // restarts at row ENDS -- element j ends a row when a row starts at j + 1 (the kernel that sets the bits also sets
    // the one behind the last row).
    auto mem = [](int i) { return REV ? 3 - i : i; };

    // a run that lies inside the range as a whole (all but the first and the last few) takes straight-line loads and stores
    const bool whole_in = !REV && __builtin_amdgcn_readfirstlane((int)(R.in_vec && R.lead == 0u && R.rem >= kEPW)) != 0;
    const bool whole_out = __builtin_amdgcn_readfirstlane((int)(R.out_vec && R.lead == 0u && R.rem >= kEPW)) != 0;   // (either direction)
    __builtin_amdgcn_s_setprio(3);                  // loads first, as in scan_kernel
    u32x4 g[NT];
    // row starts among this lane's elements: 4 bits per granule, granule t in bits 4t .. 4t + 3
    const uint64_t bit0 = (uint64_t)(lo - (long long)lead) + base + shift;     // bit of the run's first slot (a multiple of 4)
    uint32_t starts = 0u;
    if (whole_in) {
#pragma unroll
        for (int t = 0; t < NT; ++t) g[t] = *(const u32x4 *)(R.in + ((uint32_t)t * 256u + 4u * lane) * 4u);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint64_t b = bit0 + (uint32_t)t * 256u + 4u * lane;
            starts |= ((heads[b >> 5] >> (b & 31)) & 0xFu) << (4 * t);
        }
    } else {
        load_run<DT, NT, REV, true>(R, lane, g);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint32_t e0 = slot_offset<DT, NT, REV>(t, lane);
            if (e0 < R.rem) {
                const uint64_t b = bit0 + e0;
                if constexpr (REV) {
                    const uint64_t w = (uint64_t)heads[b >> 5] | ((uint64_t)heads[(b >> 5) + 1] << 32);
                    const uint32_t ends = (uint32_t)(w >> ((b & 31) + 1)) & 0xFu;                     // memory order
                    starts |= (((ends & 1u) << 3) | ((ends & 2u) << 1) | ((ends & 4u) >> 1) | ((ends & 8u) >> 3)) << (4 * t);
                } else {
                    starts |= ((heads[b >> 5] >> (b & 31)) & 0xFu) << (4 * t);
                }
            }
        }
    }

    __builtin_amdgcn_s_setprio(0);
    // ---- the run by itself: segmented scan in place, (sum since the last row start, any row start) of the run
    const typename T::AConst Aop = T::make(lane, false, REV);
    A carry = acc_from_bits<A>(0u);                            // sum since the last row start, up to the end of the tile before
    bool run_open = true;                                      // no row start in the run so far
    uint32_t open = 0u;                                        // bit t: no row start in the run before this lane's granule of tile t
    A in[NT];                                                  // what the open row brings into that granule from inside the run
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const uint32_t fb = (starts >> (4 * t)) & 0xFu;
        A y[4];
        if (__ballot((fb & 0xEu) != 0u) == 0ull) {             // no granule of this tile is cut: the product is the scan
            typename T::acc4 d[1];
            T::mma(Aop, g[t], lane, false, REV, d);
            for (int i = 0; i < 4; ++i) y[i] = acc_from_bits<A>(bits<u32x4>(d[0])[mem(i)]);
        } else {                                               // three dependent adds; a row start drops what came before
            y[0] = acc_from_bits<A>(g[t][mem(0)]);
            for (int i = 1; i < 4; ++i) {
                const uint32_t keep = (uint32_t)(((int32_t)(~fb << (31 - i))) >> 31);       // all ones unless a row starts at i
                y[i] = acc_add(acc_from_bits<A>(acc_bits(y[i - 1]) & keep), acc_from_bits<A>(g[t][mem(i)]));
            }
        }
        for (int i = 0; i < 4; ++i) g[t][mem(i)] = acc_bits(y[i]);
        A v = y[3];
        uint32_t h = fb ? 1u : 0u;
        seg_wave_inclusive(v, h);
        const A vex = wave_shift_up(v);
        const uint32_t hex = dpp0<kWaveShr1>(h);
        in[t] = hex ? vex : acc_add(carry, vex);
        if (run_open && !hex) open |= 1u << t;
        carry = uniform_from_lane(fb ? y[3] : acc_add(in[t], y[3]), 63);
        run_open = run_open && __ballot(fb != 0u) == 0ull;
    }

    // ---- the wavefronts of the workgroup, then the tiles before this one: the open row's sum at the start of this run
    const A wave_in = seg_open_sum_before_run<A, W, REV>(P, tile, lane, wave, carry, run_open, s_sum, s_head, &s_bcast);

    // ---- what the open row brings, to the elements that no row start of their granule precedes; store
    A last = wave_in;                                          // the inclusive result of the element before the granule (exclusive scans)
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const uint32_t fb = (starts >> (4 * t)) & 0xFu;
        const A add = ((open >> t) & 1u) ? acc_add(wave_in, in[t]) : in[t];
        const uint32_t first = fb ? (uint32_t)__builtin_ctz(fb) : 4u;     // elements before the granule's first row start
        A y[4];
        for (int i = 0; i < 4; ++i) {
            y[i] = acc_from_bits<A>(g[t][mem(i)]);
            if ((uint32_t)i < first) y[i] = acc_add(add, y[i]);
        }
        u32x4 v;
        if constexpr (EXCL) {
            A prev = wave_shift_up(y[3]);
            if (lane == 0) prev = last;
            last = uniform_from_lane(y[3], 63);
            v[mem(0)] = (fb & 1u) ? 0u : acc_bits(prev);
            for (int i = 1; i < 4; ++i) v[mem(i)] = ((fb >> i) & 1u) ? 0u : acc_bits(y[i - 1]);
        } else {
            for (int i = 0; i < 4; ++i) v[mem(i)] = acc_bits(y[i]);
        }
        const uint32_t e0 = slot_offset<DT, NT, REV>(t, lane);
        if (whole_out) {
            __builtin_nontemporal_store(v, (u32x4 *)(R.out + e0 * 4));
        } else if (R.out_vec && e0 + 4 <= R.rem && e0 >= R.lead) {
            __builtin_nontemporal_store(v, (u32x4 *)(R.out + e0 * 4));
        } else {
            for (int i = 0; i < 4; ++i)
                if (e0 + i < R.rem && e0 + i >= R.lead) ((uint32_t *)R.out)[e0 + i] = v[i];
        }
    }
}

// ---- the same for 8- and 16-bit inputs
//
// A lane's granule is 16 or 8 elements, and the matrix unit would hand its results to four or two other lanes (the
// result layout that makes the plain scan's stores contiguous).  Here level 0 stays in the lane: the granule is
// unpacked and scanned by dependent adds that drop what came before a row start, so the lane that knows a granule's
// row starts also holds all of its results; everything above level 0 is the 32-bit kernel's.  The results -- four or two
// 16-byte groups per lane -- change lanes just before the store (lane swaps: a 4 x 4 or 2 x 2 transpose between
// registers and lane rows), so that every store instruction still writes 1 KiB of consecutive outputs.

template <int DT> __device__ __forceinline__ typename Tr<DT>::acc narrow_elem(const u32x4 &g, int i);
template <> __device__ __forceinline__ uint32_t narrow_elem<TCUSCAN_I8_I32>(const u32x4 &g, int i)
{
    return (uint32_t)(int32_t)(int8_t)(uint8_t)(g[i >> 2] >> (8 * (i & 3)));
}
template <> __device__ __forceinline__ float narrow_elem<TCUSCAN_BF16_F32>(const u32x4 &g, int i)
{
    return bits<float>((i & 1) ? (g[i >> 1] & 0xFFFF0000u) : (g[i >> 1] << 16));
}
template <> __device__ __forceinline__ float narrow_elem<TCUSCAN_F16_F32>(const u32x4 &g, int i)
{
    return (float)bits<_Float16>((uint16_t)(g[i >> 1] >> (16 * (i & 1))));
}

template <int DT, bool EXCL, bool REV, int W>
__global__ __launch_bounds__(64 * W) void seg_flat_narrow_kernel(Params P, const long long *offsets, const uint32_t *heads, uint32_t shift)
{
    using T = Tr<DT>;
    using A = typename T::acc;
    constexpr int G = T::kG, NT = 32 / G, Q = G / 4;           // elements per granule, granules per lane, 16-byte result groups per granule
    static_assert(G == 8 || G == 16, "8- and 16-bit inputs");
    constexpr uint32_t kTile = 64u * G;                        // elements one load instruction of the wavefront covers
    constexpr uint32_t kEPW = NT * kTile;                      // 2048
    constexpr uint32_t kWgElems = kEPW * W;
    constexpr uint32_t kMask = (1u << G) - 1u;
    __shared__ uint32_t s_sum[W], s_head[W];
    __shared__ uint32_t s_bcast;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t tile = take_tile(P, &s_bcast);

    long long lo = offsets[0], hi = offsets[P.rows];
    const long long total = (long long)P.cols;
    lo = lo < 0 ? 0 : (lo > total ? total : lo);
    hi = hi < lo ? lo : (hi > total ? total : hi);
    const uint32_t lead = seg_lead<DT>(P, lo);
    const uint64_t vlen = (uint64_t)(hi - lo) + lead;
    const uint64_t tiles = (vlen + kWgElems - 1) / kWgElems;
    if (tile >= tiles) return;                                 // the grid is an upper bound
    const uint64_t pos = REV ? tiles - 1 - tile : tile;        // a reverse scan starts at the end of the range
    const uint64_t base = pos * kWgElems + (uint64_t)wave * kEPW;
    const Run R = make_seg_run<DT>(P, lo, (uint64_t)(hi - lo), lead, base);
    auto mem = [](int i) { return REV ? G - 1 - i : i; };      // processing order -> element of the granule (as in seg_flat_kernel)
    const bool whole_in = !REV && __builtin_amdgcn_readfirstlane((int)(R.in_vec && R.lead == 0u && R.rem >= kEPW)) != 0;
    const bool whole_out = __builtin_amdgcn_readfirstlane((int)(R.out_vec && R.lead == 0u && R.rem >= kEPW)) != 0;

    __builtin_amdgcn_s_setprio(3);                  // loads first, as in scan_kernel
    u32x4 g[NT];
    const uint64_t bit0 = (uint64_t)(lo - (long long)lead) + base + shift;     // bit of the run's first slot (a multiple of G)
    uint32_t starts = 0u;                                      // G bits per granule, granule t in bits G t ..
    if (whole_in) {
#pragma unroll
        for (int t = 0; t < NT; ++t) g[t] = *(const u32x4 *)(R.in + ((uint32_t)t * kTile + (uint32_t)G * lane) * T::kEsz);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint64_t b = bit0 + (uint32_t)t * kTile + (uint32_t)G * lane;
            starts |= ((heads[b >> 5] >> (b & 31)) & kMask) << (G * t);
        }
    } else {
        load_run<DT, NT, REV, true>(R, lane, g);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint32_t e0 = slot_offset<DT, NT, REV>(t, lane);
            if (e0 < R.rem) {
                const uint64_t b = bit0 + e0;
                if constexpr (REV) {                           // row ends: a row starts one element further on; mirrored
                    const uint64_t w = (uint64_t)heads[b >> 5] | ((uint64_t)heads[(b >> 5) + 1] << 32);
                    const uint32_t ends = (uint32_t)(w >> ((b & 31) + 1)) & kMask;
                    starts |= (__builtin_bitreverse32(ends) >> (32 - G)) << (G * t);
                } else {
                    starts |= ((heads[b >> 5] >> (b & 31)) & kMask) << (G * t);
                }
            }
        }
    }

    __builtin_amdgcn_s_setprio(0);
    // ---- the run by itself
    A y[NT][G];
    A carry = acc_from_bits<A>(0u);
    bool run_open = true;
    uint32_t open = 0u;
    A in[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const uint32_t fb = (starts >> (G * t)) & kMask;
        y[t][0] = narrow_elem<DT>(g[t], mem(0));
#pragma unroll
        for (int i = 1; i < G; ++i) {
            const uint32_t keep = (uint32_t)(((int32_t)(~fb << (31 - i))) >> 31);           // all ones unless a row starts at i
            y[t][i] = acc_add(acc_from_bits<A>(acc_bits(y[t][i - 1]) & keep), narrow_elem<DT>(g[t], mem(i)));
        }
        A v = y[t][G - 1];
        uint32_t h = fb ? 1u : 0u;
        seg_wave_inclusive(v, h);
        const A vex = wave_shift_up(v);
        const uint32_t hex = dpp0<kWaveShr1>(h);
        in[t] = hex ? vex : acc_add(carry, vex);
        if (run_open && !hex) open |= 1u << t;
        carry = uniform_from_lane(fb ? y[t][G - 1] : acc_add(in[t], y[t][G - 1]), 63);
        run_open = run_open && __ballot(fb != 0u) == 0ull;
    }

    // ---- the wavefronts of the workgroup, then the tiles before this one: the open row's sum at the start of this run
    const A wave_in = seg_open_sum_before_run<A, W, REV>(P, tile, lane, wave, carry, run_open, s_sum, s_head, &s_bcast);

    // ---- the open row's sum to the elements that no row start of their granule precedes; results change lanes; store
    A last = wave_in;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const uint32_t fb = (starts >> (G * t)) & kMask;
        const A add = ((open >> t) & 1u) ? acc_add(wave_in, in[t]) : in[t];
        const uint32_t first = fb ? (uint32_t)__builtin_ctz(fb) : (uint32_t)G;
#pragma unroll
        for (int i = 0; i < G; ++i)
            if ((uint32_t)i < first) y[t][i] = acc_add(add, y[t][i]);
        u32x4 v[Q];
        if constexpr (EXCL) {
            A prev = wave_shift_up(y[t][G - 1]);
            if (lane == 0) prev = last;
            last = uniform_from_lane(y[t][G - 1], 63);
            v[mem(0) >> 2][mem(0) & 3] = (fb & 1u) ? 0u : acc_bits(prev);
#pragma unroll
            for (int i = 1; i < G; ++i) v[mem(i) >> 2][mem(i) & 3] = ((fb >> i) & 1u) ? 0u : acc_bits(y[t][i - 1]);
        } else {
#pragma unroll
            for (int i = 0; i < G; ++i) v[mem(i) >> 2][mem(i) & 3] = acc_bits(y[t][i]);
        }
        // group k of the lane in row P (16 lanes) / half P (32 lanes) <- group P of the lane in row / half k, same column
        uint32_t e[Q];                                         // where the group this lane now holds in register k belongs
        if constexpr (Q == 4) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t col[4] = {v[0][w], v[1][w], v[2][w], v[3][w]};
                const u32x4 tr = rows_transpose(col);
                for (int k = 0; k < 4; ++k) v[k][w] = tr[k];
            }
            for (int k = 0; k < 4; ++k) e[k] = slot_offset<DT, NT, REV>(t, 16 * k + (lane & 15)) + 4u * (lane >> 4);
        } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const auto sw = __builtin_amdgcn_permlane32_swap(v[0][w], v[1][w], false, false);
                v[0][w] = sw[0]; v[1][w] = sw[1];
            }
            for (int k = 0; k < 2; ++k) e[k] = slot_offset<DT, NT, REV>(t, 32 * k + (lane & 31)) + 4u * (lane >> 5);
        }
#pragma unroll
        for (int k = 0; k < Q; ++k) {
            if (whole_out || (R.out_vec && e[k] + 4 <= R.rem && e[k] >= R.lead)) {
                __builtin_nontemporal_store(v[k], (u32x4 *)(R.out + e[k] * 4));
            } else {
                for (int i = 0; i < 4; ++i)
                    if (e[k] + i < R.rem && e[k] + i >= R.lead) ((uint32_t *)R.out)[e[k] + i] = v[k][i];
            }
        }
    }
}

// ---------------------------------------------------------------------- short-row kernel
//
// Rows no longer than one wavefront's run (NT tiles): every wavefront scans rows of its own -- no
// totals to exchange, no carry chain, no barrier.  Many short independent rows are the shape of
// the histogram prefix sums in gradient-boosted-tree split finding, one of the paper's two
// motivating applications.

// LEAD: the rows do not start at 16-byte boundaries (odd row lengths, or an unaligned array): every row is then tiled
// from the boundary at or below its start, the elements in front of it read as zero and not written -- what the
// segmented scans do -- so that all full granules still take the 128-bit path (element by element, the same rows
// run at a third of the speed).
template <int DT, int NT, bool EXCL, bool REV, bool LEAD = false>
__global__ __launch_bounds__(kThreads) void scan_rows_kernel(Params P)
{
    using T = Tr<DT>;
    using A = typename T::acc;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint64_t row = (uint64_t)blockIdx.x * kWaves + wave;
    if (row >= P.rows) return;
    u32x4 g[NT];
    const typename T::AConst Aop = T::make(lane, EXCL, REV);
    if constexpr (!LEAD && NT == 2 && T::kEsz != 2) {
        // Two MFMA tiles of 8- or 32-bit elements: one after the other, the first one's total as the second one's
        // carry.  With one KiB per wavefront in flight at a time the memory system does better than with both tiles
        // loaded at once (131072 x 2048 int8 rows 238 -> 215 us, 174762 x 1536 int8 240 -> 225, 524288 x 512 f32 342 ->
        // 331); 16-bit rows gain or lose a per cent or two (262144 x 1024 bf16 260 -> 257, 262144 x 1000 f16 287 -> 295)
        // and keep the plain form, and from three tiles on it is the other way round (174762 x 1536 f16 266 -> 276).
        A carry = acc_from_bits<A>(0u);
        const typename T::AConst Atot = T::make(lane, false, false);
#pragma unroll 1
        for (int k = 0; k < 2; ++k) {
            const uint64_t base = (uint64_t)(REV ? 1 - k : k) * Geo<DT>::kTileElems;     // a reverse scan starts with the last tile
            if (base >= P.cols) continue;
            const Run R1 = make_run<DT>(P, row, base);
            u32x4 g1[1];
            load_run<DT, 1, REV>(R1, lane, g1);
            const A total = k == 0 ? reduce_run<DT, 1>(lane, Atot, g1) : acc_from_bits<A>(0u);
            scan_and_store<DT, 1, EXCL, REV>(lane, Aop, R1, g1, carry);
            carry = total;
        }
    } else if constexpr (!LEAD) {
        const Run R = make_run<DT>(P, row, 0);
        load_run<DT, NT, REV>(R, lane, g);
        scan_and_store<DT, NT, EXCL, REV>(lane, Aop, R, g, acc_from_bits<A>(0u));
    } else {
        Params Q = P;
        Q.cols = P.rows * P.cols;                              // make_seg_run: the length of the arrays (no access beyond it)
        const long long off = (long long)(row * P.cols);
        const Run R = make_seg_run<DT>(Q, off, P.cols, seg_lead<DT>(P, off), 0);
        load_run<DT, NT, REV, true>(R, lane, g);
        scan_and_store<DT, NT, EXCL, REV, true>(lane, Aop, R, g, acc_from_bits<A>(0u));
    }
}

// Segmented scans, step 1: tiles per row.  A row [off, off + len) is tiled from the 16-byte boundary at or below its
// start, so it needs ceil((lead + len) / tile) tiles (none when it is empty).  Offsets that decrease or leave
// [0, total] give the row no tiles and raise the fault word instead of letting the scan touch memory outside the
// caller's arrays.  Entry `rows` is zero: the exclusive scan of this array then ends with the total number of tiles.
// Tiles of row r (a row is tiled from the 16-byte boundary at or below its first element); offsets that leave the
// arrays or run backwards get no tiles and raise fault word 2.
__device__ __forceinline__ int32_t seg_row_tiles(const long long *offsets, size_t r, size_t total, uintptr_t in_addr, uint32_t esz,
                                                 uint32_t tile, WsHeader *ws)
{
    const long long off = offsets[r], end = offsets[r + 1];
    if (off < 0 || end < off || (unsigned long long)end > total) {
        __hip_atomic_store(&ws->fault, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return 0;
    }
    if (end == off) return 0;
    const uint64_t lead = ((in_addr + (uint64_t)off * esz) & 15) / esz;
    return (int32_t)((lead + (uint64_t)(end - off) + tile - 1) / tile);
}

// The descriptor of tile t, given the first tile of every row (tile_start[0 .. rows], in global memory or LDS).
__device__ __forceinline__ TileDesc seg_tile_desc(const uint32_t *tile_start, const long long *offsets, size_t rows, uint32_t t)
{
    TileDesc d = {0, 0ull, 0u, 0u, {0u, 0u}};
    if (t < tile_start[rows]) {
        size_t lo = 0, hi = rows;                 // tile_start[lo] <= t < tile_start[hi]
        while (hi - lo > 1) {
            const size_t mid = (lo + hi) / 2;
            if (tile_start[mid] <= t) lo = mid; else hi = mid;
        }
        d.off = offsets[lo];
        d.len = (unsigned long long)(offsets[lo + 1] - d.off);
        d.first_tile = tile_start[lo];
        d.tiles_in_row = tile_start[lo + 1] - d.first_tile;
    }
    return d;
}

__global__ void seg_tiles_kernel(const long long *offsets, size_t rows, size_t total, uintptr_t in_addr, uint32_t esz,
                                 uint32_t tile, int32_t *counts, WsHeader *ws)
{
    const size_t r = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r > rows) return;
    counts[r] = r < rows ? seg_row_tiles(offsets, r, total, in_addr, esz, tile, ws) : 0;
}
__global__ void seg_desc_kernel(const uint32_t *tile_start, const long long *offsets, size_t rows, TileDesc *desc, uint32_t max_tiles)
{
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= max_tiles) return;
    desc[t] = seg_tile_desc(tile_start, offsets, rows, t);
}

// The three preparation steps and the clearing of the status words in ONE launch, for calls with few rows (ragged
// batches of some hundred sequences: four small launches in front of the scan cost more than they compute).  Every
// workgroup works out the first tile of every row by itself -- kSegPrepRows / 1024 rows per thread, one scan over the
// workgroup in LDS -- and then writes the descriptors and clears the status slots of its own 1024 tiles.
constexpr size_t kSegPrepRows = 4096;                  // rows + 1 entries must fit: calls with fewer rows than this
__global__ __launch_bounds__(1024) void seg_prepare_kernel(const long long *offsets, size_t rows, size_t total, uintptr_t in_addr, uint32_t esz,
                                                           uint32_t tile, TileDesc *desc, uint32_t max_tiles, WsHeader *ws)
{
    constexpr int kPer = (int)(kSegPrepRows / 1024);
    __shared__ uint32_t s_start[kSegPrepRows + 1];
    __shared__ uint32_t s_wave[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t c[kPer], mine = 0u;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const size_t r = (size_t)kPer * threadIdx.x + j;
        c[j] = r < rows ? (uint32_t)seg_row_tiles(offsets, r, total, in_addr, esz, tile, ws) : 0u;
        mine += c[j];
    }
    const uint32_t incl = wave_inclusive_scan(mine);
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    uint32_t before = incl - mine;                       // tiles of the rows of the threads before this one
    for (int w = 0; w < wave; ++w) before += s_wave[w];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const size_t r = (size_t)kPer * threadIdx.x + j;
        if (r <= rows) s_start[r] = before;
        before += c[j];
    }
    __syncthreads();
    const uint32_t t = blockIdx.x * 1024u + threadIdx.x;
    if (t >= max_tiles) return;
    desc[t] = seg_tile_desc(s_start, offsets, rows, t);
    u32x4 *slot = (u32x4 *)((uint64_t *)(ws + 1) + (size_t)t * kStatusStride);
#pragma unroll
    for (int k = 0; k < (int)(8 * kStatusStride / 16); ++k) slot[k] = u32x4{0u, 0u, 0u, 0u};
}

// One 16-byte store per thread where the address allows it (p is 4-byte aligned; the words in front of the first
// 16-byte boundary and behind the last go one by one).
// A second range (p2, words2) is cleared by the blocks behind the first range's `blocks1` blocks: two regions of a
// workspace in one launch.
__global__ void fill_zero_kernel(uint32_t *p, size_t words, uint32_t *p2, size_t words2, unsigned blocks1)
{
    unsigned block = blockIdx.x;
    if (block >= blocks1) { p = p2; words = words2; block -= blocks1; }
    const size_t i = (size_t)block * blockDim.x + threadIdx.x;           // group of four words, counted from the boundary
    const size_t head = ((16u - ((uintptr_t)p & 15u)) & 15u) / 4u;         // words before the first boundary
    const size_t h = head < words ? head : words;
    const size_t first = h + 4 * i;
    if (first + 4 <= words) {
        *(u32x4 *)(p + first) = u32x4{0u, 0u, 0u, 0u};
    } else {
        for (size_t k = first; k < words; ++k) p[k] = 0u;
    }
    if (i == 0)
        for (size_t k = 0; k < h; ++k) p[k] = 0u;
}

// ------------------------------------------------------------------------ host side

constexpr size_t kSmallTile = 8192;                      // elements per workgroup tile, small variant (all dtypes)
constexpr size_t kShortRowMax = 2048;                    // rows up to this length can be scanned one per wavefront
constexpr size_t kShortRowMax32 = 2816;                  // ... 32-bit inputs: up to 11 of their 256-element MFMA tiles
constexpr size_t kShortRowMax8 = 2560;                   // ... 8-bit inputs: two and a half of their 1024-element MFMA tiles
constexpr size_t kShortRowMinRows = 8;                   // ... when there are enough of them to fill wavefronts

bool valid_dtype(int dt) { return dt >= 0 && dt <= 4; }
size_t in_size(int dt) { return dt == TCUSCAN_I8_I32 ? 1 : (dt == TCUSCAN_F16_F32 || dt == TCUSCAN_BF16_F32) ? 2 : 4; }

// MFMA tiles per wavefront and wavefronts per workgroup for the three tile sizes of each dtype.  Small is
// 8192 elements per workgroup for every dtype; large and huge keep 32 .. 128 input registers per lane
// waiting for the carry (the longer the carry chain, the more a big tile pays: fewer status words to
// publish and poll per byte).  For 32-bit inputs the big tiles are 8 wavefronts of 8 or 16 MFMA tiles (16384 /
// 32768 elements): half the registers per wavefront of the same tile made of 4 wavefronts, which measures faster
// on long chains.
template <int DT> struct Tiles;   // MFMA tiles per wavefront (k..) and wavefronts per workgroup (w..) for each tile size
template <> struct Tiles<TCUSCAN_I8_I32>   { static constexpr int kSmall = 2, kLarge = 8,  kHuge = 16, wSmall = 4, wLarge = 4, wHuge = 4; };
template <> struct Tiles<TCUSCAN_F16_F32>  { static constexpr int kSmall = 4, kLarge = 16, kHuge = 32, wSmall = 4, wLarge = 4, wHuge = 4; };
template <> struct Tiles<TCUSCAN_BF16_F32> { static constexpr int kSmall = 4, kLarge = 16, kHuge = 32, wSmall = 4, wLarge = 4, wHuge = 4; };
template <> struct Tiles<TCUSCAN_F32_F32>  { static constexpr int kSmall = 8, kLarge = 8,  kHuge = 16, wSmall = 4, wLarge = 8, wHuge = 8; };
template <> struct Tiles<TCUSCAN_I32_I32>  { static constexpr int kSmall = 8, kLarge = 8,  kHuge = 16, wSmall = 4, wLarge = 8, wHuge = 8; };

enum TileSize { kTileSmall = 0, kTileLarge = 1, kTileHuge = 2 };

template <int DT> size_t tile_elems_dt(int size)
{
    using Ti = Tiles<DT>;
    const size_t per_tile = Geo<DT>::kTileElems;
    return size == kTileHuge ? per_tile * Ti::kHuge * Ti::wHuge : size == kTileLarge ? per_tile * Ti::kLarge * Ti::wLarge
                                                                                    : per_tile * Ti::kSmall * Ti::wSmall;
}

size_t tile_elems(int dt, int size)
{
    switch (dt) {
    case TCUSCAN_I8_I32:   return tile_elems_dt<TCUSCAN_I8_I32>(size);
    case TCUSCAN_F16_F32:  return tile_elems_dt<TCUSCAN_F16_F32>(size);
    case TCUSCAN_BF16_F32: return tile_elems_dt<TCUSCAN_BF16_F32>(size);
    case TCUSCAN_F32_F32:  return tile_elems_dt<TCUSCAN_F32_F32>(size);
    default:               return tile_elems_dt<TCUSCAN_I32_I32>(size);
    }
}
static_assert(Geo<TCUSCAN_I8_I32>::kTileElems * Tiles<TCUSCAN_I8_I32>::kSmall * Tiles<TCUSCAN_I8_I32>::wSmall == kSmallTile &&
              Geo<TCUSCAN_F16_F32>::kTileElems * Tiles<TCUSCAN_F16_F32>::kSmall * Tiles<TCUSCAN_F16_F32>::wSmall == kSmallTile &&
              Geo<TCUSCAN_F32_F32>::kTileElems * Tiles<TCUSCAN_F32_F32>::kSmall * Tiles<TCUSCAN_F32_F32>::wSmall == kSmallTile,
              "the small tile is the same number of elements for every dtype");

// 0 = choose by shape, 1 = always the small tile, 2 / 3 = the large / huge tile whenever a row is longer
// than a small one
std::atomic<int> g_tile_policy{0};

int choose_tile(int dt, size_t rows, size_t cols)
{
    const int f = g_tile_policy.load(std::memory_order_relaxed);
    if (f) return (f == 1 || cols <= kSmallTile) ? kTileSmall : (f == 2 ? kTileLarge : kTileHuge);
    // Measured on MI355X with inputs that come from HBM (every launch of a timing loop on another copy of the input;
    // an input read again within a few hundred MB of reads comes from the memory-side cache in part and shifts these
    // crossovers): 2^28 elements split into rows of 2^14 .. 2^28, and single rows and groups of four rows of 2^18 ..
    // 2^26.  Short carry chains run best on small tiles (loads and stores alternate at a finer grain), long ones on
    // big tiles (fewer status words per byte); the crossover depends on the input width:
    //   8-bit   large beyond 2^17 (rows of 2^16: small 219, large 239 us; 2^18: 241, 232; one row of 2^28: 364, 222, huge 236)
    //   16-bit  large beyond 2^18 (2^28 in one row: small 395, large 265, huge 279 us)
    //   32-bit  large beyond 2^17, huge beyond 2^19 (2^27 in one row: small 230, large 184, huge 174 us)
    // Big tiles need enough tiles to fill the chip, but a long chain of small tiles costs more than idle compute
    // units: the large tile pays from 256 tiles in all, or from 128 of them in a row (one f16 row of 2^22: small 9.4,
    // large 8.2 us; four rows of 2^20: 7.0, 8.0), the huge 32-bit tile from 512 (four rows of 2^22: large 28.2, huge
    // 23.0 us; one row of 2^23: 13.3, 13.9).
    // For 8- and 16-bit inputs the huge tile only pays when the whole call is one generation of workgroups anyway
    // (no more than 512 large tiles: everything is resident at once, and fewer, larger tiles mean fewer hops of the
    // carry chain: 2^24 f16 in one row 19.1 us against 19.6; from 2^25 on the large tile is ahead, 35.2 against 36.6).
    const size_t esz = in_size(dt);
    const size_t to_large = esz == 2 ? ((size_t)1 << 18) + 1 : ((size_t)1 << 17) + 1;
    if (cols < to_large) return kTileSmall;
    const size_t lt = tile_elems(dt, kTileLarge), ht = tile_elems(dt, kTileHuge);
    const size_t large_per_row = (cols + lt - 1) / lt;
    const size_t large_tiles = rows * large_per_row, huge_tiles = rows * ((cols + ht - 1) / ht);
    if (esz == 4) {
        if (cols > ((size_t)1 << 19) && huge_tiles >= 512) return kTileHuge;
    } else {
        if (cols > ((size_t)1 << (esz == 2 ? 23 : 22)) && large_tiles <= 512 && huge_tiles >= 256) return kTileHuge;
    }
    return large_tiles >= 256 || large_per_row >= 128 ? kTileLarge : kTileSmall;
}

std::atomic<uint64_t> g_calls{0};          // calls that drew a tag so far (64 bits: does not wrap in practice)
std::atomic<int> g_seg_flat{1};            // see tcuscan_set_segmented_form
std::atomic<int> g_chain_policy{0};        // see tcuscan_set_chain_policy
std::atomic<uint32_t> g_spin_limit{kDefaultSpinLimit}, g_mute_tile{kNoTile};     // see tcuscan_test_chain_fault
chain_tags::CleanTable g_clean;            // which workspaces hold no status words of older tag generations

// Short rows: the smallest run length (1, 2, 4 or 8 MFMA tiles per wavefront) that holds a row.
// The four (exclusive, reverse) instantiations of one kernel shape.
template <int DT, int NT, bool LEAD> const void *rows_kernel_for(bool excl, bool rev)
{
    if (rev) return excl ? (const void *)scan_rows_kernel<DT, NT, true, true, LEAD> : (const void *)scan_rows_kernel<DT, NT, false, true, LEAD>;
    return excl ? (const void *)scan_rows_kernel<DT, NT, true, false, LEAD> : (const void *)scan_rows_kernel<DT, NT, false, false, LEAD>;
}
template <int DT, int NT, int W> const void *scan_kernel_for(bool excl, bool rev)
{
    if (rev) return excl ? (const void *)scan_kernel<DT, NT, true, true, W> : (const void *)scan_kernel<DT, NT, false, true, W>;
    return excl ? (const void *)scan_kernel<DT, NT, true, false, W> : (const void *)scan_kernel<DT, NT, false, false, W>;
}

template <int DT, int NT> hipError_t launch_rows_nt(Params P, bool excl, bool lead, hipStream_t s)
{
    void *args[] = {&P};
    const void *fn = lead ? rows_kernel_for<DT, NT, true>(excl, P.reverse != 0) : rows_kernel_for<DT, NT, false>(excl, P.reverse != 0);
    return hipLaunchKernel(fn, dim3((unsigned)((P.rows + kWaves - 1) / kWaves)), dim3(kThreads), args, 0, s);
}

template <int DT> hipError_t launch_rows(Params P, bool excl, hipStream_t s)
{
    // rows that start at 16-byte boundaries take the plain form; the others are tiled from the boundary below their
    // start, which can cost one more MFMA tile
    const bool lead = ((uintptr_t)P.in & 15) != 0 || (P.cols * Tr<DT>::kEsz) % 16 != 0;
    const size_t tiles = (P.cols + (lead ? Tr<DT>::kG - 1 : 0) + Geo<DT>::kTileElems - 1) / Geo<DT>::kTileElems;
    if (tiles <= 1) return launch_rows_nt<DT, 1>(P, excl, lead, s);
    if (tiles <= 2) return launch_rows_nt<DT, 2>(P, excl, lead, s);
    if (tiles <= 4) return launch_rows_nt<DT, 4>(P, excl, lead, s);
    if (tiles <= 8) return launch_rows_nt<DT, 8>(P, excl, lead, s);
    return launch_rows_nt<DT, 12>(P, excl, lead, s);
}

template <int DT> hipError_t launch_dt(Params P, bool excl, int size, hipStream_t s)
{
    // 32-bit rows a little longer than 2048 still do better one per wavefront (12 MFMA tiles, partly masked) than in a
    // workgroup tile of 8192 that is a quarter full: measured 2100 / 2304 / 2560 columns 70 / 76 / 76 % of peak against
    // 50 / 61 / 69 %, equal at 2816, and the workgroup tile ahead from there (3000: 73.5 % against 70 %); 8-bit rows of
    // 2304 / 2560 elements likewise (237 us for 2^28 elements against 305 / 253; from 2816 on the workgroup tile is
    // ahead, 223 against 239); for 16-bit inputs the workgroup tile is ahead everywhere above 2048.
    const size_t row_max = Tr<DT>::kEsz == 4 ? kShortRowMax32 : Tr<DT>::kEsz == 1 ? kShortRowMax8 : kShortRowMax;
    if (P.rows >= kShortRowMinRows && P.cols <= row_max) return launch_rows<DT>(P, excl, s);
    // hipLaunchKernel reports this launch's own status (hipGetLastError could return a stale,
    // unrelated code left behind by another library's polling calls).
    void *args[] = {&P};
    const void *fn;
    using Ti = Tiles<DT>;
    const bool rev = P.reverse != 0;
    int waves;
    if (size == kTileHuge)       { waves = Ti::wHuge;  fn = scan_kernel_for<DT, Ti::kHuge, Ti::wHuge>(excl, rev); }
    else if (size == kTileLarge) { waves = Ti::wLarge; fn = scan_kernel_for<DT, Ti::kLarge, Ti::wLarge>(excl, rev); }
    else                         { waves = Ti::wSmall; fn = scan_kernel_for<DT, Ti::kSmall, Ti::wSmall>(excl, rev); }
    return hipLaunchKernel(fn, dim3(P.num_tiles), dim3(64 * waves), args, 0, s);
}

hipError_t launch_fill(void *d, size_t bytes, hipStream_t s, void *d2 = nullptr, size_t bytes2 = 0)
{
    size_t words = bytes / 4, words2 = d2 ? bytes2 / 4 : 0;
    uint32_t *p = (uint32_t *)d, *p2 = (uint32_t *)d2;
    unsigned blocks1 = (unsigned)((words / 4 + 1 + 255) / 256);
    const unsigned blocks2 = words2 ? (unsigned)((words2 / 4 + 1 + 255) / 256) : 0u;
    void *args[] = {&p, &words, &p2, &words2, &blocks1};
    return hipLaunchKernel((const void *)fill_zero_kernel, dim3(blocks1 + blocks2), dim3(256), args, 0, s);
}

// What a launch has to know about the carry chain, and whatever has to run in front of it on the stream.  `tiles`
// status words behind the header of `d_ws` are going to be used (0: no chain).
//   * A call normally draws a fresh tag from the call counter; the first call on a workspace in a new tag generation
//     clears the status words first (chain_tags.h).
//   * A call recorded by stream capture is replayed with the tag it was recorded with, and `clear_first` marks a
//     workspace region whose contents the library cannot vouch for: both get the reserved tag and a fill kernel in
//     front of every run (a kernel, not a memset node).
//   * Ticket policy: the header's ticket counter is cleared.
// `also` / `also_bytes`: another region of the workspace that a clear-first call wants zeroed (same launch).
tcuscan_status_t begin_chain(Params &P, void *d_ws, size_t tiles, bool clear_first, hipStream_t s, void *also = nullptr,
                             size_t also_bytes = 0, bool cleared_by_caller = false)
{
    P.ticket = 0u;
    P.spin_limit = g_spin_limit.load(std::memory_order_relaxed);
    P.mute_tile = g_mute_tile.load(std::memory_order_relaxed);
    P.tag = 1u;
    if (!d_ws || tiles == 0) return TCUSCAN_OK;
    const size_t status_bytes = 8 * kStatusStride * tiles;
    void *status = (char *)d_ws + sizeof(WsHeader);
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cs) != hipSuccess) { (void)hipGetLastError(); cs = hipStreamCaptureStatusNone; }
    if (clear_first || cs == hipStreamCaptureStatusActive) {
        P.tag = chain_tags::kClearFirstTag;
        if (!cleared_by_caller && launch_fill(status, status_bytes, s, also, also_bytes) != hipSuccess) return TCUSCAN_ERR_HIP;
    } else {
        if (also && launch_fill(also, also_bytes, s) != hipSuccess) return TCUSCAN_ERR_HIP;
        const chain_tags::CallId id = chain_tags::call_id(g_calls.fetch_add(1u, std::memory_order_relaxed));
        P.tag = id.tag;
        if (g_clean.needs_clear((uintptr_t)d_ws, sizeof(WsHeader) + status_bytes, id.generation) &&
            launch_fill(status, status_bytes, s) != hipSuccess) return TCUSCAN_ERR_HIP;
    }
    if (g_chain_policy.load(std::memory_order_relaxed) == 1) {
        P.ticket = 1u;
        if (launch_fill(&((WsHeader *)d_ws)->ticket, sizeof(uint32_t), s) != hipSuccess) return TCUSCAN_ERR_HIP;
    }
    return TCUSCAN_OK;
}

// Which way a row-wise call takes (tcuscan_path_for reports it; run() follows it).
struct Plan {
    int path;            // TCUSCAN_PATH_*
    int seg_cls;         // tiles from the boundary below: which tile (kSegSmall / kSegLarge)
    size_t tpr, need;    // ... tiles per row (the row and the elements in front of it) and workspace bytes they take
};
Plan plan_for(uintptr_t in_addr, size_t rows, size_t cols, int dt, bool ws_usable, size_t ws_bytes);     // below, with the segmented launches
tcuscan_status_t run_unaligned_rows(const void *d_in, void *d_out, size_t rows, size_t cols, int dt, int exclusive, int reverse, void *d_ws,
                                    const Plan &plan, bool clear_first, hipStream_t s);

// `clear_first`: the workspace is a region whose former contents are unknown (see begin_chain).
tcuscan_status_t run(const void *d_in, void *d_out, size_t rows, size_t cols, int dt, int exclusive, int reverse,
                     void *d_ws, size_t ws_bytes, tcuscan_stream_t stream, bool clear_first = false)
{
    if (!valid_dtype(dt)) return TCUSCAN_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return TCUSCAN_OK;
    if (!d_in || !d_out) return TCUSCAN_ERR_INVALID_ARG;
    if (((uintptr_t)d_in % in_size(dt)) != 0 || ((uintptr_t)d_out % 4) != 0) return TCUSCAN_ERR_INVALID_ARG;
    if (d_in == d_out && in_size(dt) != 4) return TCUSCAN_ERR_INVALID_ARG;
    if (rows > 0x7FFFFFFFull / ((cols + kSmallTile - 1) / kSmallTile)) return TCUSCAN_ERR_UNSUPPORTED;   // tile index: 31 bits
    // the least a call needs: one status word per small tile of the rows themselves (tcuscan_workspace_bytes promises
    // one more per row where a row and the elements in front of it can need one; see plan_for)
    const size_t tpr_small = (cols + kSmallTile - 1) / kSmallTile;
    const size_t need = tpr_small > 1 ? sizeof(WsHeader) + 8 * kStatusStride * rows * tpr_small : 0;
    const bool ws_usable = d_ws && ((uintptr_t)d_ws % 8) == 0;
    if (need && (!ws_usable || ws_bytes < need)) return TCUSCAN_ERR_WORKSPACE;

    hipStream_t s = (hipStream_t)stream;
    const Plan plan = plan_for((uintptr_t)d_in, rows, cols, dt, ws_usable, ws_bytes);
    // long rows that do not start at 16-byte boundaries: tiled from the boundary below, like segmented rows
    if (plan.path == TCUSCAN_PATH_TILES_FROM_BOUNDARY)
        return run_unaligned_rows(d_in, d_out, rows, cols, dt, exclusive, reverse, d_ws, plan, clear_first, s);
    const int size = choose_tile(dt, rows, cols);
    const size_t tile = tile_elems(dt, size);
    const size_t tpr = (cols + tile - 1) / tile;
    Params P;
    P.in = d_in; P.out = d_out; P.rows = rows; P.cols = cols;
    P.tiles_per_row = (uint32_t)tpr; P.num_tiles = (uint32_t)(rows * tpr);
    P.ws = need ? (WsHeader *)d_ws : nullptr;
    P.reverse = reverse ? 1u : 0u;
    P.tile_desc = nullptr;
    // Every call gets a fresh tag, so status words of earlier calls are stale by construction.
    const tcuscan_status_t bst = begin_chain(P, P.ws && tpr > 1 ? d_ws : nullptr, rows * tpr, clear_first, s);
    if (bst != TCUSCAN_OK) return bst;
    hipError_t e;
    switch (dt) {
    case TCUSCAN_I32_I32:  e = launch_dt<TCUSCAN_I32_I32>(P, exclusive != 0, size, s); break;
    case TCUSCAN_F16_F32:  e = launch_dt<TCUSCAN_F16_F32>(P, exclusive != 0, size, s); break;
    case TCUSCAN_I8_I32:   e = launch_dt<TCUSCAN_I8_I32>(P, exclusive != 0, size, s); break;
    case TCUSCAN_F32_F32:  e = launch_dt<TCUSCAN_F32_F32>(P, exclusive != 0, size, s); break;
    default:               e = launch_dt<TCUSCAN_BF16_F32>(P, exclusive != 0, size, s); break;
    }
    return e == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

// ---- segmented scans (rows of different lengths, stored back to back)


// The tile a segmented scan uses is decided by the average row length (the only thing the host knows): one
// wavefront per tile for short rows, the small workgroup tile, or the large one for very long rows.
enum SegTile { kSegShort = 0, kSegSmall = 1, kSegLarge = 2 };

int seg_tile_class(int dt, size_t rows, size_t total)
{
    const size_t short_tile = (size_t)kSegShortNT * 64 * (16 / in_size(dt));
    const size_t avg = rows ? total / rows : total;
    return avg < 4 * short_tile ? kSegShort : avg < ((size_t)1 << 19) ? kSegSmall : kSegLarge;
}

size_t seg_tile_elems(int dt, int cls)
{
    return cls == kSegShort ? (size_t)kSegShortNT * 64 * (16 / in_size(dt)) : cls == kSegSmall ? kSmallTile : tile_elems(dt, kTileLarge);
}

struct SegLayout {
    size_t max_tiles;        // upper bound on the number of tiles = grid size
    size_t counts_off, starts_off, rowmap_off, inner_off, inner_bytes, total_bytes;
    size_t heads_off, heads_words;   // row-start bits (short 32-bit rows only, else 0 words): never where status words may lie
};

bool seg_layout(int dt, size_t rows, size_t total, SegLayout &L)
{
    const size_t tile = seg_tile_elems(dt, seg_tile_class(dt, rows, total));
    L.max_tiles = total / tile + 2 * rows + 1;           // a row of len elements has at most len / tile + 2 tiles
    if (L.max_tiles > 0x7FFFFFFFull || rows + 1 > 0x7FFFFFFFull) return false;
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    L.counts_off = up(sizeof(WsHeader) + 8 * kStatusStride * L.max_tiles);
    L.starts_off = up(L.counts_off + 4 * (rows + 1));
    L.rowmap_off = up(L.starts_off + 4 * (rows + 1));
    L.inner_off = up(L.rowmap_off + sizeof(TileDesc) * L.max_tiles);
    L.inner_bytes = tcuscan_workspace_bytes(1, rows + 1, TCUSCAN_I32_I32);
    L.heads_off = up(L.inner_off + L.inner_bytes);
    L.heads_words = seg_tile_class(dt, rows, total) == kSegShort ? (total + 32) / 32 + 2 : 0;
    L.total_bytes = L.heads_off + 4 * L.heads_words;
    return true;
}

template <int DT, int NT, int W> const void *seg_kernel_for(bool excl, bool rev)
{
    if (rev) return excl ? (const void *)scan_kernel<DT, NT, true, true, W, true> : (const void *)scan_kernel<DT, NT, false, true, W, true>;
    return excl ? (const void *)scan_kernel<DT, NT, true, false, W, true> : (const void *)scan_kernel<DT, NT, false, false, W, true>;
}
template <int DT> const void *seg_short_kernel_for(bool excl, bool rev)
{
    if (rev) return excl ? (const void *)seg_short_kernel<DT, true, true> : (const void *)seg_short_kernel<DT, false, true>;
    return excl ? (const void *)seg_short_kernel<DT, true, false> : (const void *)seg_short_kernel<DT, false, false>;
}

template <int DT> hipError_t launch_seg(Params P, bool excl, int cls, hipStream_t s)
{
    void *args[] = {&P};
    using Ti = Tiles<DT>;
    const bool rev = P.reverse != 0;
    if (cls == kSegLarge) return hipLaunchKernel(seg_kernel_for<DT, Ti::kLarge, Ti::wLarge>(excl, rev), dim3(P.num_tiles), dim3(64 * Ti::wLarge), args, 0, s);
    if (cls == kSegSmall) return hipLaunchKernel(seg_kernel_for<DT, Ti::kSmall, Ti::wSmall>(excl, rev), dim3(P.num_tiles), dim3(64 * Ti::wSmall), args, 0, s);
    constexpr unsigned per_wg = kSegPack * kSegUnroll;
    return hipLaunchKernel(seg_short_kernel_for<DT>(excl, rev), dim3((P.num_tiles + per_wg - 1) / per_wg), dim3(64 * kSegPack), args, 0, s);
}

// Short rows of 32-bit elements: the covered range as one row with row-start bits (seg_flat_kernel).  Three
// launches: clear the bits, set them from the offsets, scan.  Measured on 2^26 fp32 elements cut at random into rows of
// mean length 20 / 200 / 1500 / 5000 / 20000: 172 / 107 / 108 / 110 / 114 us against 1436 / 213 / 137 / 102 / 97 us with
// tiles of their own for every row -- hence for the short class only (average below 2048 elements).  The status words are the first ones of the general
// layout; the bits have a region of their own behind everything else (a word of bits where another call expects a
// status word could pass for one).
constexpr int kFlatNT = 8, kFlatW = 8;
template <int DT> const void *seg_flat_kernel_for(bool excl, bool rev)
{
    if (rev) return excl ? (const void *)seg_flat_kernel<DT, kFlatNT, true, true, kFlatW> : (const void *)seg_flat_kernel<DT, kFlatNT, false, true, kFlatW>;
    return excl ? (const void *)seg_flat_kernel<DT, kFlatNT, true, false, kFlatW> : (const void *)seg_flat_kernel<DT, kFlatNT, false, false, kFlatW>;
}
template <int DT> const void *seg_flat_narrow_kernel_for(bool excl, bool rev)
{
    if (rev) return excl ? (const void *)seg_flat_narrow_kernel<DT, true, true, kFlatW> : (const void *)seg_flat_narrow_kernel<DT, false, true, kFlatW>;
    return excl ? (const void *)seg_flat_narrow_kernel<DT, true, false, kFlatW> : (const void *)seg_flat_narrow_kernel<DT, false, false, kFlatW>;
}
tcuscan_status_t run_segmented_flat(const void *d_in, void *d_out, const long long *d_offsets, size_t rows, size_t total, int dt,
                                    int exclusive, int reverse, void *d_ws, const SegLayout &L, hipStream_t s)
{
    const size_t tile = (size_t)kFlatNT * kFlatW * 256;
    const size_t tiles = total / tile + 2;                       // the range is at most `total` long and starts less than a granule late
    if (tiles > L.max_tiles) return TCUSCAN_ERR_UNSUPPORTED;     // (never: the general layout counts smaller tiles)
    uint32_t *heads = (uint32_t *)((char *)d_ws + L.heads_off);
    const uint32_t shift = (uint32_t)(((uintptr_t)d_in / in_size(dt)) & (16 / in_size(dt) - 1));    // granules start at bit multiples of their length
    Params P;
    P.in = d_in; P.out = d_out; P.rows = rows; P.cols = total;
    P.tiles_per_row = 0; P.num_tiles = (uint32_t)tiles;
    P.ws = (WsHeader *)d_ws;
    P.reverse = reverse ? 1u : 0u; P.tile_desc = nullptr;
    // one fill launch clears the status words and the row-start bits
    const tcuscan_status_t bst = begin_chain(P, d_ws, tiles, true, s, heads, 4 * L.heads_words);
    if (bst != TCUSCAN_OK) return bst;
    {
        const long long *off = d_offsets; size_t r = rows, t = total; uint32_t sh = shift; WsHeader *h = (WsHeader *)d_ws;
        void *args[] = {&off, &r, &t, &sh, &heads, &h};
        if (hipLaunchKernel((const void *)seg_heads_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), args, 0, s) != hipSuccess)
            return TCUSCAN_ERR_HIP;
    }
    const long long *off = d_offsets; const uint32_t *hd = heads; uint32_t sh = shift;
    void *args[] = {&P, &off, &hd, &sh};
    const bool ex = exclusive != 0;
    const void *fn;
    switch (dt) {
    case TCUSCAN_F32_F32:  fn = seg_flat_kernel_for<TCUSCAN_F32_F32>(ex, reverse != 0); break;
    case TCUSCAN_I32_I32:  fn = seg_flat_kernel_for<TCUSCAN_I32_I32>(ex, reverse != 0); break;
    case TCUSCAN_I8_I32:   fn = seg_flat_narrow_kernel_for<TCUSCAN_I8_I32>(ex, reverse != 0); break;
    case TCUSCAN_F16_F32:  fn = seg_flat_narrow_kernel_for<TCUSCAN_F16_F32>(ex, reverse != 0); break;
    default:               fn = seg_flat_narrow_kernel_for<TCUSCAN_BF16_F32>(ex, reverse != 0); break;
    }
    return hipLaunchKernel(fn, dim3(P.num_tiles), dim3(64 * kFlatW), args, 0, s) == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

// Equal rows of a batched call that do not start at 16-byte boundaries (odd row length, unaligned array) and are too
// long for one wavefront each: the segmented kernel without descriptors (it derives the row from the tile index), so
// that every full granule takes the 128-bit path (element by element such rows run at 22 .. 40 % of peak instead of
// 74 .. 79 %).  A row and the few elements in front of it can need one tile more than the row alone; when the
// caller's workspace has no status word for that tile (it was sized by an older rule than tcuscan_workspace_bytes'), the
// other tile size is tried, and failing that the call is left to the element-wise path.
Plan plan_for(uintptr_t in_addr, size_t rows, size_t cols, int dt, bool ws_usable, size_t ws_bytes)
{
    Plan plan = {TCUSCAN_PATH_TILES, kSegSmall, 0, 0};
    const size_t row_max = in_size(dt) == 4 ? kShortRowMax32 : in_size(dt) == 1 ? kShortRowMax8 : kShortRowMax;
    if (rows >= kShortRowMinRows && cols <= row_max) { plan.path = TCUSCAN_PATH_ROWS; return plan; }
    if ((in_addr & 15) == 0 && (rows <= 1 || (cols * in_size(dt)) % 16 == 0)) return plan;       // every row starts at a 16-byte boundary
    // the tile the row-length rule picks, or the other one if the workspace only has the status words for that
    int cls = cols < ((size_t)1 << 19) ? kSegSmall : kSegLarge;
    for (int attempt = 0; attempt < 2; ++attempt, cls = cls == kSegSmall ? kSegLarge : kSegSmall) {
        const size_t tile = seg_tile_elems(dt, cls), granule = 16 / in_size(dt);
        const size_t tpr = (cols + granule - 1 + tile - 1) / tile;
        const size_t need = tpr > 1 ? sizeof(WsHeader) + 8 * kStatusStride * rows * tpr : 0;
        if (rows * tpr <= 0x7FFFFFFFull && rows <= 0x7FFFFFFFull && (!need || (ws_usable && ws_bytes >= need))) {
            plan.path = TCUSCAN_PATH_TILES_FROM_BOUNDARY; plan.seg_cls = cls; plan.tpr = tpr; plan.need = need;
            return plan;
        }
    }
    plan.path = TCUSCAN_PATH_ELEMENTWISE;       // a workspace sized by an older rule: one status word per row short
    return plan;
}

tcuscan_status_t run_unaligned_rows(const void *d_in, void *d_out, size_t rows, size_t cols, int dt, int exclusive, int reverse, void *d_ws,
                                    const Plan &plan, bool clear_first, hipStream_t s)
{
    const int cls = plan.seg_cls;
    const size_t tpr = plan.tpr, need = plan.need;
    Params P;
    P.in = d_in; P.out = d_out; P.rows = rows; P.cols = rows * cols;     // cols: the length of the arrays, as for segmented calls
    P.tiles_per_row = (uint32_t)tpr; P.num_tiles = (uint32_t)(rows * tpr);
    P.ws = need ? (WsHeader *)d_ws : nullptr;
    P.reverse = reverse ? 1u : 0u;
    P.tile_desc = nullptr;
    const tcuscan_status_t bst = begin_chain(P, need ? d_ws : nullptr, rows * tpr, clear_first, s);
    if (bst != TCUSCAN_OK) return bst;
    hipError_t e;
    switch (dt) {
    case TCUSCAN_I32_I32:  e = launch_seg<TCUSCAN_I32_I32>(P, exclusive != 0, cls, s); break;
    case TCUSCAN_F16_F32:  e = launch_seg<TCUSCAN_F16_F32>(P, exclusive != 0, cls, s); break;
    case TCUSCAN_I8_I32:   e = launch_seg<TCUSCAN_I8_I32>(P, exclusive != 0, cls, s); break;
    case TCUSCAN_F32_F32:  e = launch_seg<TCUSCAN_F32_F32>(P, exclusive != 0, cls, s); break;
    default:               e = launch_seg<TCUSCAN_BF16_F32>(P, exclusive != 0, cls, s); break;
    }
    return e == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

tcuscan_status_t run_segmented(const void *d_in, void *d_out, const long long *d_offsets, size_t rows, size_t total, int dt,
                               int exclusive, int reverse, void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    if (!valid_dtype(dt)) return TCUSCAN_ERR_UNSUPPORTED;
    if (rows == 0 || total == 0) return TCUSCAN_OK;
    if (!d_in || !d_out || !d_offsets) return TCUSCAN_ERR_INVALID_ARG;
    if (((uintptr_t)d_in % in_size(dt)) != 0 || ((uintptr_t)d_out % 4) != 0 || ((uintptr_t)d_offsets % 8) != 0) return TCUSCAN_ERR_INVALID_ARG;
    if (d_in == d_out && in_size(dt) != 4) return TCUSCAN_ERR_INVALID_ARG;
    SegLayout L;
    if (!seg_layout(dt, rows, total, L)) return TCUSCAN_ERR_UNSUPPORTED;
    if (!d_ws || ws_bytes < L.total_bytes || ((uintptr_t)d_ws % 8) != 0) return TCUSCAN_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int cls = seg_tile_class(dt, rows, total);
    // This call puts row maps where a later call of another shape may expect status words: the workspace is no
    // longer known to be clean (segmented calls themselves clear their status words in front of every run).
    g_clean.mark_dirty((uintptr_t)d_ws, chain_tags::call_id(g_calls.load(std::memory_order_relaxed)).generation);
    if (L.heads_words && g_seg_flat.load(std::memory_order_relaxed))
        return run_segmented_flat(d_in, d_out, d_offsets, rows, total, dt, exclusive, reverse, d_ws, L, s);
    const size_t tile = seg_tile_elems(dt, cls);
    int32_t *counts = (int32_t *)((char *)d_ws + L.counts_off);
    uint32_t *starts = (uint32_t *)((char *)d_ws + L.starts_off);
    TileDesc *desc = (TileDesc *)((char *)d_ws + L.rowmap_off);
    const bool few_rows = rows < kSegPrepRows;
    if (few_rows) {   // steps 1 - 3 and the clearing of the status words in one launch
        const long long *off = d_offsets; size_t r = rows, t = total; uintptr_t in_addr = (uintptr_t)d_in;
        uint32_t esz = (uint32_t)in_size(dt), tl = (uint32_t)tile, mt = (uint32_t)L.max_tiles; WsHeader *h = (WsHeader *)d_ws;
        void *args[] = {&off, &r, &t, &in_addr, &esz, &tl, &desc, &mt, &h};
        if (hipLaunchKernel((const void *)seg_prepare_kernel, dim3((unsigned)((L.max_tiles + 1023) / 1024)), dim3(1024), args, 0, s) != hipSuccess)
            return TCUSCAN_ERR_HIP;
    } else {
        {   // step 1: tiles per row
            const long long *off = d_offsets; size_t r = rows, t = total; uintptr_t in_addr = (uintptr_t)d_in;
            uint32_t esz = (uint32_t)in_size(dt), tl = (uint32_t)tile; WsHeader *h = (WsHeader *)d_ws;
            void *args[] = {&off, &r, &t, &in_addr, &esz, &tl, &counts, &h};
            if (hipLaunchKernel((const void *)seg_tiles_kernel, dim3((unsigned)((rows + 1 + 255) / 256)), dim3(256), args, 0, s) != hipSuccess)
                return TCUSCAN_ERR_HIP;
        }
        // step 2: first tile of every row = exclusive scan of the counts (this library's own int32 scan)
        // (its workspace is a region of this one whose former contents depend on the shapes of earlier calls: cleared first)
        tcuscan_status_t st = run(counts, starts, 1, rows + 1, TCUSCAN_I32_I32, 1, 0, L.inner_bytes ? (char *)d_ws + L.inner_off : nullptr,
                                  L.inner_bytes, stream, true);
        if (st != TCUSCAN_OK) return st;
        {   // step 3: one descriptor per tile
            const uint32_t *ts = starts; const long long *off = d_offsets; size_t r = rows; uint32_t mt = (uint32_t)L.max_tiles;
            void *args[] = {&ts, &off, &r, &desc, &mt};
            if (hipLaunchKernel((const void *)seg_desc_kernel, dim3((unsigned)((L.max_tiles + 255) / 256)), dim3(256), args, 0, s) != hipSuccess)
                return TCUSCAN_ERR_HIP;
        }
    }
    // step 4: the scan itself; the grid is the upper bound on the number of tiles, surplus workgroups leave at once
    Params P;
    P.in = d_in; P.out = d_out; P.rows = rows; P.cols = total;          // cols: the length of the arrays (no access beyond it)
    P.tiles_per_row = 0; P.num_tiles = (uint32_t)L.max_tiles;
    P.ws = (WsHeader *)d_ws;
    P.reverse = reverse ? 1u : 0u;
    P.tile_desc = desc;
    const tcuscan_status_t bst = begin_chain(P, d_ws, L.max_tiles, true, s, nullptr, 0, few_rows);
    if (bst != TCUSCAN_OK) return bst;
    hipError_t e;
    switch (dt) {
    case TCUSCAN_I32_I32:  e = launch_seg<TCUSCAN_I32_I32>(P, exclusive != 0, cls, s); break;
    case TCUSCAN_F16_F32:  e = launch_seg<TCUSCAN_F16_F32>(P, exclusive != 0, cls, s); break;
    case TCUSCAN_I8_I32:   e = launch_seg<TCUSCAN_I8_I32>(P, exclusive != 0, cls, s); break;
    case TCUSCAN_F32_F32:  e = launch_seg<TCUSCAN_F32_F32>(P, exclusive != 0, cls, s); break;
    default:               e = launch_seg<TCUSCAN_BF16_F32>(P, exclusive != 0, cls, s); break;
    }
    return e == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

// ---- fused split and fused stream compaction: one row of n elements in tiles of `tile`, chained through d_ws

tcuscan_status_t flag_kernel_params(Params &P, size_t n, size_t tile, void *d_ws, size_t ws_bytes, hipStream_t s)
{
    const size_t tiles = (n + tile - 1) / tile;
    if (tiles > 0x7FFFFFFFull) return TCUSCAN_ERR_UNSUPPORTED;
    const size_t need = tiles > 1 ? sizeof(WsHeader) + 8 * kStatusStride * tiles : 0;
    if (need && (!d_ws || ws_bytes < need || ((uintptr_t)d_ws % 8) != 0)) return TCUSCAN_ERR_WORKSPACE;
    P.in = nullptr; P.out = nullptr; P.rows = 1; P.cols = n;
    P.tiles_per_row = (uint32_t)tiles; P.num_tiles = (uint32_t)tiles;
    P.ws = need ? (WsHeader *)d_ws : nullptr;
    P.reverse = 0; P.tile_desc = nullptr;
    return begin_chain(P, need ? d_ws : nullptr, tiles, false, s);
}

// 2048 elements per wavefront (their words stay in registers from the load to the scatter), 8 wavefronts: 16384 per
// workgroup, 64.5 KiB of LDS, two workgroups per compute unit.  (1024 per wavefront, four workgroups and twice the
// wavefronts per compute unit: compaction 407 us against 367, sort 3.76 ms against 3.11 -- more tiles, no better overlap.)
constexpr int kFlagNT = 2, kFlagW = 8;

}  // namespace

// Used by tcuscan_split_radix_sort_u32 (apps.hip): the zero counts of all 32 bits, and one fused split pass.
extern "C" __attribute__((visibility("hidden")))
tcuscan_status_t tcuscan_internal_bit_zero_counts(const void *d_keys, size_t n, unsigned *d_counts32, tcuscan_stream_t stream)
{
    hipStream_t s = (hipStream_t)stream;
    if (launch_fill(d_counts32, 32 * sizeof(unsigned), s) != hipSuccess) return TCUSCAN_ERR_HIP;
    const uint32_t *k = (const uint32_t *)d_keys; uint32_t *c = d_counts32;
    void *args[] = {&k, &n, &c};
    const unsigned grid = (unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048);
    return hipLaunchKernel((const void *)bit_zero_counts_kernel, dim3(grid), dim3(256), args, 0, s) == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

extern "C" __attribute__((visibility("hidden")))
tcuscan_status_t tcuscan_internal_split_pass(const void *d_keys, const void *d_vals, void *d_keys_out, void *d_vals_out, size_t n, int bit,
                                             const unsigned *d_zeros_total, void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    constexpr int NT = kFlagNT, W = kFlagW;
    hipStream_t s = (hipStream_t)stream;
    Params P;
    const tcuscan_status_t st = flag_kernel_params(P, n, (size_t)NT * W * 1024, d_ws, ws_bytes, s);
    if (st != TCUSCAN_OK) return st;
    SplitArgs S;
    S.keys = (const uint32_t *)d_keys; S.vals = (const uint32_t *)d_vals;
    S.keys_out = (uint32_t *)d_keys_out; S.vals_out = (uint32_t *)d_vals_out;
    S.zeros_total = d_zeros_total; S.bit = bit;
    void *args[] = {&P, &S};
    const void *fn = d_vals ? (const void *)split_kernel<NT, W, true> : (const void *)split_kernel<NT, W, false>;
    return hipLaunchKernel(fn, dim3(P.num_tiles), dim3(64 * W), args, 0, s) == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

extern "C" __attribute__((visibility("hidden")))
tcuscan_status_t tcuscan_internal_digit_counts(const void *d_keys, size_t n, unsigned *d_counts64, tcuscan_stream_t stream)
{
    hipStream_t s = (hipStream_t)stream;
    if (launch_fill(d_counts64, 64 * sizeof(unsigned), s) != hipSuccess) return TCUSCAN_ERR_HIP;
    const uint32_t *k = (const uint32_t *)d_keys; uint32_t *c = d_counts64;
    void *args[] = {&k, &n, &c};
    // 512 workgroups: every workgroup ends with 48 atomic adds on the same 48 counters, and with 2048 of them those were
    // a third of the run time (2^26 keys: 84 us against 70)
    const unsigned grid = (unsigned)((n + 255) / 256 < 512 ? (n + 255) / 256 : 512);
    if (hipLaunchKernel((const void *)digit_counts_kernel, dim3(grid), dim3(256), args, 0, s) != hipSuccess) return TCUSCAN_ERR_HIP;
    void *args2[] = {&c, &n};
    return hipLaunchKernel((const void *)digit_zero_counts_kernel, dim3(1), dim3(64), args2, 0, s) == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

extern "C" __attribute__((visibility("hidden")))
tcuscan_status_t tcuscan_internal_split4_pass(const void *d_keys, const void *d_vals, void *d_keys_out, void *d_vals_out, size_t n, int bit,
                                              const unsigned *d_hist4, void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    // Keys alone: 8 wavefronts per workgroup, and the register allocator is held to 128 registers so that two workgroups
    // (64.5 KiB of LDS each) share a compute unit (a dozen spilled registers; without the limit one workgroup: 208 us
    // per pass of 2^26 keys against 177).  With payloads, which cost 32 registers more, 4 wavefronts per workgroup.
    constexpr int NT = kFlagNT;
    const int W = d_vals ? 4 : kFlagW;
    hipStream_t s = (hipStream_t)stream;
    Params P;
    const tcuscan_status_t st = flag_kernel_params(P, n, (size_t)NT * W * 1024, d_ws, ws_bytes, s);
    if (st != TCUSCAN_OK) return st;
    Split4Args S;
    S.keys = (const uint32_t *)d_keys; S.vals = (const uint32_t *)d_vals;
    S.keys_out = (uint32_t *)d_keys_out; S.vals_out = (uint32_t *)d_vals_out;
    S.hist = d_hist4; S.bit = bit;
    void *args[] = {&P, &S};
    const void *fn = d_vals ? (const void *)split4_kernel<NT, 4, true> : (const void *)split4_kernel<NT, kFlagW, false>;
    return hipLaunchKernel(fn, dim3(P.num_tiles), dim3(64 * W), args, 0, s) == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

// Used by tcuscan_compact_u32 (apps.hip) when the caller does not ask for the positions: one pass over the mask
// and the values, nothing else written than the kept values.  Not part of the public interface.
extern "C" __attribute__((visibility("hidden")))
tcuscan_status_t tcuscan_internal_compact_fused(const void *d_values, const void *d_mask, void *d_out, size_t n, unsigned *d_count,
                                                void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    constexpr int NT = kFlagNT, W = kFlagW;
    hipStream_t s = (hipStream_t)stream;
    Params P;
    const tcuscan_status_t st = flag_kernel_params(P, n, (size_t)NT * W * 1024, d_ws, ws_bytes, s);
    if (st != TCUSCAN_OK) return st;
    CompactArgs C;
    C.mask = (const uint8_t *)d_mask; C.values = (const uint32_t *)d_values; C.out = (uint32_t *)d_out; C.count = d_count;
    void *args[] = {&P, &C};
    return hipLaunchKernel((const void *)compact_kernel<NT, W>, dim3(P.num_tiles), dim3(64 * W), args, 0, s) == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

// ---- the entry point that allocates nothing: its carry-chain workspace is a fixed device array of the library
//
// One copy of the array exists on every GPU the library's code object is loaded on, each at its own address; in host
// code the array's NAME is only a handle for hipGetSymbolAddress (passing it to a kernel would hand the kernel a host
// address).  The device address is looked up once per device, with that device current, and kept.
static __device__ __align__(256) unsigned char g_static_scratch[TCUSCAN_STATIC_SCRATCH_BYTES];
static_assert(TCUSCAN_STATIC_SCRATCH_BYTES % 256 == 0 && TCUSCAN_STATIC_SCRATCH_BYTES > sizeof(WsHeader), "scratch size");

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void *g_static_ptr[kMaxDevices] = {};          // device address of g_static_scratch on device i (null: not looked up yet)

tcuscan_status_t static_scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TCUSCAN_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return TCUSCAN_ERR_HIP; }
        g_static_ptr[dev] = p;
    }
    *out = g_static_ptr[dev];
    return TCUSCAN_OK;
}

}  // namespace

extern "C" {

size_t tcuscan_tile_elems(tcuscan_dtype_t dt) { return valid_dtype((int)dt) ? kSmallTile : 0; }

size_t tcuscan_large_tile_elems(tcuscan_dtype_t dt) { return valid_dtype((int)dt) ? tile_elems((int)dt, kTileLarge) : 0; }

size_t tcuscan_huge_tile_elems(tcuscan_dtype_t dt) { return valid_dtype((int)dt) ? tile_elems((int)dt, kTileHuge) : 0; }

tcuscan_status_t tcuscan_set_segmented_form(int flat)
{
    g_seg_flat.store(flat != 0 ? 1 : 0, std::memory_order_relaxed);
    return TCUSCAN_OK;
}

tcuscan_status_t tcuscan_set_tile_policy(int policy)
{
    if (policy < 0 || policy > 3) return TCUSCAN_ERR_INVALID_ARG;
    g_tile_policy.store(policy, std::memory_order_relaxed);
    return TCUSCAN_OK;
}

size_t tcuscan_workspace_bytes(size_t rows, size_t cols, tcuscan_dtype_t dt)
{
    if (!valid_dtype((int)dt) || rows == 0 || cols == 0) return 0;
    // One status word per small tile of a row -- counted for the row AND the elements in front of it up to the
    // 16-byte boundary below (fewer than a granule): rows that do not start at such a boundary are tiled from there,
    // which takes one tile more when the row's length is within a granule of a multiple of the tile.
    // (Rows of up to one small tile never need a workspace: if such a row needs a second small tile, it fits one
    // large tile.)
    if (cols <= kSmallTile) return 0;
    const size_t granule = 16 / in_size((int)dt);
    const size_t tpr = (cols + granule - 1 + kSmallTile - 1) / kSmallTile;
    return sizeof(WsHeader) + 8 * kStatusStride * rows * tpr;
}

tcuscan_status_t tcuscan_workspace_init(void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    if (ws_bytes == 0) return TCUSCAN_OK;
    if (!d_ws || ((uintptr_t)d_ws % 8) != 0 || (ws_bytes % 4) != 0) return TCUSCAN_ERR_INVALID_ARG;
    return launch_fill(d_ws, ws_bytes, (hipStream_t)stream) == hipSuccess ? TCUSCAN_OK : TCUSCAN_ERR_HIP;
}

tcuscan_status_t tcuscan_inclusive(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt,
                                   void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    return run(d_in, d_out, n ? 1 : 0, n, (int)dt, 0, 0, d_ws, ws_bytes, stream);
}

tcuscan_status_t tcuscan_exclusive(const void *d_in, void *d_out, size_t n, tcuscan_dtype_t dt,
                                   void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    return run(d_in, d_out, n ? 1 : 0, n, (int)dt, 1, 0, d_ws, ws_bytes, stream);
}

tcuscan_status_t tcuscan_batched(const void *d_in, void *d_out, size_t rows, size_t cols,
                                 tcuscan_dtype_t dt, int exclusive,
                                 void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    return run(d_in, d_out, rows, cols, (int)dt, exclusive, 0, d_ws, ws_bytes, stream);
}

tcuscan_status_t tcuscan_scan(const void *d_in, void *d_out, size_t rows, size_t cols, tcuscan_dtype_t dt, unsigned flags,
                              void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    if (flags & ~(unsigned)(TCUSCAN_EXCLUSIVE | TCUSCAN_REVERSE)) return TCUSCAN_ERR_INVALID_ARG;
    return run(d_in, d_out, rows, cols, (int)dt, (flags & TCUSCAN_EXCLUSIVE) != 0, (flags & TCUSCAN_REVERSE) != 0, d_ws, ws_bytes, stream);
}

size_t tcuscan_segmented_workspace_bytes(size_t rows, size_t total, tcuscan_dtype_t dt)
{
    SegLayout L;
    if (!valid_dtype((int)dt) || rows == 0 || total == 0 || !seg_layout((int)dt, rows, total, L)) return 0;
    return L.total_bytes;
}

tcuscan_status_t tcuscan_segmented(const void *d_in, void *d_out, const long long *d_offsets, size_t rows, size_t total,
                                   tcuscan_dtype_t dt, unsigned flags, void *d_ws, size_t ws_bytes, tcuscan_stream_t stream)
{
    if (flags & ~(unsigned)(TCUSCAN_EXCLUSIVE | TCUSCAN_REVERSE)) return TCUSCAN_ERR_INVALID_ARG;
    return run_segmented(d_in, d_out, d_offsets, rows, total, (int)dt, (flags & TCUSCAN_EXCLUSIVE) != 0, (flags & TCUSCAN_REVERSE) != 0,
                         d_ws, ws_bytes, stream);
}

int tcuscan_path_for(const void *d_in, size_t rows, size_t cols, tcuscan_dtype_t dt, size_t ws_bytes)
{
    if (!valid_dtype((int)dt) || rows == 0 || cols == 0) return -1;
    return plan_for((uintptr_t)d_in, rows, cols, (int)dt, true, ws_bytes).path;
}

tcuscan_status_t tcuscan_set_chain_policy(int policy)
{
    if (policy < 0 || policy > 1) return TCUSCAN_ERR_INVALID_ARG;
    g_chain_policy.store(policy, std::memory_order_relaxed);
    return TCUSCAN_OK;
}

tcuscan_status_t tcuscan_test_advance_calls(unsigned long long calls)
{
    g_calls.fetch_add(calls, std::memory_order_relaxed);
    return TCUSCAN_OK;
}

unsigned long long tcuscan_test_tag_period(void) { return chain_tags::kTagMod; }

tcuscan_status_t tcuscan_test_chain_fault(unsigned spin_limit, long long mute_tile)
{
    if (mute_tile > 0x7FFFFFFFll) return TCUSCAN_ERR_INVALID_ARG;
    g_spin_limit.store(spin_limit ? spin_limit : kDefaultSpinLimit, std::memory_order_relaxed);
    g_mute_tile.store(mute_tile < 0 ? kNoTile : (uint32_t)mute_tile, std::memory_order_relaxed);
    return TCUSCAN_OK;
}

tcuscan_status_t tcuscan_scan_static(const void *d_in, void *d_out, size_t rows, size_t cols, tcuscan_dtype_t dt, unsigned flags,
                                     tcuscan_stream_t stream)
{
    if (flags & ~(unsigned)(TCUSCAN_EXCLUSIVE | TCUSCAN_REVERSE)) return TCUSCAN_ERR_INVALID_ARG;
    if (!valid_dtype((int)dt)) return TCUSCAN_ERR_UNSUPPORTED;
    if (rows == 0 || cols == 0) return TCUSCAN_OK;
    if (rows > 0x7FFFFFFFull / ((cols + kSmallTile - 1) / kSmallTile)) return TCUSCAN_ERR_UNSUPPORTED;
    if (tcuscan_workspace_bytes(rows, cols, dt) > sizeof(g_static_scratch)) return TCUSCAN_ERR_WORKSPACE;   // beyond the fixed scratch
    void *scratch = nullptr;
    const tcuscan_status_t st = static_scratch_of_current_device(&scratch);
    if (st != TCUSCAN_OK) return st;
    return run(d_in, d_out, rows, cols, (int)dt, (flags & TCUSCAN_EXCLUSIVE) != 0, (flags & TCUSCAN_REVERSE) != 0,
               scratch, sizeof(g_static_scratch), stream);
}

tcuscan_status_t tcuscan_workspace_fault(const void *d_ws, tcuscan_stream_t stream, unsigned *h_fault)
{
    if (!d_ws || !h_fault) return TCUSCAN_ERR_INVALID_ARG;
    if (d_ws == TCUSCAN_STATIC_SCRATCH) {          // the fixed scratch of tcuscan_scan_static on the current device
        void *scratch = nullptr;
        const tcuscan_status_t st = static_scratch_of_current_device(&scratch);
        if (st != TCUSCAN_OK) return st;
        d_ws = scratch;
    }
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
