// Internal header of libogq: the quantize kernels of the schemes with random rounding (ORQ: Theorem 1, its
// discrete remark, Corollary 1, Algorithm 1 and the random rounding of Section 3.1 of arXiv 2002.11082;
// BinGrad-pb; evenly spaced and Linear-s levels) and their launcher templates.  Included by rounding_part.hip,
// which instantiates one bucket capacity per object file.  Compile with -ffp-contract=off: the rounding decision
// is specified operation by operation in fp32.
#ifndef OGQ_ROUNDING_KERNELS_H
#define OGQ_ROUNDING_KERNELS_H

#include <type_traits>

#include "device_common.h"
#include "launch.h"

namespace ogq {

// ----------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter (c0, c1, 0, 0), key (k0, k1).
// ----------------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1, uint32_t (&r)[4])
{
    uint32_t c2 = 0, c3 = 0;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t pa = (uint64_t)0xD2511F53u * c0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
        // three-input exclusive or in one instruction (v_bitop3_b32, truth table 0x96)
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(pb >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(pa >> 32), c3, k1, 0x96);
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    r[0] = c0; r[1] = c1; r[2] = c2; r[3] = c3;
}

// ----------------------------------------------------------------------------------------------
// ORQ quantize.  One wavefront (= one workgroup) owns one bucket.  Lane l holds, for chunk c, the
// four consecutive bucket elements 256*c + 4*l + {0,1,2,3} (one 16-byte load), which are also the
// four elements that share one Philox block.
//
// A level solve needs (a) counts and sums of the elements below a level and (b) the element of a
// given rank.  The bucket is therefore grouped once, in LDS, by a monotone bin of the value (sign,
// exponent and top mantissa bits, relative to the largest magnitude of the bucket; everything more
// than 16 binades below that shares the two centre bins).  Per-bin counts and fp64 sums are
// prefix-summed; after that a solve touches one bin: the bin holding the wanted rank is sorted
// across the 64 lanes, and the counts and sums below the chosen element are added to the bin's
// prefix.  All values of a regular bin share sign and exponent, so its fp64 sum is exact.
// ----------------------------------------------------------------------------------------------
// Order-preserving map of fp32 onto unsigned integers.
__device__ __forceinline__ uint32_t float_to_key(float f)
{
    const uint32_t u = __float_as_uint(f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}

__device__ __forceinline__ float key_to_float(uint32_t k)
{
    const uint32_t u = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
    return __uint_as_float(u);
}

// Order of the greedy solves (Algorithm 1): the level in the middle of [l, r] is solved from the
// two outer levels, then both halves are treated the same way; the middle index is rounded down
// when s is not of the form 2^K + 1.  Each step is packed as 4 bits of k, l, r; five steps per word.
struct GreedyOrder {
    uint64_t packed[2];
    int count;
};

constexpr void greedy_visit(GreedyOrder& o, int l, int r)
{
    if (r - l < 2) return;
    const int mid = (l + r) / 2;
    o.packed[o.count / 5] |= (uint64_t)(mid | (l << 4) | (r << 8)) << (12 * (o.count % 5));
    ++o.count;
    greedy_visit(o, l, mid);
    greedy_visit(o, mid, r);
}

template <int S>
constexpr GreedyOrder greedy_order()
{
    GreedyOrder o{{0, 0}, 0};
    greedy_visit(o, 0, S - 1);
    return o;
}

// Limbs of the exact sums behind floor(T) (exact_floor_t below): value = sum_i limb[i] * 2^(32 i - 149).  An fp32 value
// starts in limb 7 at the latest and touches three limbs; what the 64 bits of the top limb hold beyond 32 is headroom
// for the sum and the coefficients, and the carry out of it gives the sign.
constexpr int kExactLimbs = 10;

// LDS of one bucket: D = element capacity, B = number of bins.
template <int D_, int B_, int S_>
struct OrqLds {
    static constexpr int D = D_, B = B_;
    static constexpr int BLOCK = D_ / 64;  // positions per entry of the fp64 block prefix
    // fp32 bit patterns grouped by bin (-0 lies with +0), unsorted inside a bin.  Position i lives at
    // word i + i/64, so that the 64 lanes reading consecutive blocks of D/64 positions hit distinct banks.
    uint32_t grouped[D + D / 64];
    uint32_t bin_start[B + 1];  // histogram, then first position of each bin; [B] = bucket length
    double block_prefix[64];    // fp64 sum of all positions before block l (block = D/64 positions)
    // per level k: value; #{v < value}; #{v <= value}; sum{v < value}; sum{v <= value}; the rank it
    // was picked at (0 = not picked by rank)
    double lvl_sum_lt[S_];
    double lvl_sum_le[S_];
    float lvl_value[S_];
    uint32_t lvl_count_lt[S_];
    uint32_t lvl_count_le[S_];
    uint32_t lvl_rank[S_];
    double sum_error_bound;  // 0 when every fp64 sum of the bucket is exact (see floor_t_from_sums)
    unsigned long long exact_limb[1][kExactLimbs];  // workspace of exact_floor_t
};

__device__ __forceinline__ uint32_t skewed(uint32_t position) { return position + (position >> 6); }

// Byte offset of a skewed position in the grouped array, as one shift and one add-and-shift (v_add_lshl_u32; written
// in plain C++ the compiler distributes the shift over the sum and needs three instructions).
__device__ __forceinline__ uint32_t skewed_byte_offset(uint32_t position)
{
    uint32_t offset;
    asm("v_add_lshl_u32 %0, %1, %2, 2" : "=v"(offset) : "v"(position), "v"(position >> 6));
    return offset;
}

// A zero the compiler cannot see through.  x + this turns -0 into +0 like x + 0.0f does, and, unlike that, is not
// recognised as the same value in a later phase: what is derived from the register-resident bucket is computed again
// where it is needed instead of being kept in registers (and no copy of x is made to hide it).
__device__ __forceinline__ float opaque_zero()
{
    float zero = 0.0f;
    asm volatile("" : "+v"(zero));
    return zero;
}

// What the histogram keeps per element: the element's position inside its bin in the upper half, and in the lower half
// the byte offset of its bin's counter from the middle of the bin table (signed, at most +-4096: the low half of the
// very register that addressed the returning add; one byte permute packs the two).
__device__ __forceinline__ uint32_t pack_slot(uint32_t position_in_bin, uint32_t bin, uint32_t half)
{
    return __builtin_amdgcn_perm(position_in_bin, (bin - half) * 4u, 0x05040100u);
}

// First position of the slot's bin: table = the middle of the bin-start table (one sign-extending bit-field extract).
template <class T>
__device__ __forceinline__ uint32_t slot_bin_start(const T* table_middle, uint32_t slot)
{
    const int32_t byte_offset = (int32_t)(int16_t)(slot & 0xFFFFu);
    return *reinterpret_cast<const T*>(reinterpret_cast<const char*>(table_middle) + byte_offset);
}

__device__ __forceinline__ uint32_t umin32(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint32_t umax32(uint32_t a, uint32_t b) { return a > b ? a : b; }

// Bin of a value (with -0 already turned into +0): the HALF bins of either sign cover 16 binades below the
// largest magnitude of the bucket (t_low = its lowest regular bin index); everything smaller shares the two
// centre bins HALF - 1 and HALF.  The upper clamp only acts on NaN.
template <int HALF, int SHIFT>
__device__ __forceinline__ uint32_t value_bin(float canonical, uint32_t t_low)
{
    const uint32_t bits = __float_as_uint(canonical);
    const uint32_t t = (bits & 0x7FFFFFFFu) >> SHIFT;
    const uint32_t u = umin32(__builtin_elementwise_sub_sat(t, t_low), (uint32_t)(HALF - 1));  // 0 .. HALF-1
    const uint32_t negative = (uint32_t)((int32_t)bits >> 31);                                 // 0 or ~0
    return (uint32_t)HALF + (u ^ negative);  // HALF + u, or HALF - 1 - u for a negative value
}

// Sort key of a value as stored in the grouped array (bit pattern of the element; -0 counts as +0).
__device__ __forceinline__ uint32_t stored_key(uint32_t stored) { return float_to_key(__uint_as_float(stored) + 0.0f); }

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x)
{
    x = umax32(x, dpp_u32<kDppXor1>(x));
    x = umax32(x, dpp_u32<kDppXor2>(x));
    x = umax32(x, dpp_u32<kDppHalfMirror>(x));
    x = umax32(x, dpp_u32<kDppMirror>(x));
    return umax32(umax32(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
                  umax32(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) { return ~wave_max_u32(~x); }

// Inclusive scans over the lanes in ascending lane order, in registers: four shifts inside every row of 16
// lanes (a lane without a source adds 0), then the last lane of row 0 / 2 is added to row 1 / 3 and lane 31
// to the upper half (DPP row_shr, row_bcast:15, row_bcast:31).
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr8 = 0x118, kDppRowBcast15 = 0x142,
              kDppRowBcast31 = 0x143;

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero_u32(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xF, false);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_or_zero_f64(double x)
{
    const uint64_t u = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = dpp_or_zero_u32<CTRL, ROW_MASK>((uint32_t)u), hi = dpp_or_zero_u32<CTRL, ROW_MASK>((uint32_t)(u >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x)
{
    x += dpp_or_zero_u32<kDppRowShr1, 0xF>(x);
    x += dpp_or_zero_u32<kDppRowShr2, 0xF>(x);
    x += dpp_or_zero_u32<kDppRowShr4, 0xF>(x);
    x += dpp_or_zero_u32<kDppRowShr8, 0xF>(x);
    x += dpp_or_zero_u32<kDppRowBcast15, 0xA>(x);
    x += dpp_or_zero_u32<kDppRowBcast31, 0xC>(x);
    return x;
}

__device__ __forceinline__ double wave_inclusive_scan_f64(double x)
{
    x += dpp_or_zero_f64<kDppRowShr1, 0xF>(x);
    x += dpp_or_zero_f64<kDppRowShr2, 0xF>(x);
    x += dpp_or_zero_f64<kDppRowShr4, 0xF>(x);
    x += dpp_or_zero_f64<kDppRowShr8, 0xF>(x);
    x += dpp_or_zero_f64<kDppRowBcast15, 0xA>(x);
    x += dpp_or_zero_f64<kDppRowBcast31, 0xC>(x);
    return x;
}

// Ascending bitonic sorts in registers.  Every compare-exchange is ascending: the first step of a merge pairs
// element e with e ^ (run length - 1), i.e. meets the second run in reverse, the others pair e with e ^ J; the lane
// whose bit (run length / 2, or J) is clear keeps the smaller key.  So no step needs a direction, a step is one
// cross-lane move and one median of three, and every row of 16 lanes (half of the wavefront) is sorted ascending
// on its own after 10 (15) of the 21 steps.
constexpr int kDppQuadReverse = 0x1B;  // quad_perm [3,2,1,0]: partner lane ^ 3

// Value held by lane (lane ^ (2 M - 1)): every group of 2 M lanes in reverse order.
template <int M>
__device__ __forceinline__ uint32_t lane_reverse(uint32_t x, uint32_t lane)
{
    if constexpr (M == 1) {
        return dpp_u32<kDppXor1>(x);
    } else if constexpr (M == 2) {
        return dpp_u32<kDppQuadReverse>(x);
    } else if constexpr (M == 4) {
        return dpp_u32<kDppHalfMirror>(x);
    } else if constexpr (M == 8) {
        return dpp_u32<kDppMirror>(x);
    } else if constexpr (M == 16) {
        return lane_xor<16>(dpp_u32<kDppMirror>(x), lane);
    } else {
        static_assert(M == 32, "groups of at most 64 lanes");
        return lane_xor<32>(lane_xor<16>(dpp_u32<kDppMirror>(x), lane), lane);
    }
}

// Median of three (v_med3_u32): with bound = 0 the smaller, with bound = 0xFFFFFFFF the larger of x and y.
__device__ __forceinline__ uint32_t smaller_or_larger(uint32_t x, uint32_t y, uint32_t bound)
{
    return umax32(umin32(x, y), umin32(umax32(x, y), bound));
}

// 0 in the lanes whose bit BIT is clear (they keep the smaller key of a pair), 0xFFFFFFFF in the others.
template <int BIT>
__device__ __forceinline__ uint32_t upper_lanes(uint32_t lane)
{
    return (lane & (uint32_t)BIT) ? 0xFFFFFFFFu : 0u;
}

// One key per lane: merges sorted runs of M lanes into runs of 2 M.
template <int M>
__device__ __forceinline__ uint32_t wave_sort_merge(uint32_t x, uint32_t lane)
{
    x = smaller_or_larger(x, lane_reverse<M>(x, lane), upper_lanes<M>(lane));
    if constexpr (M >= 32) x = smaller_or_larger(x, lane_xor<16>(x, lane), upper_lanes<16>(lane));
    if constexpr (M >= 16) x = smaller_or_larger(x, lane_xor<8>(x, lane), upper_lanes<8>(lane));
    if constexpr (M >= 8) x = smaller_or_larger(x, lane_xor<4>(x, lane), upper_lanes<4>(lane));
    if constexpr (M >= 4) x = smaller_or_larger(x, lane_xor<2>(x, lane), upper_lanes<2>(lane));
    if constexpr (M >= 2) x = smaller_or_larger(x, lane_xor<1>(x, lane), upper_lanes<1>(lane));
    return x;
}

// `count` lanes (the first ones) hold keys, the others 0xFFFFFFFF: with at most 16 (32) keys only the first
// row (half) of the wavefront has to be sorted.
__device__ __forceinline__ uint32_t wave_sort_u32(uint32_t x, uint32_t lane, uint32_t count)
{
    x = wave_sort_merge<1>(x, lane);
    x = wave_sort_merge<2>(x, lane);
    x = wave_sort_merge<4>(x, lane);
    x = wave_sort_merge<8>(x, lane);
    if (count <= 16u) return x;
    x = wave_sort_merge<16>(x, lane);
    if (count <= 32u) return x;
    return wave_sort_merge<32>(x, lane);
}

// The bucket element of a given rank, with the counts and sums of the bucket elements strictly
// below it and not above it.
struct Picked {
    uint32_t key;
    uint32_t count_lt, count_le;
    double sum_lt, sum_le;
};

// The element of 1-based rank `rank`, which lies in the bin that holds positions [first, first + count).  BLOCK =
// positions per entry of the fp64 block prefix (at most 64).
// SUMS = false: only the element is wanted (rules whose solves never read the counts and sums of a picked level: a
// single interior level, Linear-s); the block prefix is then neither needed nor read.
template <int BLOCK, bool SUMS = true, class Lds>
__device__ __forceinline__ Picked pick_in_span(const Lds& lds, uint32_t first, uint32_t count, uint32_t rank, uint32_t lane)
{
    static_assert(BLOCK <= 64, "the head of a block is read one position per lane");
    const uint32_t r_in = rank - first;  // 1-based rank inside the bin

    // sum of everything before the bin = prefix of its block + the block's positions before `first`
    const uint32_t block = first / BLOCK;
    const uint32_t block_first = block * BLOCK;
    double before_block = 0.0;
    float head = 0.0f;
    if constexpr (SUMS) {
        before_block = uniform_f64(lds.block_prefix[block]);
        head = lane < first - block_first ? __uint_as_float(lds.grouped[skewed(block_first + lane)]) : 0.0f;
    }

    uint32_t key, c_lt, c_le;
    double s_lt;
    if (count <= 64u) {
        const uint32_t mine =
            lane < count ? stored_key(lds.grouped[skewed(first + lane)]) : 0xFFFFFFFFu;
        const uint32_t sorted = wave_sort_u32(mine, lane, count);
        key = __builtin_amdgcn_readlane(sorted, r_in - 1u);
        if constexpr (SUMS) {
            const bool lt = sorted < key;
            const bool le = (sorted <= key) && (lane < count);
            c_lt = (uint32_t)__popcll(__ballot(lt));
            c_le = (uint32_t)__popcll(__ballot(le));
            s_lt = wave_sum((double)head + (lt ? (double)key_to_float(sorted) : 0.0));
        } else {
            c_lt = c_le = 0u;
            s_lt = 0.0;
        }
    } else {
        // A crowded bin (many equal or nearly equal values): bisection on the key, over the bits in which the bin's
        // smallest and largest key differ (none when all its values are equal).  Up to 256 keys stay in registers.
        constexpr int HELD = 4;
        const bool held = count <= 64u * HELD;
        uint32_t mine[HELD];
        uint32_t smallest = 0xFFFFFFFFu, largest = 0u;
        if (held) {
#pragma unroll
            for (int c = 0; c < HELD; ++c) {
                const uint32_t i = 64u * c + lane;
                const bool valid = i < count;
                mine[c] = valid ? stored_key(lds.grouped[skewed(first + (valid ? i : 0u))]) : 0xFFFFFFFFu;
                smallest = umin32(smallest, mine[c]);
                largest = umax32(largest, valid ? mine[c] : 0u);
            }
        } else {
            for (uint32_t base = 0; base < count; base += 64u) {
                const uint32_t i = base + lane;
                if (i < count) {
                    const uint32_t k = stored_key(lds.grouped[skewed(first + i)]);
                    smallest = umin32(smallest, k);
                    largest = umax32(largest, k);
                }
            }
        }
        smallest = wave_min_u32(smallest);
        largest = wave_max_u32(largest);
        const uint32_t differing = smallest ^ largest;
        uint32_t prefix = smallest;
        if (differing != 0u) {
            const int top = 31 - __builtin_clz(differing);
            prefix = top == 31 ? 0u : smallest & ~((2u << top) - 1u);  // the bits above `top` are common to all keys
            for (int bit = top; bit >= 0; --bit) {
                const uint32_t cand = prefix | (1u << bit);
                uint32_t below = 0;
                if (held) {
#pragma unroll
                    for (int c = 0; c < HELD; ++c) below += (uint32_t)__popcll(__ballot(mine[c] < cand));
                } else {
                    for (uint32_t base = 0; base < count; base += 64u) {
                        const uint32_t i = base + lane;
                        const uint32_t k = i < count ? stored_key(lds.grouped[skewed(first + i)]) : 0xFFFFFFFFu;
                        below += (uint32_t)__popcll(__ballot(k < cand));
                    }
                }
                if (below < r_in) prefix = cand;
            }
        }
        key = prefix;
        c_lt = 0;
        c_le = 0;
        double part = (double)head;
        if constexpr (SUMS)
        for (uint32_t base = 0; base < count; base += 64u) {
            const uint32_t i = base + lane;
            const float x = i < count ? __uint_as_float(lds.grouped[skewed(first + i)]) + 0.0f : 0.0f;
            const uint32_t k = i < count ? float_to_key(x) : 0xFFFFFFFFu;
            const bool lt = k < key;
            c_lt += (uint32_t)__popcll(__ballot(lt));
            c_le += (uint32_t)__popcll(__ballot(k <= key && i < count));
            part += lt ? (double)x : 0.0;
        }
        s_lt = SUMS ? wave_sum(part) : 0.0;
    }
    Picked p;
    p.key = key;
    p.count_lt = first + c_lt;
    p.count_le = first + c_le;
    p.sum_lt = before_block + s_lt;
    p.sum_le = p.sum_lt + (double)(c_le - c_lt) * (double)key_to_float(key);
    return p;
}

// The same for bin `bin`.
template <int BLOCK, bool SUMS = true, class Lds>
__device__ __forceinline__ Picked pick_in_bin(const Lds& lds, uint32_t bin, uint32_t rank, uint32_t lane)
{
    const uint32_t first = uniform_u32(lds.bin_start[bin]);
    const uint32_t count = uniform_u32(lds.bin_start[bin + 1]) - first;
    return pick_in_span<BLOCK, SUMS>(lds, first, count, rank, lane);
}

// rank is 1-based, 1 <= rank <= bucket length.  my_start[t] = bin_start[lane * PER + t], kept in registers.
template <int D, int B, int S, bool SUMS = true>
__device__ __forceinline__ Picked pick_rank(const OrqLds<D, B, S>& lds, const uint32_t (&my_start)[B / 64],
                                            uint32_t rank, uint32_t lane)
{
    constexpr int PER = B / 64;
    // the bin holding the rank: the last bin whose first position is below the rank (counted on the scalar unit)
    uint32_t starts_below = 0;
#pragma unroll
    for (int t = 0; t < PER; ++t) starts_below += (uint32_t)__popcll(__ballot(my_start[t] < rank));
    const uint32_t bin = starts_below - 1u;  // bin_start[0] = 0 < rank: at least one
    return pick_in_bin<D / 64, SUMS>(lds, bin, rank, lane);
}

// The same with the bin found by two looks into LDS (every (B/64)-th bin start, then the B/64 bins in between):
// no registers are tied up by the bin starts.
template <bool SUMS = true, class Lds>
__device__ __forceinline__ Picked pick_rank_by_lookup(const Lds& lds, uint32_t rank, uint32_t lane)
{
    constexpr uint32_t PER = Lds::B / 64;
    static_assert(PER <= 64, "one lane per bin of a segment");
    const uint32_t coarse = lds.bin_start[lane * PER];
    const uint32_t segment = (uint32_t)__popcll(__ballot(coarse < rank)) - 1u;
    const uint32_t fine = lds.bin_start[segment * PER + (lane < PER ? lane : 0u)];
    const uint32_t within = (uint32_t)__popcll(__ballot(lane < PER && fine < rank)) - 1u;  // the bin is segment * PER + within
    // its first position and that of the next bin are already in the registers of two lanes
    const uint32_t first = __builtin_amdgcn_readlane(fine, within);
    const uint32_t next = within + 1u < PER ? __builtin_amdgcn_readlane(fine, (within + 1u) & 63u)
                          : segment < 63u   ? __builtin_amdgcn_readlane(coarse, (segment + 1u) & 63u)
                                            : uniform_u32(lds.bin_start[Lds::B]);
    return pick_in_span<Lds::BLOCK, SUMS>(lds, first, next - first, rank, lane);
}

// ----------------------------------------------------------------------------------------------
// floor(T) of the discrete optimal condition (second remark after Theorem 1), T = S / (R - L) with
// S = sum over the bucket elements v in [L, R] of (v - L).  The floor decides which element becomes the level, so it
// is the exact one: the largest integer m with S - m (R - L) >= 0.
//
// Fast path.  The sums a solve reads are fp64 sums of fp32 values.  They are exact, whatever their order, when every
// non-zero element of the bucket is at most safe_binades(len) binades below the largest magnitude M < 2^(E+1): every
// element is then a multiple of q = 2^(E - safe - 23), every intermediate value (prefix sums below len * M; their
// differences, S and m (R - L) below 2 len M < len * 2^(E+2)) is a multiple of q below 2^53 q, so no addition,
// difference or product ever rounds.  With
// S exact, floor(S / (R - L)) is corrected by at most one through the sign of the exact rest S - m (R - L).  A bucket
// with smaller non-zero elements ("tiny" ones: they sit in the two centre bins of the grouping) keeps the same
// arithmetic, but a rest within sum_error_bound of 0 or of R - L does not decide; the bound covers 256 roundings of
// half a unit in the last place of a value below 2 len M, more than any prefix sum here goes through.
//
// Exact path (undecided solves only).  Every fp32 value is an integer multiple of 2^-149: the elements in [L, R] are
// added up as signed fixed-point numbers in 10 limbs of 32 payload bits (64-bit LDS atomics; a limb takes at most
// 32768 pieces below 2^32 before the carries are propagated), and m is searched with the sign of
// sum - (c - m) L - m R, c the number of elements in [L, R], which does not grow with m.
// ----------------------------------------------------------------------------------------------

__host__ __device__ constexpr uint32_t ceil_log2(uint32_t n)
{
    uint32_t k = 0;
    while ((1u << k) < n) ++k;
    return k;
}

// How many binades below the largest magnitude a non-zero element may lie for all fp64 sums of a bucket of at most
// `capacity` elements to be exact: capacity * 2 M / q < 2^53 with q = 2^(E - safe - 23) and M < 2^(E+1).
__host__ __device__ constexpr uint32_t safe_binades(uint32_t capacity) { return 28u - ceil_log2(capacity); }

// What the fp64 sums of a bucket with tiny elements can be off by: 2^(ceil_log2(capacity) + E - 44), E the
// unbiased exponent of the largest magnitude (at least the smallest normal double).
__device__ __forceinline__ double sum_error_bound_of(uint32_t mag_max_bits, uint32_t capacity)
{
    const int field = 1023 + ((int)(mag_max_bits >> 23) - 127) + (int)ceil_log2(capacity) - 44;
    return __longlong_as_double((long long)(uint64_t)(field < 1 ? 1 : field) << 52);
}

// Cuts |c * v| into the three 32-bit pieces that go to limbs first, first + 1, first + 2.  first <= 7.
struct ExactPieces {
    uint32_t first;
    bool negative;
    uint64_t piece[3];
};

__device__ __forceinline__ ExactPieces exact_pieces(float v, long long c)
{
    const uint32_t bits = __float_as_uint(v);
    const uint32_t biased = (bits >> 23) & 0xFFu, fraction = bits & 0x7FFFFFu;
    // |v| = mantissa * 2^(position - 149); subnormals have position 0 and no hidden bit
    const uint64_t mantissa = biased ? (fraction | 0x800000u) : fraction;
    const uint32_t position = biased ? biased - 1u : 0u;
    const uint64_t magnitude = mantissa * (uint64_t)(c < 0 ? -c : c);  // below 2^44
    const uint32_t shift = position & 31u;
    const uint64_t low = magnitude << shift;                          // bits 0 .. 63 of magnitude << shift
    const uint64_t high = shift > 20u ? magnitude >> (64u - shift) : 0ull;  // bits 64 .. 74
    ExactPieces p;
    p.first = position >> 5;
    p.negative = ((bits >> 31) != 0u) != (c < 0);
    p.piece[0] = low & 0xFFFFFFFFull;
    p.piece[1] = low >> 32;
    p.piece[2] = high;
    return p;
}

// limb (LDS, shared by the lanes of the group) += v
__device__ __forceinline__ void exact_add_shared(unsigned long long* limb, float v)
{
    const ExactPieces p = exact_pieces(v, 1);
#pragma unroll
    for (int k = 0; k < 3; ++k)
        if (p.piece[k] != 0ull) atomicAdd(&limb[p.first + k], p.negative ? 0ull - p.piece[k] : p.piece[k]);  // signed, mod 2^64
}

// The piece of p that belongs to limb i.
__device__ __forceinline__ long long exact_piece_of(const ExactPieces& p, uint32_t i)
{
    const uint32_t k = i - p.first;  // 0, 1, 2 for the three limbs the value touches
    const uint64_t piece = k == 0u ? p.piece[0] : k == 1u ? p.piece[1] : k == 2u ? p.piece[2] : 0ull;
    return p.negative ? -(long long)piece : (long long)piece;
}

// sum (the limbs) + cl * L + cr * R >= 0 ?  The limbs are only read.  (A rolled loop over the limbs: this rare path
// must not raise the register count of the kernels it is inlined into.)
__device__ __forceinline__ bool exact_not_negative(const unsigned long long* limb, float L, long long cl, float R,
                                                   long long cr)
{
    const ExactPieces pl = exact_pieces(L, cl), pr = exact_pieces(R, cr);
    long long carry = 0;
#pragma unroll 1
    for (uint32_t i = 0; i < (uint32_t)kExactLimbs; ++i) {
        const long long t = (long long)limb[i] + exact_piece_of(pl, i) + exact_piece_of(pr, i) + carry;
        carry = t >> 32;  // floor division by 2^32
    }
    return carry >= 0;  // what is left above the top limb carries the sign
}

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// floor(T), exactly.  Called by all lanes that hold the bucket (a wavefront, or the group of lanes of a small bucket)
// with the same limb array, L < R, count_in = #{L <= v <= R} and a first guess; each_of_mine(f) runs f(x) on the bucket
// elements this lane answers for; lane_in_group counts the calling lanes from 0.
template <class EachFn>
__device__ __forceinline__ uint32_t exact_floor_t(unsigned long long* limb, uint32_t lane_in_group, float L, float R,
                                                  uint32_t count_in, uint32_t guess, EachFn each_of_mine)
{
    if (lane_in_group < (uint32_t)kExactLimbs) limb[lane_in_group] = 0ull;
    wave_lds_sync();
    each_of_mine([&](float x) {
        if (L <= x && x <= R) exact_add_shared(limb, x);
    });
    wave_lds_sync();
    // S - m (R - L) = sum - (count_in - m) L - m R; the first two probes sit at the guess
    uint32_t lo = 0u, hi = count_in;  // m = 0 fits: S >= 0
    uint32_t probe = guess < count_in ? guess : count_in;
    if (probe == 0u) probe = hi > 0u ? 1u : 0u;
    for (int step = 0; lo < hi; ++step) {
        const uint32_t mid = step == 0 ? probe : (step == 1 && lo == probe && probe < hi) ? probe + 1u
                                                                                         : lo + (hi - lo + 1u) / 2u;
        if (exact_not_negative(limb, L, -(long long)(count_in - mid), R, -(long long)mid)) lo = mid;
        else hi = mid - 1u;
    }
    wave_lds_sync();  // every lane is through with the limbs before a later call clears them
    return lo;
}

// The two forms the kernels call, as real functions: inlined into every level solve, this rare path cost the kernels
// 3 to 20 % of their speed (code size, registers) without ever running.
//   bucket grouped in LDS: the calling lanes take the positions lane, lane + stride, ... below len
static __device__ __attribute__((noinline)) uint32_t exact_floor_t_grouped(unsigned long long* limb, const uint32_t* grouped,
                                                                   uint32_t len, uint32_t lane, uint32_t stride, float L,
                                                                   float R, uint32_t count_in, uint32_t guess)
{
    return exact_floor_t(limb, lane, L, R, count_in, guess, [&](auto add) {
        for (uint32_t i = lane; i < len; i += stride) add(__uint_as_float(grouped[skewed(i)]));
    });
}

//   small bucket in registers: every lane of the bucket's group brings four elements, `valid` of which exist
static __device__ __attribute__((noinline)) uint32_t exact_floor_t_registers(unsigned long long* limb, uint32_t lane_in_group,
                                                                     float L, float R, uint32_t count_in, uint32_t guess,
                                                                     float x0, float x1, float x2, float x3, uint32_t valid)
{
    return exact_floor_t(limb, lane_in_group, L, R, count_in, guess, [&](auto add) {
        if (valid > 0u) add(x0);
        if (valid > 1u) add(x1);
        if (valid > 2u) add(x2);
        if (valid > 3u) add(x3);
    });
}

// floor(T) of one solve from the fp64 sums (see above): Ssum = the sums' S, width = R - L > 0 in fp64, bound = the
// bucket's sum_error_bound (0: every sum is exact).  Returns false when the sums do not decide; m is then the guess for
// exact_floor_t.  The quotient only proposes m (a reciprocal and a product instead of a division: any m whose rest
// S - m width lies inside (bound, width - bound) is the floor); the common case costs the reciprocal, a product, a
// floor, a fused multiply-add for the rest and two comparisons.  A rest of exactly 0 (T an integer) or outside
// [0, width) takes the second branch, which moves m by one where the quotient's rounding asks for it.
__device__ __forceinline__ bool floor_t_from_sums(double Ssum, double width, double bound, double& m)
{
    m = fmax(floor(Ssum * __builtin_amdgcn_rcp(width)), 0.0);  // (NaN from non-finite input becomes 0)
    double rest = __builtin_fma(-m, width, Ssum);  // exact when bound == 0: m * width has at most 41 bits
    if (rest > bound && width - rest > bound) return true;
    if (rest < 0.0) {
        m = fmax(m - 1.0, 0.0);
        rest = __builtin_fma(-m, width, Ssum);
    } else if (rest >= width) {
        m += 1.0;
        rest = __builtin_fma(-m, width, Ssum);
    }
    if (bound == 0.0) return true;  // exact sums, exact rest: 0 <= rest < width now
    return rest > bound && width - rest > bound;
}

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Runs f(c, all) for the chunks c (256 elements each) that hold at least one of the `len` valid elements.  `all` is a
// std::true_type when every element of the chunk is valid, so that f can drop its per-element bounds tests: at most one
// chunk of a bucket is cut by its end, and the chunks past it are skipped altogether (wave-uniform branches).
template <int C, bool FULL, class F>
__device__ __forceinline__ void for_each_chunk(uint32_t len, F f)
{
#pragma unroll
    for (int c = 0; c < C; ++c) {
        if (FULL || 256u * (uint32_t)(c + 1) <= len) f(c, std::true_type{});
        else if (256u * (uint32_t)c < len) f(c, std::false_type{});
    }
}

// ---- encode (random rounding, Section 3.1) + pack ------------------------------------------------
// v: the 256*C elements a wavefront holds (lane l, chunk c: elements 256c + 4l + {0..3} of the range that
// starts at global element `begin` and has `len` valid elements; FULL: len == 256*C); lv: the levels.
template <int C, int S, int BITS, bool FULL>
__device__ __forceinline__ void orq_encode(const float (&v)[C][4], const float (&lv)[S], uint32_t len, size_t begin,
                                           uint64_t seed, uint64_t index_offset, uint32_t* __restrict__ codes32)
{
    const uint32_t lane = threadIdx.x & 63u;
    // Per element only the level compares, the selects of (level below, interval width) and the rounding
    // test run on the vector unit; the level index is assembled from the compare masks on the scalar unit
    // (the masks are a thermometer code of the interval, to which the rounding bit is added with carry).
    float width[S - 1];
#pragma unroll
    for (int k = 0; k < S - 1; ++k) width[k] = lv[k + 1] - lv[k];
    uint32_t bit_of[4];  // where element k of this lane sits in its 32-bit half of a packed word
#pragma unroll
    for (int k = 0; k < 4; ++k) bit_of[k] = 1u << (4u * (lane & 7u) + k);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const uint32_t padded_len = (len + 63u) & ~63u;
    const size_t word0 = begin / 64;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        constexpr bool ALL = FULL;
        if constexpr (!FULL) {
            if (256u * (uint32_t)c >= len) continue;  // nothing of the bucket in this chunk: no words to write
        }
        const uint64_t block = (index_offset + begin + 256u * c + 4u * lane) >> 2;
        uint32_t r[4];
        philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), k0, k1, r);
        uint32_t plane[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) plane[p] = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float x = v[c][k];
            // interval: last level not above x, at most S-2
            uint64_t not_below[S];  // [t]: lanes whose element is >= level t, t = 1 .. S-2
            float base = lv[0], w = width[0];
#pragma unroll
            for (int t = 1; t < S - 1; ++t) {
                const bool ge = lv[t] <= x;
                not_below[t] = __ballot(ge);
                base = ge ? lv[t] : base;
                w = ge ? width[t] : w;
            }
            const float delta = x - base;
            const float u = (float)(r[k] >> 8) * 0x1p-24f;
            const float scaled = u * w;
            uint64_t carry = __ballot(scaled < delta);  // rounded up
            if constexpr (!ALL) carry &= __ballot(256u * c + 4u * lane + k < len);
#pragma unroll
            for (int p = 0; p < BITS; ++p) {
                // bit p of the number of levels 1..S-2 not above x
                uint64_t index_bit = 0;
#pragma unroll
                for (int j = 1; (j << p) <= S - 2; j += 2) {
                    const int lo_t = j << p, hi_t = (j + 1) << p;
                    index_bit |= hi_t <= S - 2 ? (not_below[lo_t] & ~not_below[hi_t]) : not_below[lo_t];
                }
                if constexpr (!ALL) index_bit &= __ballot(256u * c + 4u * lane + k < len);
                const uint64_t code_bit = index_bit ^ carry;
                carry &= index_bit;
                plane[p] |= __builtin_amdgcn_inverse_ballot_w64(code_bit) ? bit_of[k] : 0u;
            }
        }
        // OR over the 8 lanes that make up one 32-bit half of a packed word
#pragma unroll
        for (int p = 0; p < BITS; ++p) {
            uint32_t x = plane[p];
            x |= dpp_u32<kDppXor1>(x);
            x |= dpp_u32<kDppXor2>(x);
            x |= dpp_u32<kDppHalfMirror>(x);
            const uint32_t first = 256u * c + 32u * (lane >> 3);  // first element of this half word
            if ((lane & 7u) == 0 && first < padded_len) {
                const size_t word = (word0 + 4u * c + (lane >> 4)) * BITS + p;
                codes32[word * 2 + ((lane >> 3) & 1u)] = x;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Whether the bucket holds a non-zero element more than safe_binades(capacity) binades below its largest magnitude
// (mag_max = its bit pattern), i.e. whether its fp64 sums may round.  Such elements sit in the bins next to zero: the
// two centre bins, which take everything below the binned range, and above 4096 elements also the lowest regular bins.
// Called by `threads` threads (thread = 0 .. threads - 1) once the bucket is grouped; every thread looks at its share
// of those bins and returns what it saw: the caller combines the answers.
template <int HALF, int SHIFT, class Lds>
__device__ __forceinline__ bool any_tiny_element(const Lds& lds, uint32_t capacity, uint32_t mag_max, uint32_t t_low,
                                                 uint32_t thread, uint32_t threads)
{
    const uint32_t safe = safe_binades(capacity);
    const uint32_t biased = mag_max >> 23;
    if (biased <= safe) return false;  // every element is a multiple of 2^-149 and the sums stay below 2^53 of those
    const uint32_t mag_safe = (biased - safe) << 23;  // bit pattern of the smallest safe magnitude
    const uint32_t t_safe = mag_safe >> SHIFT;
    uint32_t bins = t_safe > t_low ? t_safe - t_low : 1u;  // bins per sign that may hold smaller elements
    bins = bins > (uint32_t)HALF ? (uint32_t)HALF : bins;
    const uint32_t first = uniform_u32(lds.bin_start[(uint32_t)HALF - bins]);
    const uint32_t last = uniform_u32(lds.bin_start[(uint32_t)HALF + bins]);
    bool tiny = false;
    for (uint32_t i = first + thread; i < last; i += threads) {
        const uint32_t magnitude = lds.grouped[skewed(i)] & 0x7FFFFFFFu;
        tiny = tiny || (magnitude != 0u && magnitude < mag_safe);
    }
    return tiny;
}

// Where the levels come from; all rules share the random-rounding encoder.
//   kOptimal: ORQ (Theorem 1, Algorithm 1).
//   kPb: BinGrad-pb (Section 3.2): two levels -b_1, +b_1 from the scheme's optimal condition instead of the
//        bucket extremes; the encoder then clamps everything outside them.
//   kEven: QSGD-s / TernGrad (Section 3.1): S levels evenly spaced from -M to +M, M the largest magnitude.
//   kLinear: Linear-s (Section 5): the order statistics at the fractions k/(S-1) of the sorted bucket.
enum LevelRule { kOptimal = 0, kPb = 1, kEven = 2, kLinear = 3 };

// Lane `at` (wave-uniform) of a 64-bit value.
__device__ __forceinline__ double lane_entry_f64(double x, uint32_t at)
{
    const uint64_t u = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)u, at), hi = __builtin_amdgcn_readlane((uint32_t)(u >> 32), at);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// One level solve (discrete optimal condition, second remark after Theorem 1): level k between the current
// levels l and r, whose records (and k's) are in lds.lvl_*.  Run by one whole wavefront.
template <class Lds, class PickFn>
__device__ __forceinline__ void orq_solve_one(Lds& lds, PickFn pick, uint32_t k, uint32_t l, uint32_t r, uint32_t len,
                                              double bound, uint32_t lane)
{
    const float L = uniform_f32(lds.lvl_value[l]);
    const float R = uniform_f32(lds.lvl_value[r]);
    const uint32_t cnt_lt_L = uniform_u32(lds.lvl_count_lt[l]);
    const uint32_t cnt_le_R = uniform_u32(lds.lvl_count_le[r]);
    const double sum_lt_L = uniform_f64(lds.lvl_sum_lt[l]);
    const double sum_le_R = uniform_f64(lds.lvl_sum_le[r]);
    const uint32_t last_rank = uniform_u32(lds.lvl_rank[k]);  // read with the others: one wait for all of them
    bool copy_left = !(L < R);
    Picked p;
    uint32_t rank = 0;
    if (!copy_left) {
        // S = sum_{L<=v<=R} (v - L),  T = S / (R - L),  level = element of rank #{v<=R} - floor(T)
        const uint32_t count_in = cnt_le_R - cnt_lt_L;
        const double Ssum = (sum_le_R - sum_lt_L) - (double)L * (double)count_in;
        const double width = (double)R - (double)L;
        double m;
        if (!floor_t_from_sums(Ssum, width, bound, m)) {
            // the fp64 sums do not decide floor(T): exact sums of the elements in [L, R] (rare)
            m = (double)exact_floor_t_grouped(
                lds.exact_limb[(threadIdx.x >> 6) & (sizeof(lds.exact_limb) / sizeof(lds.exact_limb[0]) - 1u)], lds.grouped, len,
                lane, kWave, L, R, count_in, (uint32_t)m);
        }
        rank = (m >= (double)cnt_le_R) ? 1u : cnt_le_R - (uint32_t)m;
        rank = rank < 1u ? 1u : (rank > len ? len : rank);
        if (rank == last_rank) return;  // same element as last time
        p = pick(rank);
        if (key_to_float(p.key) < L) copy_left = true;
    }
    __builtin_amdgcn_wave_barrier();
    if (lane == 0u) {
        if (copy_left) {
            // the level coincides with the left end (L == R, or rounding put it below L)
            lds.lvl_value[k] = L;
            lds.lvl_count_lt[k] = cnt_lt_L;
            lds.lvl_sum_lt[k] = sum_lt_L;
            lds.lvl_count_le[k] = (L < R) ? uniform_u32(lds.lvl_count_le[l]) : cnt_le_R;
            lds.lvl_sum_le[k] = (L < R) ? uniform_f64(lds.lvl_sum_le[l]) : sum_le_R;
            lds.lvl_rank[k] = 0u;
        } else {
            lds.lvl_value[k] = key_to_float(p.key);
            lds.lvl_count_lt[k] = p.count_lt;
            lds.lvl_count_le[k] = p.count_le;
            lds.lvl_sum_lt[k] = p.sum_lt;
            lds.lvl_sum_le[k] = p.sum_le;
            lds.lvl_rank[k] = rank;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The level records of a bucket held by the wavefront itself (wave-uniform values in registers): what lds.lvl_* keeps,
// for the kernels whose solves all have compile-time level indices.
template <int S>
struct LevelRecords {
    float value[S];
    uint32_t count_lt[S], count_le[S], rank[S];
    double sum_lt[S], sum_le[S];
};

// orq_solve_one on such records: level K between the levels L_ and R_.
template <int K, int L_, int R_, int S, class Lds, class PickFn>
__device__ __forceinline__ void orq_solve_one_in_registers(LevelRecords<S>& st, Lds& lds, PickFn pick, uint32_t len,
                                                           double bound, uint32_t lane)
{
    const float L = st.value[L_], R = st.value[R_];
    const uint32_t cnt_lt_L = st.count_lt[L_], cnt_le_R = st.count_le[R_];
    const double sum_lt_L = st.sum_lt[L_], sum_le_R = st.sum_le[R_];
    if (!(L < R)) {
        // the level coincides with both ends
        st.value[K] = L;
        st.count_lt[K] = cnt_lt_L;
        st.sum_lt[K] = sum_lt_L;
        st.count_le[K] = cnt_le_R;
        st.sum_le[K] = sum_le_R;
        st.rank[K] = 0u;
        return;
    }
    // S = sum_{L<=v<=R} (v - L),  T = S / (R - L),  level = element of rank #{v<=R} - floor(T)
    const uint32_t count_in = cnt_le_R - cnt_lt_L;
    const double Ssum = (sum_le_R - sum_lt_L) - (double)L * (double)count_in;
    const double width = (double)R - (double)L;
    double m;
    if (!floor_t_from_sums(Ssum, width, bound, m)) {
        // the fp64 sums do not decide floor(T): exact sums of the elements in [L, R] (rare)
        m = (double)exact_floor_t_grouped(lds.exact_limb[0], lds.grouped, len, lane, kWave, L, R, count_in, (uint32_t)m);
    }
    uint32_t rank = (m >= (double)cnt_le_R) ? 1u : cnt_le_R - (uint32_t)m;
    rank = rank < 1u ? 1u : (rank > len ? len : rank);
    if (rank == st.rank[K]) return;  // same element as last time
    const Picked p = pick(rank);
    if (key_to_float(p.key) < L) {
        // rounding put the level below L: it coincides with the left end
        st.value[K] = L;
        st.count_lt[K] = cnt_lt_L;
        st.sum_lt[K] = sum_lt_L;
        st.count_le[K] = st.count_le[L_];
        st.sum_le[K] = st.sum_le[L_];
        st.rank[K] = 0u;
    } else {
        st.value[K] = key_to_float(p.key);
        st.count_lt[K] = p.count_lt;
        st.count_le[K] = p.count_le;
        st.sum_lt[K] = p.sum_lt;
        st.sum_le[K] = p.sum_le;
        st.rank[K] = rank;
    }
}

// Schedule of the level solves over the first two wavefronts of a team (Algorithm 1 and the re-solve sweeps;
// the results are those of the serial order).  Greedy: after the root, the solves of the left half only touch levels
// up to the root and those of the right half only levels from the root on, so wavefront 0 takes the left and
// wavefront 1 the right half, step by step.  Sweeps, two at a time: wavefront 0 runs sweep s, wavefront 1 sweep
// s + 1 two levels behind it (level k of a sweep needs level k - 1 of the same sweep and level k + 1 of the sweep
// before).  Where wavefront 0 runs out of greedy solves before wavefront 1 (8 levels), it starts the first sweep in
// those steps.  Every wavefront of the workgroup must call this; a workgroup barrier ends every step.
struct TeamGreedy {
    uint16_t entry[2][8];  // k | l << 4 | r << 8 per wavefront and step; 0 = idle
    int steps;
    // Greedy steps in which wavefront 0 has nothing left to do and can already run the first solves of the first
    // sweep (levels 1, 2): head_step[h] = the step that takes level h + 1, or -1.  Possible when the greedy value of
    // level h + 2 is final by then and the solve of wavefront 1 in that step touches none of the levels h .. h + 2.
    int head_step[2];
    int head;
};

template <int S>
constexpr TeamGreedy team_greedy()
{
    const GreedyOrder o = greedy_order<S>();
    TeamGreedy g{{{0, 0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0, 0}}, 0, {-1, -1}, 0};
    int next[2] = {1, 1};
    int root = 0;
    for (int i = 0; i < o.count; ++i) {
        const uint32_t e = (uint32_t)(o.packed[i / 5] >> (12 * (i % 5))) & 0xFFFu;
        const int k = (int)(e & 15u);
        if (i == 0) {
            root = k;
            g.entry[0][0] = (uint16_t)e;
        } else {
            const int w = k < root ? 0 : 1;
            g.entry[w][next[w]++] = (uint16_t)e;
        }
    }
    g.steps = o.count == 0 ? 0 : (next[0] > next[1] ? next[0] : next[1]);
    g.head_step[0] = g.head_step[1] = -1;
    g.head = 0;
    for (int step = 1; step < g.steps && g.head < 2; ++step) {
        if (g.entry[0][step] != 0) continue;
        bool later_work = false;  // only trailing idle steps of wavefront 0
        for (int q = step; q < g.steps; ++q) later_work = later_work || g.entry[0][q] != 0;
        if (later_work) continue;
        const int h = g.head, level = h + 1;
        if (level > S - 2) break;
        // greedy value of level + 1 final before this step (or it is the top level)
        bool right_final = level + 1 == S - 1;
        for (int w = 0; w < 2; ++w)
            for (int q = 0; q < step; ++q)
                if (g.entry[w][q] != 0 && (int)(g.entry[w][q] & 15u) == level + 1) right_final = true;
        const uint32_t other = g.entry[1][step];
        const int ok = (int)(other & 15u), ol = (int)((other >> 4) & 15u), orr = (int)((other >> 8) & 15u);
        const bool apart = other == 0 || ((ok < level - 1 || ok > level + 1) && ol != level && orr != level);
        if (!right_final || !apart) break;
        g.head_step[h] = step;
        ++g.head;
    }
    return g;
}

// The greedy steps are unrolled (their level indices are compile-time constants: measured 3-4 % faster on 8 levels
// than one loop over a packed table, at equal register counts).
template <int S, class Lds, class PickFn>
__device__ __forceinline__ void orq_team_solve(Lds& lds, PickFn pick, uint32_t wave, uint32_t len, uint32_t sweeps,
                                               uint32_t lane)
{
    constexpr TeamGreedy greedy = team_greedy<S>();
    constexpr uint32_t INTERIOR = S - 2;
    const double bound = uniform_f64(lds.sum_error_bound);  // (see floor_t_from_sums)
#pragma unroll
    for (int step = 0; step < greedy.steps; ++step) {
        if (wave < 2u) {
            const uint32_t e = wave == 0u ? greedy.entry[0][step] : greedy.entry[1][step];
            if (e != 0u) orq_solve_one(lds, pick, e & 15u, (e >> 4) & 15u, (e >> 8) & 15u, len, bound, lane);
            if (wave == 0u && sweeps > 0u) {  // head start of the first sweep
                if (greedy.head_step[0] == step) orq_solve_one(lds, pick, 1u, 0u, 2u, len, bound, lane);
                if (greedy.head_step[1] == step) orq_solve_one(lds, pick, 2u, 1u, 3u, len, bound, lane);
            }
        }
        __syncthreads();
    }
    for (uint32_t s = 0; s < sweeps; s += 2u) {
        const bool pair = s + 1u < sweeps;
        const uint32_t steps = INTERIOR + (pair ? 2u : 0u);
        for (uint32_t t = (s == 0u ? (uint32_t)greedy.head : 0u); t < steps; ++t) {
            if (wave == 0u && t < INTERIOR) orq_solve_one(lds, pick, t + 1u, t, t + 2u, len, bound, lane);
            if (wave == 1u && pair && t >= 2u) orq_solve_one(lds, pick, t - 1u, t - 2u, t, len, bound, lane);
            __syncthreads();
        }
    }
}

// fp64 sum of the grouped positions [0, position), position < bucket length: the prefix of its block plus the
// block's positions before it.
template <class Lds>
__device__ __forceinline__ double sum_before_position(const Lds& lds, uint32_t position, uint32_t lane)
{
    constexpr uint32_t BLOCK = Lds::BLOCK;
    const uint32_t block = position / BLOCK;
    const uint32_t block_first = block * BLOCK;
    const float head = lane < position - block_first ? __uint_as_float(lds.grouped[skewed(block_first + lane)]) : 0.0f;
    return uniform_f64(lds.block_prefix[block]) + wave_sum((double)head);
}

// Run solve(k, l, r) with compile-time level indices: the greedy order of Algorithm 1, and one re-solve sweep.
template <int S, int STEP, class Solve>
__device__ __forceinline__ void for_greedy_steps(Solve&& solve)
{
    constexpr GreedyOrder order = greedy_order<S>();
    if constexpr (STEP < order.count) {
        constexpr uint32_t e =
            STEP < 5 ? (uint32_t)(order.packed[0] >> (12 * STEP)) : (uint32_t)(order.packed[1] >> (12 * (STEP - 5)));
        solve(std::integral_constant<int, (int)(e & 15u)>{}, std::integral_constant<int, (int)((e >> 4) & 15u)>{},
              std::integral_constant<int, (int)((e >> 8) & 15u)>{});
        for_greedy_steps<S, STEP + 1>(solve);
    }
}

template <int S, int K, class Solve>
__device__ __forceinline__ void for_sweep_levels(Solve&& solve)
{
    if constexpr (K + 1 < S) {
        solve(std::integral_constant<int, K>{}, std::integral_constant<int, K - 1>{}, std::integral_constant<int, K + 1>{});
        for_sweep_levels<S, K + 1>(solve);
    }
}

// The level solves of one bucket, run by one wavefront once the bucket is grouped in LDS and the level
// records of the two ends are set.  pick(rank) returns the element of that 1-based rank (Picked); `zeros` is the
// number of zeros in the bucket (BinGrad-pb only).  Interior levels end up in lds.lvl_value; returns b_1 for
// BinGrad-pb.
template <int S, int RULE, class Lds, class PickFn, class EdgeFn>
__device__ __forceinline__ float orq_solve_levels(Lds& lds, PickFn pick, EdgeFn lower_edge_of_bin, uint32_t len,
                                                  uint32_t zeros, uint32_t sweeps, uint32_t lane)
{
    constexpr bool PB = RULE == kPb;
    float pb_level = 0.0f;
    if constexpr (PB) {
        // ---- b_1: minimise |b * #{v > 0} - sum_{v >= b} v| over the positive bucket values.  The
        //      difference grows with b, so the minimiser is one of the two values around its sign
        //      change, which a bisection over the ranks of the positive values finds. -------------
                const uint32_t not_positive = uniform_u32(lds.bin_start[Lds::B / 2]) + zeros;  // negatives fill the lower bins
        const uint32_t positives = len - not_positive;
        const double total = uniform_f64(lds.lvl_sum_le[S - 1]);
        if (positives > 0u) {
            // First the bin: every element of a positive bin j lies below the lower edge e of bin j + 1, so its
            // gap is below gap(e) = e * #{v > 0} - (sum of the bins above j); the wanted value sits in the first bin
            // j whose gap(e) is not negative, or is the first element after it.  One block-prefix look-up per step.
            uint32_t bin_lo = (uint32_t)(Lds::B / 2), bin_hi = (uint32_t)Lds::B - 1u;
            // All positive bins at once, one per lane: the sum before a position lies between the prefixes of the
            // block it falls into and of the next block (positive bins hold positive values), which brackets
            // gap(e) from both sides and decides its sign for every bin except the few whose first position shares
            // a block with the sign change; the bisection then runs over those only.  (A block that begins among the
            // negative values gives no lower bracket.)
            const uint32_t first_not_negative = uniform_u32(lds.bin_start[Lds::B / 2]);
            for (uint32_t bin0 = (uint32_t)(Lds::B / 2); bin0 < (uint32_t)Lds::B; bin0 += kWave) {
                const uint32_t bin = bin0 + lane;
                const uint32_t above = lds.bin_start[bin + 1u];
                const uint32_t block = above / (uint32_t)Lds::BLOCK;
                const bool inside = above < len;  // otherwise nothing lies above the bin: gap(e) >= 0
                const double before_lo = inside ? lds.block_prefix[block] : total;
                const double before_hi =
                    inside && (block + 1u) * (uint32_t)Lds::BLOCK < len ? lds.block_prefix[block + 1u] : total;
                const double scaled_edge = (double)lower_edge_of_bin(bin + 1u) * (double)positives;
                const bool bracketed_below = !inside || block * (uint32_t)Lds::BLOCK >= first_not_negative;
                const uint64_t surely_not_negative =
                    __ballot(bracketed_below && scaled_edge - (total - before_lo) >= 0.0);
                const uint64_t surely_negative = __ballot(scaled_edge - (total - before_hi) < 0.0);
                if (surely_negative != 0)
                    bin_lo = umax32(bin_lo, bin0 + 64u - (uint32_t)__builtin_clzll(surely_negative));
                if (surely_not_negative != 0)
                    bin_hi = umin32(bin_hi, bin0 + (uint32_t)__builtin_ctzll(surely_not_negative));
            }
            if (bin_lo > bin_hi) bin_lo = bin_hi;  // only rounding can make the two bounds cross
            while (bin_lo < bin_hi) {
                const uint32_t mid = (bin_lo + bin_hi) >> 1;
                const uint32_t above = uniform_u32(lds.bin_start[mid + 1u]);  // first position of the bins above mid
                const double sum_above = above < len ? total - sum_before_position(lds, above, lane) : 0.0;
                const double gap = (double)lower_edge_of_bin(mid + 1u) * (double)positives - sum_above;
                if (gap >= 0.0) bin_hi = mid;
                else bin_lo = mid + 1u;
            }
            const uint32_t first_of_bin = uniform_u32(lds.bin_start[bin_lo]);
            const uint32_t first_above = uniform_u32(lds.bin_start[bin_lo + 1u]);
            // Then the value inside it.  A bin of at most 64 elements is sorted once and every distinct positive value
            // of it gets its gap in its own lane (the sum of the strictly smaller elements is an exclusive scan at the
            // first lane that holds the value); larger bins, and the case that the wanted value is the first one
            // above the bin, take the bisection over ranks below.
            const uint32_t count = first_above - first_of_bin;
            bool done = false;
            if (count > 0u && count <= 64u) {
                const uint32_t mine = lane < count ? stored_key(lds.grouped[skewed(first_of_bin + lane)]) : 0xFFFFFFFFu;
                const uint32_t sorted = wave_sort_u32(mine, lane, count);
                const float value = lane < count ? key_to_float(sorted) : 0.0f;
                const double below_bin = sum_before_position(lds, first_of_bin, lane);
                const double smaller = below_bin + (wave_inclusive_scan_f64((double)value) - (double)value);
                const uint32_t previous = (uint32_t)__shfl_up((int)sorted, 1, kWave);
                const bool candidate = lane < count && value > 0.0f && (lane == 0u || previous != sorted);
                const double gap = (double)value * (double)positives - (total - smaller);
                const uint64_t not_negative = __ballot(candidate && gap >= 0.0);
                if (not_negative != 0) {
                    const uint32_t at = (uint32_t)__builtin_ctzll(not_negative);  // first lane of the wanted value
                    const uint32_t up_key = __builtin_amdgcn_readlane(sorted, at);
                    const double gap_up = lane_entry_f64(gap, at);
                    pb_level = key_to_float(up_key);
                    const uint32_t count_lt = first_of_bin + at;  // elements of the bucket below the wanted value
                    if (count_lt > not_positive) {  // a smaller positive value exists
                        float down;
                        double gap_down;
                        if (at > 0u) {
                            const uint32_t down_key = __builtin_amdgcn_readlane(sorted, at - 1u);
                            const uint32_t down_at = (uint32_t)__popcll(__ballot(sorted < down_key));  // its first lane
                            down = key_to_float(down_key);
                            gap_down = lane_entry_f64(gap, down_at);
                        } else {
                            const Picked below = pick(count_lt);
                            down = key_to_float(below.key);
                            gap_down = (double)down * (double)positives - (total - below.sum_lt);
                        }
                        if (fabs(gap_down) <= fabs(gap_up)) pb_level = down;  // ties take the smaller value
                    }
                    done = true;
                }
            }
            if (!done) {
                // 1-based ranks; the first element above the bin, like the largest value of the bucket, always has
                // gap >= 0
                const uint32_t hi_rank = umin32(len, first_above + 1u);
                uint32_t lo = umin32(umax32(not_positive, first_of_bin) + 1u, hi_rank), hi = hi_rank;
                while (lo < hi) {
                    const uint32_t mid = (lo + hi) >> 1;
                    const Picked p = pick(mid);
                    const double gap = (double)key_to_float(p.key) * (double)positives - (total - p.sum_lt);
                    if (gap >= 0.0) hi = mid;
                    else lo = mid + 1u;
                }
                const Picked up = pick(lo);
                const double gap_up = (double)key_to_float(up.key) * (double)positives - (total - up.sum_lt);
                pb_level = key_to_float(up.key);
                if (up.count_lt > not_positive) {  // a smaller positive value exists: rank count_lt is the next one down
                    const Picked down = pick(up.count_lt);
                    const double gap_down =
                        (double)key_to_float(down.key) * (double)positives - (total - down.sum_lt);
                    if (fabs(gap_down) <= fabs(gap_up)) pb_level = key_to_float(down.key);  // ties take the smaller value
                }
            }
        }
    }

    if constexpr (RULE == kLinear) {
        for (uint32_t k = 1; k + 1 < (uint32_t)S; ++k) {
            const uint32_t rank = 1u + (uint32_t)(((uint64_t)k * (len - 1u)) / (uint32_t)(S - 1));
            const Picked p = pick(rank);
            if (lane == 0u) lds.lvl_value[k] = key_to_float(p.key);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // ---- level solves: greedy recursion (Algorithm 1), then re-solve sweeps ------------------
    [[maybe_unused]] const double bound = RULE == kOptimal ? uniform_f64(lds.sum_error_bound) : 0.0;  // (see floor_t_from_sums)
    if constexpr (S > 2 && S <= 4 && RULE == kOptimal && std::is_same_v<decltype(lds.exact_limb), unsigned long long[1][kExactLimbs]>) {
        // One wavefront, three or four levels: every solve with compile-time level indices and the level records in the
        // wavefront's registers instead of LDS (greedy + S - 2 copies of the routine; with five levels the records no
        // longer fit the 128 registers).
        LevelRecords<S> st;
#pragma unroll
        for (int k = 0; k < S; ++k) {
            st.value[k] = uniform_f32(lds.lvl_value[k]);
            st.rank[k] = 0u;
            st.count_lt[k] = st.count_le[k] = k == S - 1 ? len : 0u;
            st.sum_lt[k] = st.sum_le[k] = k == S - 1 ? uniform_f64(lds.lvl_sum_le[S - 1]) : 0.0;
        }
        auto solve = [&](auto kc, auto lc, auto rc) {
            orq_solve_one_in_registers<decltype(kc)::value, decltype(lc)::value, decltype(rc)::value>(st, lds, pick, len, bound, lane);
        };
        for_greedy_steps<S, 0>(solve);
        for (uint32_t sweep = 0; sweep < sweeps; ++sweep) for_sweep_levels<S, 1>(solve);
        if (lane == 0u) {
#pragma unroll
            for (int k = 1; k < S - 1; ++k) lds.lvl_value[k] = st.value[k];
        }
        wave_lds_sync();
    } else if constexpr (S > 2 && S <= 5 && RULE == kOptimal) {
        // few levels: every solve with compile-time level indices
        auto solve = [&](auto kc, auto lc, auto rc) {
            orq_solve_one(lds, pick, (uint32_t)decltype(kc)::value, (uint32_t)decltype(lc)::value, (uint32_t)decltype(rc)::value,
                          len, bound, lane);
        };
        for_greedy_steps<S, 0>(solve);
        for (uint32_t sweep = 0; sweep < sweeps; ++sweep) for_sweep_levels<S, 1>(solve);
    } else if constexpr (S > 2 && RULE == kOptimal) {
    constexpr GreedyOrder order = greedy_order<S>();
    const uint32_t steps = order.count + sweeps * (S - 2);
    for (uint32_t step = 0; step < steps; ++step) {
        uint32_t k, l, r;
        if (step < (uint32_t)order.count) {
            const uint32_t e = step < 5u ? (uint32_t)(order.packed[0] >> (12 * step))
                                         : (uint32_t)(order.packed[1] >> (12 * (step - 5u)));
            k = e & 15u; l = (e >> 4) & 15u; r = (e >> 8) & 15u;
        } else {
            k = 1u + (step - order.count) % (S - 2);
            l = k - 1u; r = k + 1u;
        }
        orq_solve_one(lds, pick, k, l, r, len, bound, lane);
    }
    }
    return pb_level;
}

template <int C>
struct OrqShape {
    static constexpr int D = 256 * C;               // element capacity of the wave
    static constexpr int B = C >= 16 ? 512 : 256;   // bins
    static constexpr int SHIFT = C >= 16 ? 19 : 20; // magnitude bits dropped: keeps exponent + 4 (3) mantissa bits
};

// FULL: the bucket has exactly 256*C elements (no padding, no per-element validity tests).
// S levels per bucket, BITS bits per level index (S = 2^BITS, or 2^(BITS-1) + 1 for the paper's counts).
template <int C, int S, int BITS, bool FULL, bool CLIP, int RULE>
__device__ __forceinline__ void orq_bucket(OrqLds<OrqShape<C>::D, OrqShape<C>::B, S>& lds, const float* __restrict__ g,
                                           uint32_t len, size_t begin, uint32_t bucket, uint32_t sweeps, float clip,
                                           uint64_t seed, uint64_t index_offset, float* __restrict__ levels,
                                           uint32_t* __restrict__ codes32)
{
    static_assert(S >= 2 && S <= 9 && S <= (1 << BITS), "level count does not fit the index width");
    constexpr int D = OrqShape<C>::D;
    constexpr int B = OrqShape<C>::B;
    constexpr int PER = B / 64;   // bins per lane in the prefix step
    constexpr int HALF = B / 2;   // bins per sign
    constexpr int SHIFT = OrqShape<C>::SHIFT;
    constexpr bool full = FULL;
    constexpr bool PB = RULE == kPb;
    const uint32_t lane = threadIdx.x & 63u;

    // ---- load (read once: bypass the caches); padding holds +0 and is never binned or encoded ----
    float v[C][4];
    if (full) {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const floatx4 q = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + 256 * c + 4 * lane));
            v[c][0] = q.x; v[c][1] = q.y; v[c][2] = q.z; v[c][3] = q.w;
        }
    } else if (len % 4u == 0u) {
        // a bucket shorter than the wavefront's capacity whose length is a multiple of 4 (every bucket but a ragged
        // last one): whole 16-byte loads, the lanes past the end read the bucket's first elements and drop them
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const uint32_t e = 256u * c + 4u * lane;
            const bool inside = e < len;
            const floatx4 q = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + (inside ? e : 0u)));
            v[c][0] = inside ? q.x : 0.0f; v[c][1] = inside ? q.y : 0.0f;
            v[c][2] = inside ? q.z : 0.0f; v[c][3] = inside ? q.w : 0.0f;
        }
    } else {
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t e = 256u * c + 4u * lane + k;
                v[c][k] = e < len ? g[e] : 0.0f;
            }
    }

    if constexpr (CLIP) {
        float(&flat)[4 * C] = reinterpret_cast<float(&)[4 * C]>(v);
        clip_in_registers<4 * C>(flat, len, clip, [&](int j) { return full || (64u * (j & ~3) + 4u * lane + (j & 3) < len); });
    }

    // ---- extremes ------------------------------------------------------------------------------
    float lane_min = __uint_as_float(0x7F800000u), lane_max = __uint_as_float(0xFF800000u);
    uint32_t lane_zeros = 0;
    for_each_chunk<C, FULL>(len, [&](int c, auto all) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < len);
            lane_min = fminf(lane_min, valid ? v[c][k] : __uint_as_float(0x7F800000u));
            lane_max = fmaxf(lane_max, valid ? v[c][k] : __uint_as_float(0xFF800000u));
            if constexpr (PB) lane_zeros += (valid && v[c][k] == 0.0f) ? 1u : 0u;
        }
    });
    const float bucket_min = wave_min(lane_min) + 0.0f;  // -0 -> +0
    const float bucket_max = wave_max(lane_max) + 0.0f;
    const uint32_t key_min = float_to_key(bucket_min), key_max = float_to_key(bucket_max);
    const uint32_t mag_max = umax32(__float_as_uint(bucket_min) & 0x7FFFFFFFu, __float_as_uint(bucket_max) & 0x7FFFFFFFu);
    const uint32_t t_max = mag_max >> SHIFT;
    const uint32_t t_low = __builtin_elementwise_sub_sat(t_max, (uint32_t)(HALF - 1));

    float pb_level = 0.0f;
    if constexpr ((S > 2 && RULE != kEven) || PB) {
        // ---- histogram: the returning LDS add hands every element its position inside its bin ------
#pragma unroll
        for (int t = 0; t < PER; ++t) lds.bin_start[lane * PER + t] = 0u;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        uint32_t slot[C][4];  // bin | position inside the bin << 16 (pack_slot)
        const float zero = opaque_zero();
        for_each_chunk<C, FULL>(len, [&](int c, auto all) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < len);
                const uint32_t bin = value_bin<HALF, SHIFT>(v[c][k] + zero, t_low);
                slot[c][k] = 0u;
                if (valid) slot[c][k] = pack_slot(atomicAdd(&lds.bin_start[bin], 1u), bin, (uint32_t)HALF);
            }
        });
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- exclusive prefix over the bin counts (lane l owns bins l*PER .. l*PER+PER-1) ------------
        uint32_t my_start[PER];
        {
            uint32_t cnt[PER];
            uint32_t tot = 0;
#pragma unroll
            for (int t = 0; t < PER; ++t) {
                cnt[t] = lds.bin_start[lane * PER + t];
                tot += cnt[t];
            }
            uint32_t run = wave_inclusive_scan_u32(tot) - tot;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int t = 0; t < PER; ++t) {
                my_start[t] = run;
                lds.bin_start[lane * PER + t] = run;
                run += cnt[t];
            }
            if (lane == 63u) lds.bin_start[B] = run;  // = len
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- scatter the values into their bins: the bin starts of a group of elements are all read before the
        //      group's values are written (a read behind a write to the same LDS object would wait for it) ------
        constexpr int GROUP = C < 4 ? C : 4;
        auto scatter_group = [&](int c0, auto all) {
#pragma unroll
            for (int c = c0; c < c0 + GROUP; ++c)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < len);
                    if (valid) slot[c][k] = slot_bin_start(&lds.bin_start[HALF], slot[c][k]) + (slot[c][k] >> 16);
                }
#pragma unroll
            for (int c = c0; c < c0 + GROUP; ++c)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < len);
                    if (valid)
                        *reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(lds.grouped) + skewed_byte_offset(slot[c][k])) =
                            __float_as_uint(v[c][k]);
                }
        };
#pragma unroll
        for (int c0 = 0; c0 < C; c0 += GROUP) {
            if (full || 256u * (uint32_t)(c0 + GROUP) <= len) scatter_group(c0, std::true_type{});
            else if (256u * (uint32_t)c0 < len) scatter_group(c0, std::false_type{});
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- fp64 prefix of the grouped values at block granularity (lane l sums block l) ------------
        // Only the rules whose solves read the counts and sums of picked levels need it: with a single interior
        // level the one solve reads the bucket's total alone, and Linear-s reads nothing.
        constexpr bool SUMS = (RULE == kOptimal && S > 3) || PB;
        {
            double incl = 0.0;
            if constexpr (SUMS) {
                constexpr uint32_t BLOCK = D / 64;
                double part = 0.0;
#pragma unroll
                for (uint32_t i = 0; i < BLOCK; ++i) {
                    const uint32_t position = lane * BLOCK + i;
                    const float x = position < len ? __uint_as_float(lds.grouped[skewed(position)]) : 0.0f;
                    part += (double)x;
                }
                incl = wave_inclusive_scan_f64(part);
                lds.block_prefix[lane] = incl - part;
            } else if constexpr (RULE == kOptimal) {
                double part = 0.0;
                for_each_chunk<C, FULL>(len, [&](int c, auto all) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < len);
                        part += valid ? (double)v[c][k] : 0.0;
                    }
                });
                incl = wave_sum(part);  // the same in every lane
            }
            if (lane == 63u) {
                // the top level is only ever the right end of a solve
                lds.lvl_count_le[S - 1] = len;
                lds.lvl_sum_le[S - 1] = incl;
                lds.lvl_count_lt[S - 1] = len;
                lds.lvl_sum_lt[S - 1] = incl;
            }
        }
        if (lane == 0u) {
            // the bottom level is only ever the left end of a solve
            lds.lvl_count_lt[0] = 0u;
            lds.lvl_sum_lt[0] = 0.0;
            lds.lvl_count_le[0] = 0u;
            lds.lvl_sum_le[0] = 0.0;
        }
        if (lane < (uint32_t)S) {
            lds.lvl_value[lane] = key_to_float(lane == (uint32_t)(S - 1) ? key_max : key_min);
            lds.lvl_rank[lane] = 0u;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        if constexpr (RULE == kOptimal && S > 2) {
            const bool tiny = __ballot(any_tiny_element<HALF, SHIFT>(lds, (uint32_t)D, mag_max, t_low, lane, kWave)) != 0;
            if (lane == 0u) lds.sum_error_bound = tiny ? sum_error_bound_of(mag_max, (uint32_t)D) : 0.0;
            wave_lds_sync();
        }
        const uint32_t zeros = PB ? wave_sum_u32(lane_zeros) : 0u;
        pb_level = orq_solve_levels<S, RULE>(
            lds, [&](uint32_t rank) { return pick_rank<D, B, S, SUMS>(lds, my_start, rank, lane); },
            [&](uint32_t bin) { return __uint_as_float((t_low + (bin - (uint32_t)HALF)) << SHIFT); }, len, zeros, sweeps, lane);
    }

    // every lane holds its own copy of the levels (the selects of the encoder take vector sources)
    float lv[S];
    if constexpr (RULE == kEven) {
        const double largest = (double)__uint_as_float(mag_max);
#pragma unroll
        for (int k = 0; k < S; ++k) lv[k] = (float)(largest * (double)(2 * k - (S - 1)) / (double)(S - 1));
    } else {
        lv[0] = PB ? -pb_level : key_to_float(key_min);
        lv[S - 1] = PB ? pb_level : key_to_float(key_max);
#pragma unroll
        for (int k = 1; k < S - 1; ++k) lv[k] = lds.lvl_value[k];
    }

    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < S; ++k) levels[(size_t)bucket * S + k] = lv[k];
    }

    orq_encode<C, S, BITS, FULL>(v, lv, len, begin, seed, index_offset, codes32);
}

// C = 8 (2048-element buckets): 16 buckets fit the LDS of a CU, so the kernel is held to the 128 registers
// that let 4 wavefronts share a SIMD (the clipping variants would otherwise take ~138).
template <int C, int S, int BITS, bool CLIP, int RULE>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(C == 8 ? 4 : 1))) void orq_quantize_kernel(const float* __restrict__ grad, size_t n,
                                                             uint32_t bucket_size, uint32_t sweeps, float clip,
                                                             uint32_t num_buckets, uint64_t seed,
                                                             uint64_t index_offset, float* __restrict__ levels,
                                                             uint32_t* __restrict__ codes32)
{
    __shared__ OrqLds<OrqShape<C>::D, OrqShape<C>::B, S> lds;
    const uint32_t bucket = blockIdx.x;
    if (bucket >= num_buckets) return;
    const size_t begin = (size_t)bucket * bucket_size;
    const size_t rest = n - begin;
    const uint32_t len = rest < bucket_size ? (uint32_t)rest : bucket_size;
    if (len == (uint32_t)OrqShape<C>::D)
        orq_bucket<C, S, BITS, true, CLIP, RULE>(lds, grad + begin, len, begin, bucket, sweeps, clip, seed, index_offset, levels, codes32);
    else
        orq_bucket<C, S, BITS, false, CLIP, RULE>(lds, grad + begin, len, begin, bucket, sweeps, clip, seed, index_offset, levels, codes32);
}

// Clipping when a wavefront holds NB whole buckets (lane l: elements 4l .. 4l+3 of the wavefront's 256, bucket
// l / G with G = 64 / NB): clip_in_registers with the sums taken over the bucket's group of lanes.
template <int NB, bool FULL>
__device__ __forceinline__ void clip_small_buckets(float (&v)[4], uint32_t len, float clip, uint32_t lane)
{
    constexpr uint32_t G = 64u / NB, D = 256u / NB;
    const uint32_t q = lane / G;
    uint32_t count = D;
    if constexpr (!FULL) count = q * D < len ? (len - q * D < D ? len - q * D : D) : 1u;  // (no element: nothing is stored)
    clip_in_registers<4>(
        v, count, clip, [&](int j) { return FULL || 4u * lane + j < len; },
        [&](double x) {
            x += dpp_f64<kDppXor1>(x);
            x += dpp_f64<kDppXor2>(x);
            x += dpp_f64<kDppHalfMirror>(x);
            x += dpp_f64<kDppMirror>(x);
            if constexpr (G == 32u) {
                const uint64_t u = (uint64_t)__double_as_longlong(x);
                const uint32_t lo = lane_xor<16>((uint32_t)u, lane), hi = lane_xor<16>((uint32_t)(u >> 32), lane);
                x += __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
            }
            return x;
        });
}

// ----------------------------------------------------------------------------------------------
// Evenly spaced levels (QSGD-s, TernGrad) for buckets of 64 or 128 elements: one wavefront takes 256 consecutive
// elements, i.e. NB = 4 or 2 whole buckets (lane l holds elements 4l .. 4l+3, bucket l / G of the wavefront with
// G = 64 / NB lanes per bucket), instead of leaving three quarters or half of its lanes idle.  The only statistic of
// the rule, the largest magnitude, is reduced inside each group of G lanes; every lane then holds the levels of its
// own bucket, which is all the encoder needs.
// ----------------------------------------------------------------------------------------------
template <int S, int BITS, int NB, bool FULL>
__device__ __forceinline__ void even_small_span(const float* __restrict__ g, uint32_t len, size_t begin, uint32_t first_bucket,
                                                float clip, uint64_t seed, uint64_t index_offset,
                                                float* __restrict__ levels, uint32_t* __restrict__ codes32)
{
    constexpr uint32_t G = 64u / NB;           // lanes per bucket
    constexpr uint32_t D = 256u / NB;          // elements per bucket
    const uint32_t lane = threadIdx.x & 63u;
    float v[1][4];
    if (FULL || len % 4u == 0u) {
        const bool inside = FULL || 4u * lane < len;
        const floatx4 q = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + (inside ? 4u * lane : 0u)));
        v[0][0] = inside ? q.x : 0.0f; v[0][1] = inside ? q.y : 0.0f;
        v[0][2] = inside ? q.z : 0.0f; v[0][3] = inside ? q.w : 0.0f;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[0][k] = 4u * lane + k < len ? g[4u * lane + k] : 0.0f;
    }
    if (clip > 0.0f) clip_small_buckets<NB, FULL>(v[0], len, clip, lane);
    // largest magnitude of the lane's bucket (padding holds 0)
    uint32_t mag = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) mag = umax32(mag, __float_as_uint(v[0][k]) & 0x7FFFFFFFu);
    mag = umax32(mag, dpp_u32<kDppXor1>(mag));
    mag = umax32(mag, dpp_u32<kDppXor2>(mag));
    mag = umax32(mag, dpp_u32<kDppHalfMirror>(mag));
    mag = umax32(mag, dpp_u32<kDppMirror>(mag));  // the 16 lanes of a row
    if constexpr (G == 32u) mag = umax32(mag, lane_xor<16>(mag, lane));
    float lv[S];
    const double largest = (double)__uint_as_float(mag);
#pragma unroll
    for (int k = 0; k < S; ++k) lv[k] = (float)(largest * (double)(2 * k - (S - 1)) / (double)(S - 1));
    const uint32_t q = lane / G;  // bucket of this lane inside the wavefront
    if (lane % G == 0u && (FULL || q * D < len)) {
#pragma unroll
        for (int k = 0; k < S; ++k) levels[(size_t)(first_bucket + q) * S + k] = lv[k];
    }
    orq_encode<1, S, BITS, FULL>(v, lv, len, begin, seed, index_offset, codes32);
}

template <int S, int BITS, int NB>
__global__ __launch_bounds__(4 * kWave) void even_small_kernel(const float* __restrict__ grad, size_t n, float clip,
                                                               uint64_t seed, uint64_t index_offset,
                                                               float* __restrict__ levels, uint32_t* __restrict__ codes32)
{
    const size_t span = (size_t)blockIdx.x * 4u + (threadIdx.x >> 6);  // 256 elements each
    const size_t begin = span * 256u;
    if (begin >= n) return;
    const size_t rest = n - begin;
    const uint32_t first_bucket = (uint32_t)(span * NB);
    if (rest >= 256u)
        even_small_span<S, BITS, NB, true>(grad + begin, 256u, begin, first_bucket, clip, seed, index_offset, levels, codes32);
    else
        even_small_span<S, BITS, NB, false>(grad + begin, (uint32_t)rest, begin, first_bucket, clip, seed, index_offset, levels,
                                            codes32);
}

// ----------------------------------------------------------------------------------------------
// ORQ, Linear-s and BinGrad-pb for buckets of 64 or 128 elements, NB = 4 or 2 whole buckets per wavefront in the
// layout of even_small_span.  A bucket this small is not grouped into bins: its 4 G keys (G = 64 / NB lanes, 4 registers
// each) are sorted in registers by a bitonic network whose every compare-exchange is ascending -- the first step of
// a merge pairs element e with e ^ (run length - 1), i.e. reverses the second run -- so that no step needs a
// direction.  Element e = 4 * (lane inside the bucket) + register.  The levels are then order statistics fetched
// from the sorted registers: the extremes, and either Linear-s's ranks or the elements of the ranks that the optimal
// condition asks for.  With three levels there is one solve, between the extremes, and it reads the bucket's total
// alone (sweeps repeat it unchanged); with more, every lane keeps the level records of its bucket and the solves of
// all buckets of the wavefront run side by side.  Two levels are the extremes and need no sort.  BinGrad-pb's level
// is the positive value at the sign change of its condition, which every element evaluates for itself from the
// exclusive fp64 prefix of the sorted values.
// ----------------------------------------------------------------------------------------------
__device__ __forceinline__ void sort_pair(uint32_t& a, uint32_t& b)
{
    const uint32_t mn = umin32(a, b), mx = umax32(a, b);
    a = mn;
    b = mx;
}

// The steps of a merge that pair lanes J apart (J = M / 2 ... 1), register by register.
template <int J>
__device__ __forceinline__ void row_sort_across(uint32_t (&x)[4], uint32_t lane)
{
    if constexpr (J >= 1) {
        const uint32_t bound = upper_lanes<J>(lane);
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = smaller_or_larger(x[r], lane_xor<J>(x[r], lane), bound);
        row_sort_across<J / 2>(x, lane);
    }
}

// Merges the sorted runs of 4 M elements (M lanes) pairwise into sorted runs of 8 M, and so on up to 4 G.
template <int M, int G>
__device__ __forceinline__ void row_sort_merge(uint32_t (&x)[4], uint32_t lane)
{
    if constexpr (2 * M <= G) {
        const uint32_t bound = upper_lanes<M>(lane);
        uint32_t y[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] = lane_reverse<M>(x[3 - r], lane);
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = smaller_or_larger(x[r], y[r], bound);
        row_sort_across<M / 2>(x, lane);
        sort_pair(x[0], x[2]);
        sort_pair(x[1], x[3]);
        sort_pair(x[0], x[1]);
        sort_pair(x[2], x[3]);
        row_sort_merge<2 * M, G>(x, lane);
    }
}

// Ascending sort of the 4 G keys of every group of G lanes (G = 16 or 32).
template <int G>
__device__ __forceinline__ void row_sort(uint32_t (&x)[4], uint32_t lane)
{
    sort_pair(x[0], x[1]);  // runs of 2
    sort_pair(x[2], x[3]);
    sort_pair(x[0], x[3]);  // runs of 4
    sort_pair(x[1], x[2]);
    sort_pair(x[0], x[1]);
    sort_pair(x[2], x[3]);
    row_sort_merge<1, G>(x, lane);
}

// Element `index` (0-based, the same in all lanes of the group) of the sorted group whose first lane is `first_lane`.
__device__ __forceinline__ uint32_t row_fetch(const uint32_t (&x)[4], uint32_t index, uint32_t first_lane)
{
    const uint32_t lo = (index & 1u) ? x[1] : x[0];
    const uint32_t hi = (index & 1u) ? x[3] : x[2];
    const uint32_t mine = (index & 2u) ? hi : lo;
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)((first_lane + (index >> 2)) << 2), (int)mine);
}

// Sum over the group of G lanes, in every lane of the group.
template <int G>
__device__ __forceinline__ double row_sum_f64(double x, uint32_t lane)
{
    x += dpp_f64<kDppXor1>(x);
    x += dpp_f64<kDppXor2>(x);
    x += dpp_f64<kDppHalfMirror>(x);
    x += dpp_f64<kDppMirror>(x);
    if constexpr (G == 32) {
        const uint64_t u = (uint64_t)__double_as_longlong(x);
        const uint32_t lo = lane_xor<16>((uint32_t)u, lane), hi = lane_xor<16>((uint32_t)(u >> 32), lane);
        x += __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
    }
    return x;
}

template <int G>
__device__ __forceinline__ uint32_t row_sum_u32(uint32_t x, uint32_t lane)
{
    x += dpp_u32<kDppXor1>(x);
    x += dpp_u32<kDppXor2>(x);
    x += dpp_u32<kDppHalfMirror>(x);
    x += dpp_u32<kDppMirror>(x);
    if constexpr (G == 32) x += lane_xor<16>(x, lane);
    return x;
}

// Minimum over the group of G lanes, in every lane of the group.
template <int G>
__device__ __forceinline__ uint32_t row_min_u32(uint32_t x, uint32_t lane)
{
    x = umin32(x, dpp_u32<kDppXor1>(x));
    x = umin32(x, dpp_u32<kDppXor2>(x));
    x = umin32(x, dpp_u32<kDppHalfMirror>(x));
    x = umin32(x, dpp_u32<kDppMirror>(x));
    if constexpr (G == 32) x = umin32(x, lane_xor<16>(x, lane));
    return x;
}

template <int G>
__device__ __forceinline__ uint32_t row_max_u32(uint32_t x, uint32_t lane)
{
    return ~row_min_u32<G>(~x, lane);
}

// Inclusive scan over the lanes of every group of G lanes (G = 16 or 32).
template <int G>
__device__ __forceinline__ double row_inclusive_scan_f64(double x)
{
    x += dpp_or_zero_f64<kDppRowShr1, 0xF>(x);
    x += dpp_or_zero_f64<kDppRowShr2, 0xF>(x);
    x += dpp_or_zero_f64<kDppRowShr4, 0xF>(x);
    x += dpp_or_zero_f64<kDppRowShr8, 0xF>(x);
    if constexpr (G == 32) x += dpp_or_zero_f64<kDppRowBcast15, 0xA>(x);
    return x;
}

__device__ __forceinline__ double lane_fetch_f64(double x, uint32_t from_lane)
{
    const uint64_t u = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(from_lane << 2), (int)(uint32_t)u);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(from_lane << 2), (int)(uint32_t)(u >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// row_fetch for the fp64 sums that sit beside the sorted keys.
__device__ __forceinline__ double row_fetch_f64(const double (&x)[4], uint32_t index, uint32_t first_lane)
{
    const double lo = (index & 1u) ? x[1] : x[0];
    const double hi = (index & 1u) ? x[3] : x[2];
    return lane_fetch_f64((index & 2u) ? hi : lo, first_lane + (index >> 2));
}

// Per level, in the registers of every lane of the bucket's group: what OrqLds keeps per level.
template <int S>
struct RowLevels {
    float value[S];
    uint32_t count_lt[S], count_le[S], rank[S];
    double sum_lt[S], sum_le[S];
};

template <int S, int BITS, int NB, bool FULL, int RULE>
__device__ __forceinline__ void sorted_small_span(const float* __restrict__ g, uint32_t len, size_t begin, uint32_t first_bucket,
                                                  uint32_t sweeps, float clip, uint64_t seed, uint64_t index_offset,
                                                  float* __restrict__ levels, uint32_t* __restrict__ codes32,
                                                  unsigned long long* exact_limbs)
{
    static_assert(RULE == kLinear || RULE == kOptimal || (RULE == kPb && S == 2), "rules that read order statistics");
    constexpr uint32_t G = 64u / NB;  // lanes per bucket
    constexpr uint32_t D = 256u / NB;  // elements per bucket
    const uint32_t lane = threadIdx.x & 63u;
    float v[1][4];
    if (FULL || len % 4u == 0u) {
        const bool inside = FULL || 4u * lane < len;
        const floatx4 q = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + (inside ? 4u * lane : 0u)));
        v[0][0] = inside ? q.x : 0.0f; v[0][1] = inside ? q.y : 0.0f;
        v[0][2] = inside ? q.z : 0.0f; v[0][3] = inside ? q.w : 0.0f;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[0][k] = 4u * lane + k < len ? g[4u * lane + k] : 0.0f;
    }
    if (clip > 0.0f) clip_small_buckets<NB, FULL>(v[0], len, clip, lane);
    const uint32_t q = lane / G;  // bucket of this lane inside the wavefront
    uint32_t count = D;           // elements of that bucket (the gradient may end inside or before it)
    if constexpr (!FULL) count = q * D < len ? (len - q * D < D ? len - q * D : D) : 0u;

    uint32_t x[4];
    double part = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const bool valid = FULL || 4u * lane + k < len;
        const float value = v[0][k] + 0.0f;  // -0 -> +0
        x[k] = valid ? float_to_key(value) : 0xFFFFFFFFu;  // padding sorts behind every value
        if constexpr (RULE == kOptimal && S == 3) part += valid ? (double)value : 0.0;
    }
    float lv[S];
    if constexpr (RULE == kPb) {
        // b_1 minimises |b * #{v > 0} - sum_{v >= b} v| over the bucket's positive values.  Every element evaluates the
        // difference for its own value in its own lane (the sum of the smaller elements is its entry of the exclusive
        // prefix if it is the first of its value); the difference grows with b, so the minimiser is the first value
        // where it is not negative, or the distinct value just below.
        row_sort<(int)G>(x, lane);
        const uint32_t first_lane = lane & ~(G - 1u);
        const uint32_t l4 = 4u * (lane & (G - 1u));
        constexpr uint32_t kZeroKey = 0x80000000u;  // key of +0
        double before[4], run = 0.0;
        uint32_t not_positive = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            before[r] = run;
            run += l4 + r < count ? (double)key_to_float(x[r]) : 0.0;
            not_positive += x[r] <= kZeroKey ? 1u : 0u;
        }
        const double incl = row_inclusive_scan_f64<(int)G>(run);
        const double lanes_before = incl - run;
        const double total = lane_fetch_f64(incl, first_lane + G - 1u);
        not_positive = row_sum_u32<(int)G>(not_positive, lane);
        const uint32_t positives = count - (not_positive < count ? not_positive : count);
        // last key of the lane in front (none for the first lane of the group: key 0 lies below every positive key)
        const uint32_t front = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((lane - 1u) << 2), (int)x[3]);
        double gap[4];
        uint32_t first_ok = 0xFFFFu, last_first = 0u;  // element indices inside the bucket
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            before[r] += lanes_before;
            const uint32_t previous = r > 0 ? x[r > 0 ? r - 1 : 0] : (lane == first_lane ? 0u : front);
            const bool candidate = l4 + r < count && x[r] > kZeroKey && x[r] != previous;  // first of a positive value
            gap[r] = (double)key_to_float(x[r]) * (double)positives - (total - before[r]);
            if (candidate && gap[r] >= 0.0) first_ok = umin32(first_ok, l4 + r);
            if (candidate) last_first = umax32(last_first, l4 + r);
        }
        first_ok = row_min_u32<(int)G>(first_ok, lane);
        last_first = row_max_u32<(int)G>(last_first, lane);
        // (the largest value's difference is >= 0 but for rounding: if no element says so, it is the answer)
        const uint32_t at = first_ok != 0xFFFFu ? first_ok : last_first;
        const float up = key_to_float(row_fetch(x, at, first_lane));
        const double gap_up = row_fetch_f64(gap, at, first_lane);
        // the distinct value just below, which counts if it is positive: its difference sits where that value begins
        const uint32_t down_key = row_fetch(x, at > 0u ? at - 1u : 0u, first_lane);
        uint32_t down_at = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) down_at += x[r] < down_key ? 1u : 0u;
        down_at = row_sum_u32<(int)G>(down_at, lane);
        const double gap_down = row_fetch_f64(gap, down_at, first_lane);
        const bool take_down = at > not_positive && fabs(gap_down) <= fabs(gap_up);  // ties take the smaller value
        const float pb_level = positives > 0u ? (take_down ? key_to_float(down_key) : up) : 0.0f;
        lv[0] = -pb_level;
        lv[1] = pb_level;
    } else if constexpr (S == 2) {
        // two levels are the extremes: no sort, two reductions over the group
        uint32_t low = umin32(umin32(x[0], x[1]), umin32(x[2], x[3])), high = 0u;
#pragma unroll
        for (int k = 0; k < 4; ++k) high = umax32(high, x[k] == 0xFFFFFFFFu ? 0u : x[k]);
        lv[0] = key_to_float(row_min_u32<(int)G>(low, lane));
        lv[1] = key_to_float(row_max_u32<(int)G>(high, lane));
    } else {
        row_sort<(int)G>(x, lane);

        const uint32_t first_lane = lane & ~(G - 1u);
        const uint32_t last = count > 0u ? count - 1u : 0u;
        lv[0] = key_to_float(row_fetch(x, 0u, first_lane));
        lv[S - 1] = key_to_float(row_fetch(x, last, first_lane));
        // Whether the fp64 sums of this lane's bucket are exact (floor_t_from_sums: no non-zero element more than
        // safe_binades(D) binades below the largest magnitude), and the bucket's workspace for exact_floor_t.
        double error_bound = 0.0;
        unsigned long long* limb = exact_limbs + ((threadIdx.x >> 6) * NB + q) * kExactLimbs;
        if constexpr (RULE == kOptimal) {
            const uint32_t mag_max = umax32(__float_as_uint(lv[0]) & 0x7FFFFFFFu, __float_as_uint(lv[S - 1]) & 0x7FFFFFFFu);
            const uint32_t biased = mag_max >> 23;
            const uint32_t mag_safe = biased > safe_binades(D) ? (biased - safe_binades(D)) << 23 : 0u;
            uint32_t tiny = 0u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t magnitude = __float_as_uint(key_to_float(x[i])) & 0x7FFFFFFFu;
                if (4u * (lane & (G - 1u)) + i < count && magnitude != 0u && magnitude < mag_safe) tiny = 1u;
            }
            if (row_max_u32<(int)G>(tiny, lane) != 0u) error_bound = sum_error_bound_of(mag_max, D);
        }
        if constexpr (RULE == kLinear) {
#pragma unroll
            for (int k = 1; k + 1 < S; ++k)
                lv[k] = key_to_float(row_fetch(x, ((uint32_t)k * last) / (uint32_t)(S - 1), first_lane));
        } else if constexpr (S > 3) {
            // The solves of orq_solve_levels, every lane keeping the records of its own bucket.  What a solve needs
            // around a picked element comes from the sorted registers: the counts of smaller and of not larger keys
            // (summed over the group), and the sum of the smaller ones, an entry of the exclusive fp64 prefix.
            const uint32_t l4 = 4u * (lane & (G - 1u));
            double before[4];  // sum of the sorted elements in front of element 4 l + r
            double total;
            {
                double run = 0.0, mine[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    mine[r] = run;
                    run += l4 + r < count ? (double)key_to_float(x[r]) : 0.0;
                }
                const double incl = row_inclusive_scan_f64<(int)G>(run);
                const double lanes_before = incl - run;
#pragma unroll
                for (int r = 0; r < 4; ++r) before[r] = lanes_before + mine[r];
                total = lane_fetch_f64(incl, first_lane + G - 1u);
            }
            RowLevels<S> st;
#pragma unroll
            for (int k = 0; k < S; ++k) {
                st.value[k] = k == S - 1 ? lv[S - 1] : lv[0];
                st.count_lt[k] = k == S - 1 ? count : 0u;
                st.count_le[k] = k == S - 1 ? count : 0u;
                st.sum_lt[k] = k == S - 1 ? total : 0.0;
                st.sum_le[k] = k == S - 1 ? total : 0.0;
                st.rank[k] = 0u;
            }
            const uint32_t count_or_one = count > 0u ? count : 1u;
            auto solve = [&](auto kc, auto lc, auto rc) {
                constexpr int k = decltype(kc)::value, l = decltype(lc)::value, r = decltype(rc)::value;
                const float L = st.value[l], R = st.value[r];
                const uint32_t cnt_lt_L = st.count_lt[l], cnt_le_R = st.count_le[r];
                const double sum_lt_L = st.sum_lt[l], sum_le_R = st.sum_le[r];
                const bool ordered = L < R;
                // S = sum_{L<=v<=R} (v - L),  T = S / (R - L),  level = element of rank #{v<=R} - floor(T)
                const uint32_t count_in = cnt_le_R - cnt_lt_L;
                const double Ssum = (sum_le_R - sum_lt_L) - (double)L * (double)count_in;
                const double width = (double)R - (double)L;
                double m;  // not used when L == R
                const bool decided = floor_t_from_sums(Ssum, width, error_bound, m);
                if (ordered && !decided) {
                    // (as in orq_solve_one: exact sums where the fp64 sums do not decide; only the lanes of such buckets)
                    m = (double)exact_floor_t_registers(limb, lane & (G - 1u), L, R, count_in, (uint32_t)m, key_to_float(x[0]),
                                                        key_to_float(x[1]), key_to_float(x[2]), key_to_float(x[3]),
                                                        count > l4 ? count - l4 : 0u);
                }
                const bool whole = m >= (double)cnt_le_R;
                uint32_t rank = whole ? 1u : cnt_le_R - (uint32_t)(whole ? 0.0 : m);
                rank = rank < 1u ? 1u : (rank > count_or_one ? count_or_one : rank);
                const bool same = ordered && rank == st.rank[k];  // same element as last time
                if (__ballot(!same) == 0) return;
                const uint32_t key = row_fetch(x, rank - 1u, first_lane);
                const float picked = key_to_float(key);
                uint32_t below = 0, not_above = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    below += x[i] < key ? 1u : 0u;
                    not_above += x[i] <= key ? 1u : 0u;
                }
                const uint32_t both = row_sum_u32<(int)G>(below | (not_above << 16), lane);  // two counts of at most 128
                const uint32_t c_lt = both & 0xFFFFu, c_le = both >> 16;
                const double s_lt = row_fetch_f64(before, c_lt, first_lane);
                const double s_le = s_lt + (double)(c_le - c_lt) * (double)picked;
                const bool copy_left = !ordered || picked < L;  // the level coincides with the left end
                const float new_value = copy_left ? L : picked;
                const uint32_t new_count_lt = copy_left ? cnt_lt_L : c_lt;
                const double new_sum_lt = copy_left ? sum_lt_L : s_lt;
                const uint32_t new_count_le = copy_left ? (ordered ? st.count_le[l] : cnt_le_R) : c_le;
                const double new_sum_le = copy_left ? (ordered ? st.sum_le[l] : sum_le_R) : s_le;
                const uint32_t new_rank = copy_left ? 0u : rank;
                st.value[k] = same ? st.value[k] : new_value;
                st.count_lt[k] = same ? st.count_lt[k] : new_count_lt;
                st.sum_lt[k] = same ? st.sum_lt[k] : new_sum_lt;
                st.count_le[k] = same ? st.count_le[k] : new_count_le;
                st.sum_le[k] = same ? st.sum_le[k] : new_sum_le;
                st.rank[k] = same ? st.rank[k] : new_rank;
            };
            for_greedy_steps<S, 0>(solve);
            for (uint32_t sweep = 0; sweep < sweeps; ++sweep) for_sweep_levels<S, 1>(solve);
#pragma unroll
            for (int k = 1; k + 1 < S; ++k) lv[k] = st.value[k];
        } else {
            // S = sum (v - L) over the bucket, T = S / (R - L), level = element of rank #{v <= R} - floor(T)
            const double total = row_sum_f64<(int)G>(part, lane);
            const float L = lv[0], R = lv[2];
            const double Ssum = total - (double)L * (double)count, width = (double)R - (double)L;
            double m;  // not used when L == R
            const bool decided = floor_t_from_sums(Ssum, width, error_bound, m);
            if (L < R && !decided) {
                // (as in orq_solve_one: exact sums where the fp64 sums do not decide; only the lanes of such buckets)
                const uint32_t mine = 4u * (lane & (G - 1u));
                m = (double)exact_floor_t_registers(limb, lane & (G - 1u), L, R, count, (uint32_t)m, key_to_float(x[0]),
                                                    key_to_float(x[1]), key_to_float(x[2]), key_to_float(x[3]),
                                                    count > mine ? count - mine : 0u);
            }
            if (m > (double)count) m = (double)count;
            uint32_t rank = m >= (double)count ? 1u : count - (uint32_t)m;
            rank = rank < 1u ? 1u : rank;
            const float picked = key_to_float(row_fetch(x, rank - 1u, first_lane));
            lv[1] = (L < R && !(picked < L)) ? picked : L;
        }
    }
    if (lane % G == 0u && (FULL || q * D < len)) {
#pragma unroll
        for (int k = 0; k < S; ++k) levels[(size_t)(first_bucket + q) * S + k] = lv[k];
    }
    orq_encode<1, S, BITS, FULL>(v, lv, len, begin, seed, index_offset, codes32);
}

template <int S, int BITS, int NB, int RULE>
__global__ __launch_bounds__(4 * kWave) void sorted_small_kernel(const float* __restrict__ grad, size_t n, uint32_t sweeps,
                                                                 float clip, uint64_t seed, uint64_t index_offset,
                                                                 float* __restrict__ levels, uint32_t* __restrict__ codes32)
{
    __shared__ unsigned long long exact_limbs[4 * NB * kExactLimbs];  // workspace of exact_floor_t per wavefront and bucket
    const size_t span = (size_t)blockIdx.x * 4u + (threadIdx.x >> 6);  // 256 elements each
    const size_t begin = span * 256u;
    if (begin >= n) return;
    const size_t rest = n - begin;
    const uint32_t first_bucket = (uint32_t)(span * NB);
    if (rest >= 256u)
        sorted_small_span<S, BITS, NB, true, RULE>(grad + begin, 256u, begin, first_bucket, sweeps, clip, seed, index_offset,
                                                   levels, codes32, exact_limbs);
    else
        sorted_small_span<S, BITS, NB, false, RULE>(grad + begin, (uint32_t)rest, begin, first_bucket, sweeps, clip, seed,
                                                    index_offset, levels, codes32, exact_limbs);
}

// ----------------------------------------------------------------------------------------------
// ORQ and the other random-rounding rules with W = 2, 4 or 8 wavefronts of a workgroup owning one bucket (up
// to 32768 elements), wavefront w holding bucket elements [256 C w, 256 C (w + 1)) in the register layout of
// orq_bucket.  All of them build the grouping of the whole bucket in LDS (histogram, bin
// starts, scatter, fp64 block prefix) with workgroup barriers in between; the level solves are serial and run
// on wavefront 0 alone; then every wavefront encodes its own elements.
// ----------------------------------------------------------------------------------------------
template <int W, int C>
struct OrqTeamLds {
    static constexpr int D = 256 * C * W;
    // bins, and magnitude bits dropped by the bin index (what is kept: the exponent and 3 .. 6 mantissa bits)
    static constexpr int B = D >= 16384 ? 2048 : D >= 8192 ? 1024 : D >= 4096 ? 512 : 256;
    static constexpr int SHIFT = D >= 16384 ? 17 : D >= 8192 ? 18 : D >= 4096 ? 19 : 20;
    static constexpr int BLOCK = 4 * C;  // positions per entry of the fp64 block prefix: one entry per thread
    uint32_t grouped[D + D / 64];
    uint32_t bin_start[B + 4];
    double block_prefix[64 * W];  // fp64 sum of all positions before block i of BLOCK positions
    double lvl_sum_lt[10];
    double lvl_sum_le[10];
    float lvl_value[10];
    uint32_t lvl_count_lt[10];
    uint32_t lvl_count_le[10];
    uint32_t lvl_rank[10];
    double sum_error_bound;  // 0 when every fp64 sum of the bucket is exact (see floor_t_from_sums)
    uint32_t tiny_flag;      // set by any thread that met an element too small for exact sums
    unsigned long long exact_limb[2][kExactLimbs];  // workspace of exact_floor_t, one per solving wavefront
    TeamSlot slots[2][W];
};

template <int W, int C, int S, int BITS, bool FULL, int RULE>
__device__ __forceinline__ void orq_team_bucket(OrqTeamLds<W, C>& lds, const float* __restrict__ g, uint32_t len,
                                                size_t begin, uint32_t bucket, uint32_t sweeps, float clip,
                                                uint64_t seed, uint64_t index_offset, float* __restrict__ levels,
                                                uint32_t* __restrict__ codes32)
{
    constexpr uint32_t PER_WAVE = 256u * C;  // bucket elements per wavefront
    constexpr int B = OrqTeamLds<W, C>::B;
    constexpr int HALF = B / 2;
    constexpr int SHIFT = OrqTeamLds<W, C>::SHIFT;
    constexpr bool PB = RULE == kPb;
    constexpr uint32_t THREADS = 64u * W;
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = uniform_u32(tid >> 6);
    const uint32_t first = PER_WAVE * wave;  // first bucket element of this wavefront
    const uint32_t my_len = len > first ? (len - first < PER_WAVE ? len - first : PER_WAVE) : 0u;
    WaveTeam<W> team{lds.slots, wave, 0u};

    float v[C][4];
    if (FULL) {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const floatx4 q =
                __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + first + 256 * c + 4 * lane));
            v[c][0] = q.x; v[c][1] = q.y; v[c][2] = q.z; v[c][3] = q.w;
        }
    } else if (len % 4u == 0u) {
        // whole 16-byte loads; the lanes past the end read the bucket's first elements and drop them
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const uint32_t e = 256u * c + 4u * lane;
            const bool inside = e < my_len;
            const floatx4 q = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + (inside ? first + e : 0u)));
            v[c][0] = inside ? q.x : 0.0f; v[c][1] = inside ? q.y : 0.0f;
            v[c][2] = inside ? q.z : 0.0f; v[c][3] = inside ? q.w : 0.0f;
        }
    } else {
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t e = 256u * c + 4u * lane + k;
                v[c][k] = e < my_len ? g[first + e] : 0.0f;
            }
    }

    if (clip > 0.0f) {  // the same for every thread of the grid
        float(&flat)[4 * C] = reinterpret_cast<float(&)[4 * C]>(v);
        clip_in_registers<4 * C>(
            flat, len, clip, [&](int j) { return FULL || (64u * (j & ~3) + 4u * lane + (j & 3) < my_len); },
            [&](double x) { return team.sum(wave_sum(x)); });
    }

    // ---- extremes of the whole bucket ----------------------------------------------------------------
    float lane_min = __uint_as_float(0x7F800000u), lane_max = __uint_as_float(0xFF800000u);
    uint32_t lane_zeros = 0;
    for_each_chunk<C, FULL>(my_len, [&](int c, auto all) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < my_len);
            lane_min = fminf(lane_min, valid ? v[c][k] : __uint_as_float(0x7F800000u));
            lane_max = fmaxf(lane_max, valid ? v[c][k] : __uint_as_float(0xFF800000u));
            if constexpr (PB) lane_zeros += (valid && v[c][k] == 0.0f) ? 1u : 0u;
        }
    });
    float bucket_min = wave_min(lane_min), bucket_max = wave_max(lane_max);
    uint32_t zeros = PB ? wave_sum_u32(lane_zeros) : 0u;
    {
        const TeamSlot* s = team.exchange((double)zeros, __float_as_uint(bucket_min), __float_as_uint(bucket_max));
        double z = 0.0;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            bucket_min = fminf(bucket_min, __uint_as_float(s[w].a));
            bucket_max = fmaxf(bucket_max, __uint_as_float(s[w].b));
            z += s[w].sum;
        }
        zeros = (uint32_t)z;
    }
    bucket_min += 0.0f;  // -0 -> +0
    bucket_max += 0.0f;
    const uint32_t key_min = float_to_key(bucket_min), key_max = float_to_key(bucket_max);
    const uint32_t mag_max = umax32(__float_as_uint(bucket_min) & 0x7FFFFFFFu, __float_as_uint(bucket_max) & 0x7FFFFFFFu);
    const uint32_t t_max = mag_max >> SHIFT;
    const uint32_t t_low = __builtin_elementwise_sub_sat(t_max, (uint32_t)(HALF - 1));

    if constexpr ((S > 2 && RULE != kEven) || PB) {
        // ---- histogram: the returning LDS add hands every element its position inside its bin ------------
        for (uint32_t i = tid; i < (uint32_t)B; i += THREADS) lds.bin_start[i] = 0u;
        if (tid == 0u) lds.tiny_flag = 0u;
        __syncthreads();
        uint32_t slot[C][4];  // bin | position inside the bin << 16 (pack_slot)
        const float zero = opaque_zero();
        for_each_chunk<C, FULL>(my_len, [&](int c, auto all) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < my_len);
                const uint32_t bin = value_bin<HALF, SHIFT>(v[c][k] + zero, t_low);
                slot[c][k] = 0u;
                if (valid) slot[c][k] = pack_slot(atomicAdd(&lds.bin_start[bin], 1u), bin, (uint32_t)HALF);
            }
        });
        __syncthreads();

        // ---- exclusive prefix over the bin counts (wavefront 0; lane l owns bins l*PER .. l*PER+PER-1) ------
        if (wave == 0u) {
            constexpr uint32_t PER = B / 64;
            uint32_t tot = 0;
            for (uint32_t i = 0; i < PER; ++i) tot += lds.bin_start[lane * PER + i];
            uint32_t run = wave_inclusive_scan_u32(tot) - tot;
            for (uint32_t i = 0; i < PER; ++i) {
                const uint32_t count = lds.bin_start[lane * PER + i];
                lds.bin_start[lane * PER + i] = run;
                run += count;
            }
            if (lane == 63u) lds.bin_start[B] = run;  // = len
        }
        __syncthreads();

        // ---- scatter the values into their bins (bin starts of a group of elements read before its writes) ------
        constexpr int GROUP = C < 4 ? C : 4;
        auto scatter_group = [&](int c0, auto all) {
#pragma unroll
            for (int c = c0; c < c0 + GROUP; ++c)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < my_len);
                    if (valid) slot[c][k] = slot_bin_start(&lds.bin_start[HALF], slot[c][k]) + (slot[c][k] >> 16);
                }
#pragma unroll
            for (int c = c0; c < c0 + GROUP; ++c)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < my_len);
                    if (valid)
                        *reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(lds.grouped) + skewed_byte_offset(slot[c][k])) =
                            __float_as_uint(v[c][k]);
                }
        };
#pragma unroll
        for (int c0 = 0; c0 < C; c0 += GROUP) {
            if (FULL || 256u * (uint32_t)(c0 + GROUP) <= my_len) scatter_group(c0, std::true_type{});
            else if (256u * (uint32_t)c0 < my_len) scatter_group(c0, std::false_type{});
        }
        __syncthreads();

        // ---- may the fp64 sums round?  (all threads look; combined before the records below are written) ----
        if constexpr (RULE == kOptimal && S > 2) {
            if (any_tiny_element<HALF, SHIFT>(lds, (uint32_t)OrqTeamLds<W, C>::D, mag_max, t_low, tid, THREADS))
                atomicOr(&lds.tiny_flag, 1u);
        }

        // ---- fp64 prefix of the grouped values per block of 4C positions (thread t sums block t) ----------
        // Skipped, but for the bucket's total, by the rules whose solves read no picked level's counts or sums.
        constexpr bool SUMS = (RULE == kOptimal && S > 3) || PB;
        {
            double total = 0.0;
            if constexpr (SUMS) {
                constexpr uint32_t BLOCK = OrqTeamLds<W, C>::BLOCK;
                double part = 0.0;
                for (uint32_t i = 0; i < BLOCK; ++i) {
                    const uint32_t position = tid * BLOCK + i;
                    const float x = position < len ? __uint_as_float(lds.grouped[skewed(position)]) : 0.0f;
                    part += (double)x;
                }
                const double incl = wave_inclusive_scan_f64(part);
                const TeamSlot* s = team.exchange(readlane_f64(incl, 63), 0u, 0u);
                double before = 0.0;
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    if ((uint32_t)w < wave) before += s[w].sum;
                    total += s[w].sum;
                }
                lds.block_prefix[tid] = before + (incl - part);
            } else if constexpr (RULE == kOptimal) {
                double part = 0.0;
                for_each_chunk<C, FULL>(my_len, [&](int c, auto all) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const bool valid = decltype(all)::value || (256u * c + 4u * lane + k < my_len);
                        part += valid ? (double)v[c][k] : 0.0;
                    }
                });
                const TeamSlot* s = team.exchange(wave_sum(part), 0u, 0u);
#pragma unroll
                for (int w = 0; w < W; ++w) total += s[w].sum;
            }
            if (tid == 0u) {
                // the bottom level is only ever the left end of a solve, the top level the right end
                lds.lvl_count_lt[0] = 0u;
                lds.lvl_sum_lt[0] = 0.0;
                lds.lvl_count_le[0] = 0u;
                lds.lvl_sum_le[0] = 0.0;
                lds.lvl_count_le[S - 1] = len;
                lds.lvl_sum_le[S - 1] = total;
                lds.lvl_count_lt[S - 1] = len;
                lds.lvl_sum_lt[S - 1] = total;
                // (every thread's look at the small elements lies before the barrier of the exchange above)
                if constexpr (RULE == kOptimal && S > 2)
                    lds.sum_error_bound = lds.tiny_flag != 0u ? sum_error_bound_of(mag_max, (uint32_t)OrqTeamLds<W, C>::D) : 0.0;
            }
            if (tid < (uint32_t)S) {
                lds.lvl_value[tid] = key_to_float(tid == (uint32_t)(S - 1) ? key_max : key_min);
                lds.lvl_rank[tid] = 0u;
            }
        }
        __syncthreads();

        if constexpr (RULE == kOptimal && S > 2) {
            // ---- the level solves, spread over the first two wavefronts ------------------------------------------
            orq_team_solve<S>(lds, [&](uint32_t rank) { return pick_rank_by_lookup<SUMS>(lds, rank, lane); }, wave, len, sweeps,
                              lane);
        } else {
            // ---- the other rules' solves are serial: wavefront 0 ---------------------------------------------------
            if (wave == 0u) {
                const float pb_level = orq_solve_levels<S, RULE>(
                    lds, [&](uint32_t rank) { return pick_rank_by_lookup<SUMS>(lds, rank, lane); },
                    [&](uint32_t bin) { return __uint_as_float((t_low + (bin - (uint32_t)HALF)) << SHIFT); }, len, zeros, sweeps,
                    lane);
                if (PB && lane == 0u) {
                    lds.lvl_value[0] = -pb_level;
                    lds.lvl_value[S - 1] = pb_level;
                }
            }
            __syncthreads();
        }
    }

    float lv[S];
    if constexpr (RULE == kEven) {
        const double largest = (double)__uint_as_float(mag_max);
#pragma unroll
        for (int k = 0; k < S; ++k) lv[k] = (float)(largest * (double)(2 * k - (S - 1)) / (double)(S - 1));
    } else if constexpr (S == 2 && !PB) {
        lv[0] = key_to_float(key_min);
        lv[1] = key_to_float(key_max);
    } else {
#pragma unroll
        for (int k = 0; k < S; ++k) lv[k] = lds.lvl_value[k];
    }
    if (tid == 0u) {
#pragma unroll
        for (int k = 0; k < S; ++k) levels[(size_t)bucket * S + k] = lv[k];
    }

    orq_encode<C, S, BITS, FULL>(v, lv, my_len, begin + first, seed, index_offset, codes32);
}

// C = 8 (2048 elements per wavefront): the LDS of a CU holds the buckets of 16 wavefronts, so the kernel is held to the
// 128 registers that let four wavefronts share a SIMD (one register more costs d = 8192 a quarter of its wavefronts);
// BinGrad-pb would spill.
template <int W, int C, int S, int BITS, int RULE>
__global__ __launch_bounds__(W* kWave) __attribute__((amdgpu_waves_per_eu(C == 8 && RULE != kPb ? 4 : 1))) void orq_team_kernel(const float* __restrict__ grad, size_t n,
                                                            uint32_t bucket_size, uint32_t sweeps, float clip,
                                                            uint32_t num_buckets, uint64_t seed, uint64_t index_offset,
                                                            float* __restrict__ levels, uint32_t* __restrict__ codes32)
{
    __shared__ OrqTeamLds<W, C> lds;
    const uint32_t bucket = blockIdx.x;
    if (bucket >= num_buckets) return;
    const size_t begin = (size_t)bucket * bucket_size;
    const size_t rest = n - begin;
    const uint32_t len = rest < bucket_size ? (uint32_t)rest : bucket_size;
    if (len == (uint32_t)OrqTeamLds<W, C>::D)
        orq_team_bucket<W, C, S, BITS, true, RULE>(lds, grad + begin, len, begin, bucket, sweeps, clip, seed, index_offset, levels, codes32);
    else
        orq_team_bucket<W, C, S, BITS, false, RULE>(lds, grad + begin, len, begin, bucket, sweeps, clip, seed, index_offset, levels, codes32);
}

// ----------------------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------------------
template <int C, int S, int BITS, int RULE = kOptimal>
void launch_orq(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes, hipStream_t st)
{
    if (p->clip_factor > 0.0f)
        launch_kernel((orq_quantize_kernel<C, S, BITS, true, RULE>), dim3(nb), dim3(kWave), st, g, n, p->bucket_size,
                           p->level_iters, p->clip_factor, nb, p->seed, p->index_offset, lv,
                           static_cast<uint32_t*>(codes));
    else
        launch_kernel((orq_quantize_kernel<C, S, BITS, false, RULE>), dim3(nb), dim3(kWave), st, g, n, p->bucket_size,
                           p->level_iters, p->clip_factor, nb, p->seed, p->index_offset, lv,
                           static_cast<uint32_t*>(codes));
}

template <int S, int BITS>
void launch_even_small(const float* g, size_t n, const ogq_params_t* p, float* lv, void* codes, hipStream_t st)
{
    const size_t spans = (n + 255u) / 256u;
    const dim3 grid((uint32_t)((spans + 3u) / 4u)), block(4 * kWave);
    if (p->bucket_size == 64u)
        launch_kernel((even_small_kernel<S, BITS, 4>), grid, block, st, g, n, p->clip_factor, p->seed, p->index_offset,
                           lv, static_cast<uint32_t*>(codes));
    else
        launch_kernel((even_small_kernel<S, BITS, 2>), grid, block, st, g, n, p->clip_factor, p->seed, p->index_offset,
                           lv, static_cast<uint32_t*>(codes));
}

template <int S, int BITS, int RULE>
void launch_sorted_small(const float* g, size_t n, const ogq_params_t* p, float* lv, void* codes, hipStream_t st)
{
    const size_t spans = (n + 255u) / 256u;
    const dim3 grid((uint32_t)((spans + 3u) / 4u)), block(4 * kWave);
    if (p->bucket_size == 64u)
        launch_kernel((sorted_small_kernel<S, BITS, 4, RULE>), grid, block, st, g, n, p->level_iters, p->clip_factor,
                           p->seed, p->index_offset, lv, static_cast<uint32_t*>(codes));
    else
        launch_kernel((sorted_small_kernel<S, BITS, 2, RULE>), grid, block, st, g, n, p->level_iters, p->clip_factor,
                           p->seed, p->index_offset, lv, static_cast<uint32_t*>(codes));
}

template <int C, int RULE>
void launch_paper_counts(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                         hipStream_t st)
{
    if constexpr (C == 1 && (RULE == kOptimal || RULE == kLinear)) {
        // buckets of 64 and 128 elements, sorted in registers, several per wavefront
        if (p->bucket_size == 64u || p->bucket_size == 128u) {
            switch (p->bits) {
                case 2: launch_sorted_small<3, 2, RULE>(g, n, p, lv, codes, st); break;
                case 3: launch_sorted_small<5, 3, RULE>(g, n, p, lv, codes, st); break;
                default: launch_sorted_small<9, 4, RULE>(g, n, p, lv, codes, st); break;
            }
            return;
        }
    }
    if constexpr (C == 1 && RULE == kEven) {
        // buckets of 64 and 128 elements: several buckets per wavefront
        if (p->bucket_size == 64u || p->bucket_size == 128u) {
            switch (p->bits) {
                case 2: launch_even_small<3, 2>(g, n, p, lv, codes, st); break;
                case 3: launch_even_small<5, 3>(g, n, p, lv, codes, st); break;
                default: launch_even_small<9, 4>(g, n, p, lv, codes, st); break;
            }
            return;
        }
    }
    switch (p->bits) {  // 2^(bits-1) + 1 levels
        case 2: launch_orq<C, 3, 2, RULE>(g, n, p, nb, lv, codes, st); break;
        case 3: launch_orq<C, 5, 3, RULE>(g, n, p, nb, lv, codes, st); break;
        default: launch_orq<C, 9, 4, RULE>(g, n, p, nb, lv, codes, st); break;
    }
}

template <int C>
void launch_orq_levels(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                       hipStream_t st)
{
    switch (p->scheme) {
        case OGQ_BINGRAD_PB:
            if constexpr (C == 1) {
                if (p->bucket_size == 64u || p->bucket_size == 128u) {
                    launch_sorted_small<2, 1, kPb>(g, n, p, lv, codes, st);
                    break;
                }
            }
            launch_orq<C, 2, 1, kPb>(g, n, p, nb, lv, codes, st);
            break;
        case OGQ_ORQ:
            if constexpr (C == 1) {
                // buckets of 64 and 128 elements, sorted in registers, several per wavefront
                if (p->bucket_size == 64u || p->bucket_size == 128u) {
                    if (p->bits == 1) launch_sorted_small<2, 1, kOptimal>(g, n, p, lv, codes, st);
                    else if (p->bits == 2) launch_sorted_small<4, 2, kOptimal>(g, n, p, lv, codes, st);
                    else launch_sorted_small<8, 3, kOptimal>(g, n, p, lv, codes, st);
                    break;
                }
            }
            switch (p->bits) {
                case 1: launch_orq<C, 2, 1>(g, n, p, nb, lv, codes, st); break;
                case 2: launch_orq<C, 4, 2>(g, n, p, nb, lv, codes, st); break;
                default: launch_orq<C, 8, 3>(g, n, p, nb, lv, codes, st); break;
            }
            break;
        case OGQ_EVEN: launch_paper_counts<C, kEven>(g, n, p, nb, lv, codes, st); break;
        case OGQ_LINEAR: launch_paper_counts<C, kLinear>(g, n, p, nb, lv, codes, st); break;
        default: launch_paper_counts<C, kOptimal>(g, n, p, nb, lv, codes, st); break;  // OGQ_ORQ_PAPER
    }
}

// Buckets above 4096 elements: W wavefronts per bucket.
template <int W, int C, int S, int BITS, int RULE = kOptimal>
void launch_orq_team(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes, hipStream_t st)
{
    launch_kernel((orq_team_kernel<W, C, S, BITS, RULE>), dim3(nb), dim3(W * kWave), st, g, n, p->bucket_size,
                       p->level_iters, p->clip_factor, nb, p->seed, p->index_offset, lv, static_cast<uint32_t*>(codes));
}

template <int W, int C, int RULE>
void launch_team_paper_counts(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                              hipStream_t st)
{
    switch (p->bits) {  // 2^(bits-1) + 1 levels
        case 2: launch_orq_team<W, C, 3, 2, RULE>(g, n, p, nb, lv, codes, st); break;
        case 3: launch_orq_team<W, C, 5, 3, RULE>(g, n, p, nb, lv, codes, st); break;
        default: launch_orq_team<W, C, 9, 4, RULE>(g, n, p, nb, lv, codes, st); break;
    }
}

template <int W, int C>
void launch_orq_team_levels(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes,
                            hipStream_t st)
{
    switch (p->scheme) {
        case OGQ_BINGRAD_PB: launch_orq_team<W, C, 2, 1, kPb>(g, n, p, nb, lv, codes, st); break;
        case OGQ_ORQ:
            switch (p->bits) {
                case 1: launch_orq_team<W, C, 2, 1>(g, n, p, nb, lv, codes, st); break;
                case 2: launch_orq_team<W, C, 4, 2>(g, n, p, nb, lv, codes, st); break;
                default: launch_orq_team<W, C, 8, 3>(g, n, p, nb, lv, codes, st); break;
            }
            break;
        case OGQ_EVEN: launch_team_paper_counts<W, C, kEven>(g, n, p, nb, lv, codes, st); break;
        case OGQ_LINEAR: launch_team_paper_counts<W, C, kLinear>(g, n, p, nb, lv, codes, st); break;
        default: launch_team_paper_counts<W, C, kOptimal>(g, n, p, nb, lv, codes, st); break;  // OGQ_ORQ_PAPER
    }
}

}  // namespace ogq
#endif  // OGQ_ROUNDING_KERNELS_H
