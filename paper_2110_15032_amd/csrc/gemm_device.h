// Device-side building blocks shared by the MFMA GEMM translation units: element conversions, the LDS
// images of operand tiles with their swizzles and fragment reads (Tile), the workgroup id -> tile
// walk, the GeLU evaluation and the memory instructions that the persistent kernels issue outside
// the compiler's bookkeeping.  Everything is internal (anonymous namespace, one copy per unit).
#pragma once
#include <cstdlib>
#include <utility>

#include "sbp_internal.h"

namespace sbp {
namespace {
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even, NaN kept quiet: the hardware conversion (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ inline uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
// two values into one dword, `lo` in the low half
__device__ inline uint32_t f32_to_bf16x2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}


constexpr int BK = 64;  // reduction extent of one LDS stage of gemm_mfma_kernel, in elements

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;
typedef __attribute__((address_space(1))) const char gbl_char;

// LDS image of a KC tile: row-major [R][BKT], the 16-byte chunks of a row permuted by XOR with
// kswz(row).  A ds_read_b128 serves 16 lanes per pass and the LDS has 64 banks of 4 bytes, so the 16
// chunks of a pass must fall in 16 different 16-byte bank groups.  The 32x32x16 fragments put 32
// consecutive rows of one chunk column on lanes 0-31:
//   BKT = 64 (128-byte rows): XOR with (row ^ row >> 3) & 7, BKT = 32 (64-byte rows): (row >> 2) & 3.
// Both measured conflict-free on gfx950 (SQ_LDS_BANK_CONFLICT = 0), whichever 16 lanes make a pass
// (see kswz16 for the lane sets that the measurements point to).
template <int BKT>
__device__ inline int kswz(int row) {
    if constexpr (BKT == 64) return (row ^ (row >> 3)) & 7;
    else return (row >> 2) & 3;
}
// KC tiles read by the 16x16x32 fragments (lane l: row l % 16, chunk l / 16).  The passes of that
// ds_read_b128 are taken not to be 16 consecutive lanes but lanes {0-3, 12-15, 20-23, 24-27}, then
// {4-7, 8-11, 16-19, 28-31}, then the same plus 32: a pass mixes rows 0-3 and 12-15 of one chunk column
// with rows 4-11 of its neighbour.  With q = row / 4, XOR values (0, 3, 2, 1)[q] keep the four rows of
// equal row % 4 in such a pass on four different chunks (and do so for 16 consecutive lanes as well).
__device__ inline int kswz16(int row) { return (0 - (row >> 2)) & 3; }
// LDS image of a not-KC tile: [BKT][R] with the 16-byte chunks of kk-row q permuted by XOR with
// nswz(q).  A ds_read_b64_tr_b16 serves 32 lanes per pass: 4 consecutive kk-rows x 64 contiguous
// bytes.  Row pitch is a multiple of 256 B, so without the permutation the 4 rows share banks;
// moving row q by (q % 4) * 64 B spreads them over all 64 banks.  The 16x16x32 fragments read kk-rows
// q and q + 8 in one pass, 32 bytes each: rows with bit 3 set move by another 32 B (a constant inside
// every pass of the 32x32x16 fragments, so those are not affected).
__device__ inline int nswz(int krow) { return ((krow & 3) << 2) ^ (((krow >> 3) & 1) << 1); }

// F16: the tile feeds v_mfma_f32_16x16x32_bf16 (frag16) and its KC image is permuted by kswz16.
template <int R, bool KC, int NT, int BKT = BK, bool F16 = false>
struct Tile {
    static constexpr int BYTES = R * BKT * 2;
    static constexpr int CHUNKS = BYTES / 16;
    static constexpr int PER_THREAD = CHUNKS / NT;
    static constexpr int CPR = R / 8;        // 16-byte chunks per kk-row of a not-KC tile
    static constexpr int CPK = BKT / 8;      // 16-byte chunks per row of a KC tile
    static constexpr int ROWB = BKT * 2;     // bytes per row of a KC tile
    __device__ static int ksw(int row) { return F16 ? kswz16(row) : kswz<BKT>(row); }
    static_assert(CHUNKS % NT == 0, "tile must divide over the workgroup");
    static_assert(KC || CPR >= 16, "not-KC swizzle needs at least 16 chunks per row");

    // Byte offset (from the operand's base, at reduction offset 0) of the 16 bytes that belong in
    // LDS chunk position p.  first = first tile row (m or n), limit = extent of that index; rows or
    // columns past the limit are clamped to valid memory and never reach an output.
    __device__ static uint32_t src_offset(int ld, int first, int limit, int p) {
        if constexpr (KC) {
            const int row = p / CPK;
            int g = first + row;
            g = g < limit ? g : limit - 1;
            return ((uint32_t)g * (uint32_t)ld + (uint32_t)(((p % CPK) ^ ksw(row)) * 8)) * 2u;
        } else {
            const int krow = p / CPR;
            int col = first + (((p % CPR) ^ nswz(krow)) * 8);
            col = col < limit ? col : limit - 8;
            return ((uint32_t)krow * (uint32_t)ld + (uint32_t)col) * 2u;
        }
    }
    // bytes to advance the source by for one BKT step
    __device__ static uint32_t step_bytes(int ld) { return KC ? BKT * 2u : (uint32_t)ld * BKT * 2u; }

    // global -> LDS without passing through registers: each lane's 16 bytes land at
    // lds + 16 * (p0 + lane), p0 uniform per wave instruction (wave must be a uniform value).
    // src is a uniform global-address-space base, off the per-lane 32-bit byte offsets.
    __device__ static void load_direct(char* lds_tile, gbl_char* src, const uint32_t (&off)[PER_THREAD], int wave) {
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int p0 = it * NT + wave * 64;
            __builtin_amdgcn_global_load_lds((gbl_void*)(src + off[it]), (lds_void*)(lds_tile + p0 * 16), 16, 0, 0);
        }
    }

    // The same load outside the compiler's bookkeeping (persistent kernel: every wait on the memory
    // counter there is explicit, see its tile loop).  M0 carries the LDS address of lane 0's 16 bytes;
    // one idle cycle separates its write from the load that reads it.
    __device__ static void load_direct_untracked(char* lds_tile, gbl_char* src, const uint32_t (&off)[PER_THREAD], int wave) {
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int p0 = it * NT + wave * 64;
            const uint32_t lds = (uint32_t)(uintptr_t)(lds_void*)(lds_tile + p0 * 16);
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                         : : "v"(off[it]), "s"(src), "s"(lds) : "memory", "m0");
        }
    }

    // Fragment addressing.  The compiler tags an LDS access with the __shared__ object it touches
    // only through SHORT pointer chains, and it needs that tag to see that fragment reads of one
    // stage cannot alias direct-to-LDS loads into another (otherwise it serialises them with a
    // vmcnt wait).  So every address is tile + (lane offset + constant): the lane offsets are
    // computed once, made opaque to reassociation, and everything else folds into the instruction's
    // immediate offset.  A KC tile needs one lane offset per ks (the swizzle XORs ks into the chunk
    // index), a not-KC tile one per 32-wide block (the swizzle XORs the block index).
    template <int F>
    static constexpr int nlo() { return KC ? BKT / 16 : F; }

    __device__ static int lane_offset(int idx, int wave_base, int lane) {
        int off;
        if constexpr (KC) {   // idx = ks; block i adds i * 32 * ROWB
            const int row = wave_base + (lane & 31);
            off = row * ROWB + (((2 * idx + (lane >> 5)) ^ kswz<BKT>(row)) << 4);
        } else {              // idx = block; ks adds 16 ks * R * 2, the second read 4 * R * 2
            const int s = lane & 15, nh = (lane >> 4) & 1, kh = lane >> 5;
            const int krow = 8 * kh + (s >> 2);
            const int chunk = ((wave_base + 32 * idx) >> 3) + 2 * nh + ((s & 3) >> 1);
            off = krow * (R * 2) + ((chunk ^ nswz(krow)) << 4) + (s & 1) * 8;
        }
        asm("" : "+v"(off));   // opaque: keep it one addend
        return off;
    }

    // LDS -> one 32x32x16 MFMA operand for 32-row block blk of the wave tile: lane l gets the 8 values
    // kk = 16 ks + 8 (l / 32) + 0..7 of row (block base + l % 32).
    template <int NLO>
    __device__ static bf16x8 frag(const char* lds_tile, const int (&lo)[NLO], int blk, int ks) {
        if constexpr (KC) {
            // BKT = 64: kswz(row + 32 blk) differs from kswz(row) by (4 blk) & 7, i.e. odd blocks flip
            // chunk bit 2.  BKT = 32: kswz does not depend on blk.
            const int flip = BKT == 64 ? ((blk & 1) << 6) : 0;
            const int off = (lo[ks] ^ flip) + blk * 32 * ROWB;
            return *reinterpret_cast<const bf16x8*>(lds_tile + off);
        } else {
            // ds_read_b64_tr_b16: in each group of 16 lanes, lane s supplies the address of 4
            // consecutive elements (row s / 4, element group s % 4) of a 4 x 16 block and receives
            // column s of it.  Two reads (kk-rows +0..3 and +4..7, same swizzle) give the 8 values.
            const int off0 = lo[blk] + ks * 16 * (R * 2);
            const int off1 = off0 + 4 * (R * 2);
            const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(lds_tile + off0));
            const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(lds_tile + off1));
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            const s16x8 v = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    }

    // ---- operands of v_mfma_f32_16x16x32_bf16 (BKT = 32: one instruction spans the whole stage) ----
    // Lane l holds the 8 values kk = 8 (l / 16) + 0..7 of row (block base + l % 16).
    // One lane offset serves every block.  KC: a 16-row block adds 16 * ROWB (kswz16 repeats every 16 rows).
    // Not KC: block b adds 2 b to the chunk index; the wave's base chunk is a multiple of 16 and b < 8, so
    // that sum is an OR, and the swizzle being an XOR, block b's offset is block 0's with (b << 5) flipped.
    __device__ static int lane_offset16(int wave_base, int lane) {
        static_assert(BKT == 32, "one 16x16x32 instruction per 32-deep stage");
        int off;
        static_assert(F16, "frag16 reads tiles laid out for it");
        if constexpr (KC) {
            const int row = wave_base + (lane & 15);
            off = row * ROWB + (((lane >> 4) ^ kswz16(row)) << 4);
        } else {              // the second read adds 4 kk-rows
            const int s = lane & 15, g = lane >> 4;
            const int krow = 8 * g + (s >> 2);
            const int chunk = (wave_base >> 3) + ((s & 3) >> 1);
            off = krow * (R * 2) + ((chunk ^ nswz(krow)) << 4) + (s & 1) * 8;
        }
        asm("" : "+v"(off));
        return off;
    }
    __device__ static bf16x8 frag16(const char* lds_tile, int lo, int blk) {
        if constexpr (KC) {
            return *reinterpret_cast<const bf16x8*>(lds_tile + (lo + blk * 16 * ROWB));
        } else {
            // (as volatile assembly: a plain XOR is loop-invariant, and the compiler would keep one copy per block
            // in registers all through the reduction loop, which has none to spare)
            int off0 = lo;
            if (blk) asm volatile("v_xor_b32 %0, %1, %2" : "=v"(off0) : "v"(lo), "v"(blk << 5));
            const int off1 = off0 + 4 * (R * 2);
            const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(lds_tile + off0));
            const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(lds_tile + off1));
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            const s16x8 v = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    }
};

template <int N, typename F, int... Is>
__device__ inline void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ inline void static_for(F&& f) {
    static_for_impl<N>(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

struct TileCoord {
    int g, tile_m, tile_n;
    bool valid;
};

// Workgroup id -> (shard, tile).  Hardware hands consecutive workgroup ids to the 8 XCDs in turn;
// re-linearise so that each XCD walks a contiguous range of tiles (with k = 8 one whole shard,
// whose W_g then lives in that XCD's L2 only), and walk the tiles of a shard in bands of GM
// tile-rows, column by column, so that the 32 CUs of an XCD share operand tiles at any time.
__device__ inline TileCoord map_tile(int bid, int nblk, int tm, int tn, int groups, int order) {
    const int per_xcd = nblk >> 3;
    const int GM = order & 0xFF;                 // tile-rows per band
    const int v = (order & 0x100) ? bid : (bid & 7) * per_xcd + (bid >> 3);   // bit 8: no XCD re-linearisation
    const int per_group = tm * tn;
    TileCoord t;
    t.valid = v < per_group * groups;
    t.g = v / per_group;
    const int tl = v - t.g * per_group;
    const int band = tl / (GM * tn);
    const int first_m = band * GM;
    const int gsz = (tm - first_m) < GM ? (tm - first_m) : GM;
    const int in_band = tl - band * GM * tn;
    t.tile_m = first_m + in_band % gsz;
    t.tile_n = in_band / gsz;
    return t;
}

// max(a, b, c) in one instruction, a NaN operand ignored next to a number (the hardware's maxNum).  Written as
// assembly because fmaxf() on values the compiler cannot prove canonical (matrix-instruction results) costs a
// canonicalising multiply per operand: 300 instead of 64 vector instructions per tile and wave in the fused row
// maximum.
__device__ inline float max3f(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// gelu(x) = 0.5 x erfc(-x / sqrt 2), with erfc(z) = t 2^(-z^2 log2 e + P(t)), t = 1 / (1 + z / 2), for
// z = |x| / sqrt 2 >= 0.  This is the form of the classic Chebyshev fit of erfc ("erfcc" in Numerical
// Recipes), which keeps its RELATIVE accuracy in the tail, so gelu of a negative argument does too.
// P is a degree-5 minimax fit of log2(erfc(z) e^(z^2) / t) on 0 <= z <= 14 made for this kernel (the
// published fit has degree 9 and 1e-7; this one costs four FMAs less).  Relative error of gelu below
// 2.2e-5 for every x whose result is a normal fp32 number, a hundredth of a bf16 rounding step.  One rcp,
// one exp2, one max (max3f: fmaxf would add a canonicalising instruction), eight FMA/mul, no branch, no select.
// The argument is clamped to +-14 (erfc underflows before that), so +-inf give +inf and -0.
__device__ inline float gelu_fast(float x) {
    const float xc = __builtin_amdgcn_fmed3f(x, -14.0f, 14.0f);
    const float t = __builtin_amdgcn_rcpf(fmaf(fabsf(xc), 0.35355339059327373f, 1.0f));
    float p = 0.320185989f;
    p = fmaf(p, t, -0.994857252f);
    p = fmaf(p, t, 0.654060185f);
    p = fmaf(p, t, 0.382378936f);
    p = fmaf(p, t, 1.46516109f);
    p = fmaf(p, t, -2.82694018f);                            // constant term less 1: the factor 0.5 below
    const float w = xc * 0.84932180028801905f;               // sqrt(log2(e) / 2): w^2 = z^2 log2 e
    const float e = t * __builtin_amdgcn_exp2f(fmaf(-w, w, p));   // 0.5 erfc(|x| / sqrt 2)
    // 0.5 x (1 + erf) = max(x, 0) - |x| 0.5 erfc(|x| / sqrt 2) for either sign; nothing cancels for x < 0
    return fmaf(-fabsf(xc), e, max3f(x, 0.0f, 0.0f));
}

template <int EPI>
__device__ inline float mfma_epilogue(float v) {
    if constexpr (EPI == SBP_EPI_GELU) return gelu_fast(v);
    else return v;
}

constexpr int STAGE_BYTES = 4096;
constexpr int vmcnt_only(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }   // s_waitcnt vmcnt(n), nothing else

// Row maximum of stored results (model-parallel softmax, Sec. 6.3.1, fused into the logits GEMM):
// max over fp32 bit patterns with one integer atomic, signed max for non-negative values and unsigned
// min for negative ones (both orders agree with the float order on their half; -0 is folded to +0
// first; a NaN matches neither and is ignored, as fmaxf ignores it in the two-pass form).  Issued as
// inline assembly like the other stores of the persistent kernel.  The target starts at -inf
// (fill_rowmax_kernel).
__device__ inline void atomic_max_f32_untracked(float* a, float v) {
    v += 0.0f;
    if (v >= 0.0f) asm volatile("global_atomic_smax %0, %1, off" : : "v"(a), "v"(v) : "memory");
    else if (v < 0.0f) asm volatile("global_atomic_umin %0, %1, off" : : "v"(a), "v"(v) : "memory");   // a NaN is ignored
}

// 16-byte streaming store the compiler does not track.  The two idle cycles cover the hardware's
// rule that the data registers of a store wider than 8 bytes must not be rewritten right behind it
// (the compiler inserts them for stores it knows; here it cannot).
// `stream` (uniform): non-temporal.  Right when every 128-byte row segment is a whole cache line;
// with a row pitch that is not a multiple of 128 bytes every segment straddles two lines that the
// neighbouring wave completes a little later, and L2 has to keep them until then (measured on the
// 250000-byte pitch of the classifier logits: 1.62 ms streaming, 1.43 ms cached).
template <typename V>
__device__ inline void store16_untracked(V* p, const V v, bool stream) {
    if (stream) asm volatile("global_store_dwordx4 %0, %1, off nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
// element stores of the same kind for edge tiles (a tracked store anywhere in the tile loop is enough
// to bring the compiler's blanket waits back)
__device__ inline void store_out_untracked(float* c, int64_t pos, float v) {
    asm volatile("global_store_dword %0, %1, off nt" : : "v"(c + pos), "v"(v) : "memory");
}
__device__ inline void store_out_untracked(uint16_t* c, int64_t pos, float v) {
    const uint32_t b = f32_to_bf16(v);
    asm volatile("global_store_short %0, %1, off nt" : : "v"(c + pos), "v"(b) : "memory");
}

}  // namespace
}  // namespace sbp
