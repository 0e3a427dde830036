// Matrix-core decode attention over the packed pool (gfx950, v_mfma_f32_32x32x16_f16).
//
// One wave owns up to 64 query rows (NT tiles of 32) of one KV head and streams 32-token tile
// records.  Per tile, with tokens as the MFMA M dimension and query rows as N:
//
//   staging  a lane's share of a record (its key-code runs, its token's scales, its value-code
//            triplets -- every wave load one contiguous run) is loaded into registers one step ahead
//            of its use, so each load has a whole step to land.
//   pipeline two tiles are in flight per wave: the scores of the next tile are computed on the matrix
//            cores while the vector ALUs run the softmax and value dequantization of the current one.
//   scores   S^T[t, r] = sum_j sum_{k in block j} (code[t,k] * s[t,j]) * q[r,k].  The dequantized key
//            code*s has up to 18 significant bits, so it is split exactly into two fp16 terms
//            hi = fp16(code*s), lo = code*s - hi (one packed fma), each fed to the two K=16 MFMAs of a
//            q8_0 block with fp32 accumulation: key dequantization stays exact.
//   softmax  online, per row, in base-2 units; a row's reference only moves when the row's probabilities
//            of one tile sum to more than 2^15 in a lane, so the accumulator rescale is rare, p fits
//            fp16, and the common case takes no maximum over the scores at all.
//   PV       O^T[v, r] += sum_t c[code[t, v]] * p[t, r]   with the score tile's accumulator layout
//            feeding the B operand directly (the value codes are stored in that k-order), centroids
//            looked up with byte permutes.  The softmax denominator is summed from the very same
//            fp16-rounded p with packed dot products.
//
// Why 32x32x16: a wave that interleaves MFMAs with vector work pays about 11.5 issue cycles per MFMA
// whatever its shape and 4 per vector instruction, so the larger tile halves the MFMA share of the
// issue time for the same arithmetic.
//
// The accumulation stays in the rotated value domain; the inverse Walsh-Hadamard rotation is done
// once per output row (sections "Compression Scheme" / "TurboQuant", dequantization), in this kernel
// when one workgroup covers the whole token range and there are no private tails, else in the merge
// kernel.  The four waves of a workgroup take interleaved tiles and are merged through LDS.
#include <hip/hip_fp16.h>

#include <mutex>
#include <type_traits>

#include "polykv_internal.hpp"
#include "polykv_layout.hpp"

namespace polykv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

union H8 {
    half8 h;
    uint32_t u[4];
    half2v p[4];
};

__device__ __forceinline__ float16v mfma32(const half8& a, const half8& b, const float16v& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// lane <-> lane ^ 32 combinations
__device__ __forceinline__ float xor32_max(float x) {
    const uint32_t xi = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_sum(float x) {
    const uint32_t xi = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ---- tile staging: global -> registers, one step ahead ------------------------------------------
// A lane's share of a tile record: its 16 bytes of every key block (the A operands of the block's two
// K=16 slices), the scales of its token, and its value-code triplets.  Every load is one contiguous,
// fully coalesced run across the wave (the record is stored in exactly this order).
template <int D> struct RawK {
    uint4v k[D / 32];      // [j]: codes of token m, block j: elements 8h..8h+7 (x, y) and 16+8h.. (z, w)
    uint32_t sc[D / 64];   // fp16 scales of token m, blocks 0..NB-1 (unused with one scale per layer tensor)
};
template <int D, int VC> struct RawV {
    uint32_t w[vc_bits(VC) == 3 ? D / 64 : 1][3];  // 3-bit codecs: the lane's code triplets
    uint4v c[vc_bits(VC) == 8 ? D / 32 : 1];       // int8 codec: the lane's 16 code bytes of every coordinate group
    // 4-bit codecs: one dword per coordinate group; 2-bit codecs: one per pair of groups
    uint32_t n[vc_bits(VC) == 4 ? D / 16 : vc_bits(VC) == 2 ? D / 32 : 1];
    // codecs with value scales: the scales of the lane's 16 tokens as fp16 pairs, in the order in which
    // the lane holds their probabilities (tokens 8b + 4h + {0,1} in g[2b], + {2,3} in g[2b+1])
    uint32_t g[vc_has_scale(VC) ? 8 : 1];
};

// The records of a KV head are read through a buffer resource: every load is "resource + wave-uniform byte
// offset of the tile (a scalar register) + the lane's constant offset (a vector register that never changes)
// + an immediate", so a step spends no vector instruction on addresses, and a load beyond the KV head's records
// would return zeros instead of touching memory.
typedef __amdgpu_buffer_rsrc_t TileRsrc;
__device__ __forceinline__ TileRsrc make_tile_rsrc(const uint8_t* unit_base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(unit_base), 0, bytes, 0x00020000);
}
template <int D, int KC> __device__ __forceinline__ void load_rawk(RawK<D>& r, TileRsrc rs, uint32_t tile, int lane) {
    const uint32_t soff = Layout<D>::kscales_off + (uint32_t)(lane & 31) * (D / 32) * 2, koff = (uint32_t)lane * 16;
    if (KC == 0) {
        if (D == 64) {
            r.sc[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, soff, tile, 0);
        } else {
#pragma unroll
            for (int x = 0; x < D / 128; ++x) {
                const auto two = __builtin_amdgcn_raw_buffer_load_b64(rs, soff + 8 * x, tile, 0);
                r.sc[2 * x] = two[0];
                r.sc[2 * x + 1] = two[1];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < D / 32; ++j) r.k[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, koff + j * 1024, tile, 0);
}
template <int D, int VC, int KC>
__device__ __forceinline__ void load_rawv(RawV<D, VC>& r, TileRsrc rs, uint32_t tile, int lane) {
    using LY = Layout<D, VC, KC>;
    constexpr int VB = vc_bits(VC);
    if (VB == 4 || VB == 2) {
        constexpr int ND = VB == 4 ? D / 16 : D / 32;  // dwords per lane, contiguous
        const uint32_t voff = LY::vcodes_off + (uint32_t)lane * (ND * 4);
        if constexpr (ND % 4 == 0) {
#pragma unroll
            for (int i = 0; i < ND; i += 4) {
                const uint4v w = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 4 * i, tile, 0);
                r.n[i] = w.x, r.n[i + 1] = w.y, r.n[i + 2] = w.z, r.n[i + 3] = w.w;
            }
        } else {
            const auto w = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, tile, 0);  // ND == 2
            r.n[0] = w[0], r.n[1] = w[1];
        }
    } else if (VB == 8) {
        const uint32_t voff = LY::vcodes_off + (uint32_t)lane * 16;
#pragma unroll
        for (int g = 0; g < D / 32; ++g) r.c[g] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + g * 1024, tile, 0);
    } else {
        const uint32_t voff = LY::vcodes_off + (uint32_t)lane * 12;
#pragma unroll
        for (int q = 0; q < D / 64; ++q) {
            const auto w = __builtin_amdgcn_raw_buffer_load_b96(rs, voff + q * 768, tile, 0);
            r.w[q][0] = w[0], r.w[q][1] = w[1], r.w[q][2] = w[2];
        }
    }
    if (vc_has_scale(VC)) {
        const uint32_t goff = LY::vscales_off + (uint32_t)(lane >> 5) * 8;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const auto two = __builtin_amdgcn_raw_buffer_load_b64(rs, goff + 16 * b, tile, 0);
            r.g[2 * b] = two[0];
            r.g[2 * b + 1] = two[1];
        }
    }
}

// Half block (j, s) of a lane's key codes -> the exact two-term fp16 split of code * scale.  With one scale
// per layer tensor (KC = 1) the scale is folded into the softmax scale instead: hi is the code itself, an
// exact fp16 integer, and there is no second term.
template <int D, int KC>
__device__ __forceinline__ void key_split(const RawK<D>& rk, int j, int s, half8& hi, half8& lo) {
    H8 a;
    codes4_to_half(s == 0 ? rk.k[j].x : rk.k[j].z, a.u[0], a.u[1]);
    codes4_to_half(s == 0 ? rk.k[j].y : rk.k[j].w, a.u[2], a.u[3]);
    a.h = a.h - (_Float16)1152.0f;
    if (KC == 1) {
        hi = a.h;
        return;
    }
    union {
        uint32_t u;
        _Float16 h[2];
    } s2;
    s2.u = rk.sc[j >> 1];
    const half8 sv = (half8)(s2.h[j & 1]);
    hi = a.h * sv;
    lo = __builtin_elementwise_fma(a.h, sv, -hi);  // exact remainder of the product
}

// Constants the main loop keeps in scalar registers.  As 32-bit literals they would double the size of every
// instruction that uses them, and a lone wave's instruction fetch is what bounds the loop.
struct LoopConsts {
    uint32_t m7, m3, m4;   // byte masks 0x07070707, 0x03030303, 0x04040404 (value-code selectors)
    half2v one2;           // (1, 1): the packed dot product that sums a pair of probabilities
};
__device__ __forceinline__ LoopConsts make_loop_consts() {
    uint32_t m7 = 0x07070707u, m3 = 0x03030303u, m4 = 0x04040404u, one = 0x3c003c00u;
    asm volatile("" : "+s"(m7), "+s"(m3), "+s"(m4), "+s"(one));   // opaque: the compiler would fold them back
    union {
        uint32_t u;
        half2v h;
    } o;
    o.u = one;
    return LoopConsts{m7, m3, m4, o.h};
}

// Value group G of a lane: eight 3-bit codes -> fp16 centroids, the A operand of one P.V product.
template <int D, int VC>
__device__ __forceinline__ void value_group(const RawV<D, VC>& rv, int G, H8& va, const LoopConsts& lc) {
    if (vc_bits(VC) == 4) {
        group8_b4(rv.n[G], va.u);
        return;
    }
    if (vc_bits(VC) == 2) {
        group8_b2(rv.n[G >> 1], G & 1, va.u);
        return;
    }
    if (vc_bits(VC) == 8) {
        // int8 codes of coordinate group G/2, token half G%2 -> exact fp16 integers (the scale rides on P)
        const uint4v& c = rv.c[G >> 1];
        codes4_to_half((G & 1) == 0 ? c.x : c.z, va.u[0], va.u[1]);
        codes4_to_half((G & 1) == 0 ? c.y : c.w, va.u[2], va.u[3]);
        va.h = va.h - (_Float16)1152.0f;
        return;
    }
    uint32_t sel_a, sel_b;
    vcode_selectors(rv.w[G >> 2][0], rv.w[G >> 2][1], rv.w[G >> 2][2], G & 3, lc.m7, lc.m3, lc.m4, sel_a, sel_b);
    lookup4(sel_a, va.u[0], va.u[1]);
    lookup4(sel_b, va.u[2], va.u[3]);
}

__device__ __forceinline__ float max16(const float16v& a) {
    float m = fmaxf(fmaxf(a[0], a[1]), a[2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) m = fmaxf(fmaxf(m, a[i]), a[i + 1]);
    return fmaxf(m, a[15]);
}

// Four scores of a row -> fp16 probabilities (packed pairs) and their sum into lsum (the tile's sum).  With
// value scales (g != nullptr: the lane's RawV::g) the P.V operand is p * scale of its token (formed in fp32,
// rounded to fp16 once), at most 2^8 * 2^7; the denominator sums the plain, unrounded p.
template <bool VS>
__device__ __forceinline__ void exp4(const float16v& S, int c, float qscale, float mneg, H8 (&pb)[2], float& lsum,
                                     const uint32_t* g, half2v one2, float* gmax = nullptr) {
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
        const int i = 4 * c + 2 * pr;
        half2v p2;
        const float e0 = __builtin_amdgcn_exp2f(fmaf(S[i], qscale, mneg)), e1 = __builtin_amdgcn_exp2f(fmaf(S[i + 1], qscale, mneg));
        p2[0] = (_Float16)e0;
        p2[1] = (_Float16)e1;
        // The denominator sums the very numbers that enter the P.V product where those are the probabilities
        // themselves (their rounding errors then cancel in the quotient); with a value scale the products p * g
        // are what is rounded, so the denominator takes the unrounded probabilities.
        if (VS) lsum += e0 + e1;
        else lsum = __builtin_amdgcn_fdot2(p2, one2, lsum, false);
        if (VS) {   // p * g in fp32, rounded to fp16 once
            union {
                uint32_t u;
                _Float16 h[2];
            } g2;
            g2.u = g[i >> 1];
            const float g0 = (float)g2.h[0], g1 = (float)g2.h[1];
            p2[0] = (_Float16)(e0 * g0);
            p2[1] = (_Float16)(e1 * g1);
            if (gmax != nullptr) *gmax = fmaxf(fmaxf(*gmax, g0), g1);   // the largest scale among the lane's tokens
        }
        pb[i >> 3].p[(i & 7) >> 1] = p2;
    }
}

// The pool's last tile when it crosses the end of the pool, read straight from memory: scores, softmax
// and PV one after the other, tokens >= T masked out.  Runs at most once per KV head.
template <int D, int NT, int VC, int KC, bool K16>
__device__ __forceinline__ void process_ragged_tile(TileRsrc rs, uint32_t lt, int tile, int T, float qscale,
                                                 int lane, const half8 (&qb)[NT][D / 32][2], float16v (&O)[D / 32][NT],
                                                 float (&Lsum)[NT], float* m_ref, float (&mneg)[NT],
                                                 const LoopConsts& lc) {
    constexpr int NB = D / 32, NG = D / 16;
    const int h = lane >> 5;
    RawK<D> rk;
    RawV<D, VC> rv;
    load_rawk<D, KC>(rk, rs, lt, lane);
    load_rawv<D, VC, KC>(rv, rs, lt, lane);
    float16v S[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) S[nt][i] = 0.0f;
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            half8 hi, lo;
            key_split<D, KC>(rk, j, s, hi, lo);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                S[nt] = mfma32(hi, qb[nt][j][s], S[nt]);
                if (KC == 0 && !K16) S[nt] = mfma32(lo, qb[nt][j][s], S[nt]);
            }
        }
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (tile * kTile + 8 * (i >> 2) + 4 * h + (i & 3) >= T) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) S[nt][i] = -INFINITY;
        }
    H8 pb[NT][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        // this path always re-references: cheap here, and it needs no vote
        const float m_old = m_ref[32 * nt];
        const float m_new = fmaxf(m_old, xor32_max(max16(S[nt])));
        const float alpha = __builtin_amdgcn_exp2f((m_old - m_new) * qscale);
        m_ref[32 * nt] = m_new;
        mneg[nt] = -m_new * qscale;
        Lsum[nt] *= alpha;
#pragma unroll
        for (int g = 0; g < D / 32; ++g) O[g][nt] *= alpha;
#pragma unroll
        for (int c = 0; c < 4; ++c) exp4<vc_has_scale(VC)>(S[nt], c, qscale, mneg[nt], pb[nt], Lsum[nt], rv.g, lc.one2);
    }
#pragma unroll
    for (int G = 0; G < NG; ++G) {
        H8 va;
        value_group<D, VC>(rv, G, va, lc);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) O[G >> 1][nt] = mfma32(va.h, pb[nt][G & 1].h, O[G >> 1][nt]);
    }
}

// One software-pipelined step.  While the matrix cores compute the scores of tile B (the next tile),
// the vector ALUs turn the scores of tile A (the current tile, computed one step earlier) into
// probabilities and dequantize A's values; then the matrix cores accumulate A's P.V.  Keeping two
// tiles in flight is what lets MFMA and VALU work overlap within a single wave: the MFMA stream of a
// step never depends on vector work of the same tile that has not had a full step to complete.
//
//   rv, rk     tile A's value codes and tile B's key codes / scales, in registers
//   rvN, rkN   the same for the next step, requested here from nextV (the tile after A) and nextK (the
//              tile after B); the caller alternates the two register sets, so nothing is copied
//   Sa         scores of tile A on entry, of tile B on exit
// Only full tiles go through here; a ragged last tile is handled by process_ragged_tile.
//
// Softmax bookkeeping: the reference m_ref (raw score units) of a row only moves when the row's probabilities
// of a tile, taken against the old reference, sum to more than kRaiseSum = 2^15 in one of the row's two lanes --
// with value scales: when that sum times the largest scale among the lane's tokens of the tile does.  Every operand
// that reaches a P.V product (a probability, or a probability times its token's scale) is therefore at most 2^15:
// fp16 holds it; what matters for the result is the relative precision of a probability, which does not depend on
// its magnitude, and a probability 2^-29 below the row's largest may flush to zero.  The common case takes no
// maximum over the scores, and on keys with outlier channels, where a row's maximum keeps creeping up, the expensive
// rescale of the accumulators stays rare: with a threshold of 2^8 it was a tenth of the kernel's time on the
// Llama-shaped workload.
constexpr float kRaiseSum = 32768.0f;

template <int D, int NT, int VC, int KC, bool K16, bool HAS_A, bool HAS_B>
__device__ __forceinline__ void pipeline_step(const RawV<D, VC>& rv, const RawK<D>& rk, RawV<D, VC>& rvN, RawK<D>& rkN,
                                              TileRsrc rs, uint32_t nextK, uint32_t nextV, float qscale, int lane,
                                              const half8 (&qb)[NT][D / 32][2], float16v (&O)[D / 32][NT],
                                              float (&Lsum)[NT], float* m_ref, float (&mneg)[NT],
                                              float16v (&Sa)[NT], const LoopConsts& lc) {
    constexpr int NB = D / 32, NG = D / 16, MG = D / 32;
    const half8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    float16v Sb[NT];
    float lt[NT];   // this tile's probability sums, per lane
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) lt[nt] = 0.0f;

    // The step is written as a sequence of slices.  Each slice pairs a batch of MFMAs whose operands
    // are ready with the vector work that prepares the operands of the NEXT batch, and is closed by a
    // scheduling barrier so that the compiler keeps the pairing; inside a slice the two streams are
    // interleaved one MFMA to a few vector instructions.
    constexpr int NQK = 2 * NB;   // half blocks of tile B: (j, s)
    constexpr int NCH = 4 * NT;   // probability chunks of tile A: 4 scores each
    auto slice_end = [](auto mfmas, auto valus) {
        constexpr int M = decltype(mfmas)::value, V = decltype(valus)::value;
        constexpr int per = M > 0 ? (V + M - 1) / M : 0;
#pragma unroll
        for (int i = 0; i < M; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (per > 0) __builtin_amdgcn_sched_group_barrier(0x402, per, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    using std::integral_constant;

    // The next step's bytes are requested into the other set of registers as soon as the first score
    // products are on the matrix cores (right here when the step has none): every load still has nearly the
    // whole step to land, and the stretch in which the matrix cores wait for vector work stays short.
    auto request_next = [&]() {
        if (HAS_B) load_rawk<D, KC>(rkN, rs, nextK, lane);
        load_rawv<D, VC, KC>(rvN, rs, nextV, lane);
    };
    if (!HAS_B) {
        request_next();
        __builtin_amdgcn_sched_barrier(0);
    }

    H8 pb[NT][2];      // probabilities of tile A: B operands of the P.V products, [row tile][k slice]
    half8 khi[2], klo[2];
    H8 va[2];
    float gmax = vc_has_scale(VC) ? 5.9604645e-8f : 1.0f;   // (not 0: an infinite sum times it must still say "move")
    auto exp_chunk = [&](int c) {
        exp4<vc_has_scale(VC)>(Sa[c >> 2], c & 3, qscale, mneg[c >> 2], pb[c >> 2], lt[c >> 2], rv.g, lc.one2,
                               vc_has_scale(VC) && c < 4 ? &gmax : nullptr);
    };
    auto kdeq = [&](int k) { key_split<D, KC>(rk, k >> 1, k & 1, khi[k & 1], klo[k & 1]); };
    auto qk = [&](int k) {
        const int j = k >> 1, s = k & 1;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) Sb[nt] = mfma32(khi[k & 1], qb[nt][j][s], Sb[nt]);
        if (KC == 0 && !K16) {   // the exact remainder term; dropped when the keys may be rounded to fp16
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) Sb[nt] = mfma32(klo[k & 1], qb[nt][j][s], Sb[nt]);
        }
    };
    auto vdeq = [&](int G) { value_group<D, VC>(rv, G, va[G & 1], lc); };
    auto pv = [&](int G) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) O[G >> 1][nt] = mfma32(va[G & 1].h, pb[nt][G & 1].h, O[G >> 1][nt]);
    };

    if (HAS_B) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) Sb[nt][i] = 0.0f;
        // lead-in: only the vector work that the first products need
        constexpr int lead = 0;
        kdeq(0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < NQK; ++k) {
            qk(k);
            if (k == 0) request_next();
            if (k + 1 < NQK) kdeq(k + 1);
            if (HAS_A) {
                // spread the remaining probability chunks over the score slices
                const int c0 = lead + (k * (NCH - lead)) / NQK, c1 = lead + ((k + 1) * (NCH - lead)) / NQK;
#pragma unroll
                for (int c = c0; c < c1; ++c) exp_chunk(c);
            }
            slice_end(integral_constant<int, (KC == 0 && !K16 ? 2 : 1) * NT>{}, integral_constant<int, (HAS_A ? 28 : 16)>{});
        }
    } else if (HAS_A) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) exp_chunk(c);
        __builtin_amdgcn_sched_barrier(0);
    }

    if (HAS_A) {
        // Does a row have to move its reference?  Rare after a row's first tiles (always at its very first tile,
        // where the reference is -inf and every probability comes out as +inf).  The probabilities of the rows
        // that move are then recomputed against the new reference; those of the other rows come out as they
        // were.  Only the rows that outgrew their reference move it: a row's result depends on that row's
        // scores alone, whatever other agents' rows share the wave.
        // gmax: the largest value scale among the lane's 16 tokens of this tile (1 without value scales), collected
        // by the chunks of row tile 0; the products probability x scale stay below kRaiseSum if the tile's sum of
        // probabilities times gmax does
        bool raise = false;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) raise |= !(lt[nt] * gmax <= kRaiseSum);   // (inf and NaN say yes)
        if (__builtin_expect(__any(raise), 0)) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const bool row_raise = !(xor32_max(lt[nt] * gmax) <= kRaiseSum);   // (+inf stays +inf through the max)
                const float row_max = xor32_max(max16(Sa[nt]));
                const float m_old = m_ref[32 * nt];
                const float m_new = row_raise ? fmaxf(m_old, row_max) : m_old;
                if (!__any(m_new != m_old)) continue;   // no row of this row tile moves: it keeps what it has
                const float alpha = m_new == m_old ? 1.0f : __builtin_amdgcn_exp2f((m_old - m_new) * qscale);
                const bool first = __all(m_old == -INFINITY);  // nothing accumulated yet: nothing to rescale
                m_ref[32 * nt] = m_new;
                mneg[nt] = -m_new * qscale;
                if (!first) {
                    // The accumulators live in accumulation registers that vector instructions cannot read; an
                    // MFMA with zero operands (D = 0*0 + C) carries them to vector registers and back, so the
                    // hot path never copies them.
                    Lsum[nt] *= alpha;
#pragma unroll
                    for (int g = 0; g < MG; ++g) {
                        float16v y = mfma32(zero8, zero8, O[g][nt]);
                        y *= alpha;
                        O[g][nt] = mfma32(zero8, zero8, y);
                    }
                }
                lt[nt] = 0.0f;
#pragma unroll
                for (int c = 4 * nt; c < 4 * nt + 4; ++c) exp_chunk(c);
            }
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) Lsum[nt] += lt[nt];
        vdeq(0);
        __builtin_amdgcn_sched_barrier(0);
    }

    if (HAS_A) {
#pragma unroll
        for (int G = 0; G < NG; ++G) {
            pv(G);
            if (G + 1 < NG) vdeq(G + 1);
            slice_end(integral_constant<int, NT>{}, integral_constant<int, 12>{});
        }
    }

    if (HAS_B) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) Sa[nt] = Sb[nt];
    }
}

// Waves per SIMD the kernel is compiled for: one where it needs all 512 registers; three for 32-row blocks at
// head_dim 64 (the small-row shape of the SmolLM2-sized pool: 768 workgroups, all resident at once on 256 CUs,
// so that one workgroup's query fetch, pipeline ramp and merge overlap the others' main loops).
constexpr int kernel_waves_per_simd(int D, int NT, int VC) { return (D == 64 && NT == 1 && vc_bits(VC) == 3 && !vc_has_scale(VC)) ? 3 : 1; }

// ws_ml / ws_o: where the kernel leaves its split's partial (direct == 0); with direct == 1 and private tails,
// the tail kernel's partials (row maxima and denominators / unnormalized sums), read in the final pass.
template <int D, int NT, int VC, int KC, bool K16>
__global__ __launch_bounds__(256, kernel_waves_per_simd(D, NT, VC)) void attend_mfma_kernel(const uint8_t* __restrict__ pool,
                                                          const __half* __restrict__ Q,
                                                          float* __restrict__ ws_ml, float* __restrict__ ws_o,
                                                          float* __restrict__ out, AttendPlan p, int direct) {
    using LY = Layout<D, VC, KC>;
    constexpr int NB = D / 32, MG = D / 32, ROWS = 32 * NT;
    constexpr int OSTRIDE = D + 4;
    constexpr int TB = LY::tile_bytes;
    __shared__ float m_s[4][ROWS];
    __shared__ float l_s[4 * ROWS];
    extern __shared__ __align__(16) float o_s[];  // four merge buffers of ROWS x OSTRIDE floats

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform
    const int h = lane >> 5, n = lane & 31;
    const int usel = blockIdx.y, ls = usel / p.H, kvh = usel - ls * p.H;
    const int row0 = blockIdx.z * ROWS;
    const int split = blockIdx.x;
    const int tps = (p.tiles + p.nsplit - 1) / p.nsplit;
    const int t_begin = split * tps, t_end = min(p.tiles, t_begin + tps);
    const uint8_t* unit_base = pool + (size_t)((p.layer_begin + ls) * p.H + kvh) * p.tiles_cap * TB;
    // One key scale per layer tensor: the keys enter the products as their integer codes and the scale
    // rides on the softmax scale (an all-zero layer has only zero codes: any positive scale will do).
    float qscale = p.qscale;
    if (KC == 1) {
        const float s_tensor = (float)tensor_key_scale(p.kmax[p.layer_begin + ls]);
        qscale *= s_tensor > 0.0f ? s_tensor : 1.0f;
    }

    // this wave's tiles: t_begin + wave, +4, +8, ...; local index k <-> tile my_first + 4k
    const int my_first = t_begin + wave;
    const int my_count = my_first < t_end ? (t_end - my_first + 3) / 4 : 0;
    // pointer to local tile k; k past the end is clamped (the refill loads of the last steps then
    // fetch the wave's own last tile again, harmlessly, instead of needing a branch per load)
    // (byte offsets from the KV head's first record; pool_create keeps a KV head's records under 4 GiB)
    const TileRsrc rs = make_tile_rsrc(unit_base, (uint32_t)p.tiles_cap * (uint32_t)TB);
    const int last_k = max(my_count - 1, 0);
    auto tile_ptr = [&](int k) { return (uint32_t)(my_first + 4 * min(k, last_k)) * (uint32_t)TB; };
    RawK<D> rk;
    RawV<D, VC> rv;
    if (my_count > 0) {
        load_rawk<D, KC>(rk, rs, tile_ptr(0), lane);
        load_rawv<D, VC, KC>(rv, rs, tile_ptr(0), lane);
    }

    // ---- query rows as MFMA B operands: lane (n, h) holds q[row 32nt+n][32j + 16s + 8h .. +7].
    // The block of rows is fetched with fully coalesced 16-byte loads (16 lanes to a row) into LDS
    // (the merge buffers are idle until the end) and picked up from there in operand order.
    constexpr int QS = D + 8;  // halves per staged row: 16-byte aligned, rotates the banks
    _Float16* q_s = reinterpret_cast<_Float16*>(o_s);
    constexpr int QP = ROWS * (D / 8) / 256;  // 16-byte pieces per thread; all requested before any is used
    static_assert(QP * 256 == ROWS * (D / 8), "");
    uint4v qraw[QP];
#pragma unroll
    for (int u = 0; u < QP; ++u) {
        // rows past the end re-read the last row (no branch between the loads) and are zeroed below
        const int i = tid + 256 * u, rr = i / (D / 8), piece = i - rr * (D / 8), r = min(row0 + rr, p.R - 1);
        qraw[u] = *reinterpret_cast<const uint4v*>(Q + q_row_index(p, ls, kvh, r) * D + 8 * piece);
    }
    // the accumulators are cleared while the queries and the first tiles are on their way
    float16v O[MG][NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int g = 0; g < MG; ++g) {
#pragma unroll
            for (int i = 0; i < 16; ++i) O[g][nt][i] = 0.0f;
            asm volatile("" : "+a"(O[g][nt]));  // now, not where the first product needs them
        }
#pragma unroll
    for (int u = 0; u < QP; ++u) {
        const int i = tid + 256 * u, rr = i / (D / 8), piece = i - rr * (D / 8);
        uint4v raw = row0 + rr < p.R ? qraw[u] : uint4v{0, 0, 0, 0};
        if (p.io_bf16) {  // bfloat16 queries become fp16 operands (exact for magnitudes fp16 holds)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const float2 f = pair16_to_float2(raw[b], true);
                union {
                    uint32_t u;
                    _Float16 h[2];
                } o;
                o.h[0] = (_Float16)f.x;
                o.h[1] = (_Float16)f.y;
                raw[b] = o.u;
            }
        }
        *reinterpret_cast<uint4v*>(q_s + rr * QS + 8 * piece) = raw;
    }
    __syncthreads();
    half8 qb[NT][NB][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int s = 0; s < 2; ++s)
                qb[nt][j][s] = *reinterpret_cast<const half8*>(q_s + (32 * nt + n) * QS + 32 * j + 16 * s + 8 * h);
    __syncthreads();  // every wave has picked up its queries: the merge at the end reuses this memory
    // The queries are only ever MFMA operands: park them in accumulation registers so that the vector
    // registers are left for the scores and the dequantization temporaries (a second loop, so that the LDS
    // reads above are all in flight before the first one is waited for).  Not at head_dim 256: there the
    // allocator has to spill, and builds that spilled parked operands to scratch memory computed wrong
    // results.
    if constexpr (D != 256) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int s = 0; s < 2; ++s) asm volatile("" : "+a"(qb[nt][j][s]));
    }

    // The references themselves are only read where a row moves its reference and at the merge: they live in the
    // wave's row of m_s (LDS), not in registers.  Both lanes of a row hold the same value and write the same value;
    // a wave's LDS accesses complete in order, so a wave reading back what it wrote needs no barrier.
    float* const m_ref = &m_s[wave][n];   // row 32 nt + n at m_ref[32 * nt]
    float Lsum[NT], mneg[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_ref[32 * nt] = -INFINITY;
        mneg[nt] = INFINITY;   // no reference yet: the first tile's probabilities come out as +inf and set one
        Lsum[nt] = 0.0f;
    }
    const LoopConsts lc = make_loop_consts();
    float16v S[NT];  // scores of the tile whose softmax comes next

    // Local tile k is "B" in step k-1 (scores) and "A" in step k (softmax, PV).  Only the pool's very
    // last tile can be ragged; it stays out of the pipeline and goes last.
    const bool last_ragged = my_count > 0 && (my_first + 4 * (my_count - 1)) * kTile + kTile > p.T;
    const int full_count = last_ragged ? my_count - 1 : my_count;
    if (full_count > 0) {
        // register sets: (rk, rv) and (rk2, rv2) alternate between "current" and "being loaded"
        RawK<D> rk2;
        RawV<D, VC> rv2;
        // prologue: scores of tile 0 from rk; requests K of tile 1 and (again) V of tile 0 into set 2
        pipeline_step<D, NT, VC, KC, K16, false, true>(rv, rk, rv2, rk2, rs, tile_ptr(1), tile_ptr(0), qscale, lane, qb, O, Lsum, m_ref, mneg, S, lc);
        // the rows' first references: the maxima of this first tile, taken here once instead of letting the first
        // step find out through infinite probabilities and compute its tile's probabilities twice
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float m0 = xor32_max(max16(S[nt]));
            m_ref[32 * nt] = m0;
            mneg[nt] = -m0 * qscale;
        }
        int s = 0;
        for (; s + 1 < full_count - 1; s += 2) {  // two steps per trip: the sets swap roles without copies
            pipeline_step<D, NT, VC, KC, K16, true, true>(rv2, rk2, rv, rk, rs, tile_ptr(s + 2), tile_ptr(s + 1), qscale, lane, qb, O, Lsum, m_ref, mneg, S, lc);
            pipeline_step<D, NT, VC, KC, K16, true, true>(rv, rk, rv2, rk2, rs, tile_ptr(s + 3), tile_ptr(s + 2), qscale, lane, qb, O, Lsum, m_ref, mneg, S, lc);
        }
        if (s < full_count - 1) {  // one step with a B tile left: current = set 2
            pipeline_step<D, NT, VC, KC, K16, true, true>(rv2, rk2, rv, rk, rs, tile_ptr(s + 2), tile_ptr(s + 1), qscale, lane, qb, O, Lsum, m_ref, mneg, S, lc);
            pipeline_step<D, NT, VC, KC, K16, true, false>(rv, rk, rv2, rk2, rs, tile_ptr(s + 2), tile_ptr(s + 2), qscale, lane, qb, O, Lsum, m_ref, mneg, S, lc);
        } else {
            pipeline_step<D, NT, VC, KC, K16, true, false>(rv2, rk2, rv, rk, rs, tile_ptr(s + 1), tile_ptr(s + 1), qscale, lane, qb, O, Lsum, m_ref, mneg, S, lc);
        }
    }
    if (last_ragged)
        process_ragged_tile<D, NT, VC, KC, K16>(rs, tile_ptr(my_count - 1), my_first + 4 * (my_count - 1), p.T, qscale, lane, qb, O, Lsum, m_ref, mneg, lc);

    // ---- merge the four waves through LDS: every wave stores its row maxima, denominators and accumulators
    // as they are into buffers of its own; the final pass rescales them to the common row maximum and adds
    // them in a fixed order, so the result is reproducible.
    {
        float* obuf = o_s + wave * (ROWS * OSTRIDE);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int r = 32 * nt + n;
            const float l = xor32_sum(Lsum[nt]);  // the lane pair (n, h) shares a row
            if (h == 0) {
                l_s[wave * ROWS + r] = l;
            }
#pragma unroll
            for (int g = 0; g < MG; ++g)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    // registers 4b..4b+3 hold coordinates 32g + 8b + 4h + 0..3 of row r
                    float4* dst = reinterpret_cast<float4*>(&obuf[r * OSTRIDE + 32 * g + 8 * b + 4 * h]);
                    *dst = make_float4(O[g][nt][4 * b + 0], O[g][nt][4 * b + 1], O[g][nt][4 * b + 2], O[g][nt][4 * b + 3]);
                }
        }
    }
    __syncthreads();

    // ---- final pass: every wave finishes ROWS/4 rows, four lanes to a row.  Lane qd of a row takes every
    // fourth 4-coordinate piece (piece 4i + qd), so that the four lanes read and write 64 contiguous bytes per
    // instruction; the rotation is then log2(D/4) in-register stages and two DPP stages, whichever index bits
    // sit in the lane.
    constexpr int CPL = D / 4, RPW = ROWS / 4;
    const int ri = lane >> 2, qd = lane & 3;
    if (ri < RPW) {
        const int rr = wave + 4 * ri, r = row0 + rr;
        const float Mr = fmaxf(fmaxf(m_s[0][rr], m_s[1][rr]), fmaxf(m_s[2][rr], m_s[3][rr]));
        float fw[4];  // a wave's weight: 2^(its maximum - the common one); 0 if it saw no tile
#pragma unroll
        for (int w = 0; w < 4; ++w)
            fw[w] = m_s[w][rr] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f((m_s[w][rr] - Mr) * qscale);
        const float l = (l_s[rr] * fw[0] + l_s[ROWS + rr] * fw[1]) + (l_s[2 * ROWS + rr] * fw[2] + l_s[3 * ROWS + rr] * fw[3]);
        // Direct output with private tails: the row's tail partial (maximum in base-2 units, denominator and
        // unnormalized sum in the original value domain; written by the tail kernel, which ran before this one
        // and whose buffers arrive in ws_ml / ws_o) joins by log-sum-exp weights: the pool part gets wa / den
        // instead of 1 / l, the tail part wb / den once the pool part has been rotated back.
        float inv_l = __builtin_amdgcn_rcpf(l), tail_w = 0.0f;
        size_t tail_row = 0;
        if (direct && p.has_tails) {
            tail_row = (size_t)usel * p.R + min(r, p.R - 1);
            const float tm = ws_ml[tail_row * 2], tl = ws_ml[tail_row * 2 + 1];
            if (tl > 0.0f) {
                const float Mp = Mr * qscale, M2 = fmaxf(Mp, tm);
                const float wa = __builtin_amdgcn_exp2f(Mp - M2), wb = __builtin_amdgcn_exp2f(tm - M2);
                const float inv = 1.0f / (wa * l + wb * tl);
                inv_l = wa * inv;
                tail_w = wb * inv;
            }
        }
        // direct: 1/l, the centroid scale, 1/sqrt(D) and the entry sign of the DPP stages in one factor
        // int8 values are accumulated unrotated and unscaled: 1/l is all that is left to do
        constexpr float kCS = inv_centroid_scale<vc_bits(VC)>();
        const float f = VC == 2 ? (direct ? inv_l : 1.0f)
                        : direct ? quad_entry_sign(lane) * (kCS * (D == 64 ? 0.125f : D == 128 ? 0.08838834764831845f : 0.0625f)) *
                                       inv_l
                                 : kCS;
#pragma unroll
        for (int w = 0; w < 4; ++w) fw[w] *= f;
        float x[CPL];  // x[4i + k] = coordinate 16i + 4qd + k
        const float4* a4 = reinterpret_cast<const float4*>(&o_s[rr * OSTRIDE]) + qd;
        constexpr int BUF4 = ROWS * OSTRIDE / 4;  // one wave's buffer, in float4 units
#pragma unroll
        for (int i = 0; i < CPL / 4; ++i) {
            const float4 a = a4[4 * i], b = a4[BUF4 + 4 * i], c = a4[2 * BUF4 + 4 * i], d = a4[3 * BUF4 + 4 * i];
            x[4 * i + 0] = (a.x * fw[0] + b.x * fw[1]) + (c.x * fw[2] + d.x * fw[3]);
            x[4 * i + 1] = (a.y * fw[0] + b.y * fw[1]) + (c.y * fw[2] + d.y * fw[3]);
            x[4 * i + 2] = (a.z * fw[0] + b.z * fw[1]) + (c.z * fw[2] + d.z * fw[3]);
            x[4 * i + 3] = (a.w * fw[0] + b.w * fw[1]) + (c.w * fw[2] + d.w * fw[3]);
        }
        if (direct) {
            if (VC != 2) {
                wht_cross_quad<CPL>(x, lane);
                wht_inlane<CPL>(x);
                // rotation variant H.D: piece i holds coordinates 16i + 4qd ..
                if (p.signs.on) {
#pragma unroll
                    for (int i = 0; i < CPL / 4; ++i) {
                        float(&x4)[4] = *reinterpret_cast<float(*)[4]>(&x[4 * i]);
                        flip_signs<4>(x4, sign_word(p.signs, i >> 1) >> (16 * (i & 1) + 4 * qd));
                    }
                }
            }
            if (tail_w != 0.0f) {
                const float4* t4 = reinterpret_cast<const float4*>(ws_o + tail_row * D) + qd;
#pragma unroll
                for (int i = 0; i < CPL / 4; ++i) {
                    const float4 t = t4[4 * i];
                    x[4 * i] = fmaf(tail_w, t.x, x[4 * i]);
                    x[4 * i + 1] = fmaf(tail_w, t.y, x[4 * i + 1]);
                    x[4 * i + 2] = fmaf(tail_w, t.z, x[4 * i + 2]);
                    x[4 * i + 3] = fmaf(tail_w, t.w, x[4 * i + 3]);
                }
            }
            if (r < p.R) {
                float4* dst = reinterpret_cast<float4*>(out + q_row_index(p, ls, kvh, r) * D) + qd;
#pragma unroll
                for (int i = 0; i < CPL / 4; ++i) dst[4 * i] = make_float4(x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]);
            }
        } else if (r < p.R) {
            const size_t prow = ((size_t)usel * p.nsplit + split) * p.R + r;
            float4* dst = reinterpret_cast<float4*>(ws_o + prow * D) + qd;
#pragma unroll
            for (int i = 0; i < CPL / 4; ++i) dst[4 * i] = make_float4(x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]);
            if (qd == 0) {
                ws_ml[prow * 2] = Mr * qscale;
                ws_ml[prow * 2 + 1] = l;
            }
        }
    }
}

// Every shape the pool supports except int8 values at head_dim 256, where two staged tiles of code bytes do not
// fit the registers next to the accumulators (the vector kernel serves that corner).
bool matrix_kernel_supports(int head_dim, int rows_per_kv_head, int value_codec) {
    return (head_dim == 64 || head_dim == 128 || (head_dim == 256 && value_codec != POLYKV_VALUES_INT8)) &&
           rows_per_kv_head >= 1;
}

// Query rows per workgroup: 64 where the accumulators, the parked queries, two tiles of scores and two staged
// tiles fit the 512 registers of a wave; 32 at head_dim 256 and, at head_dim 128, for the two codecs with the
// most staged value bytes per tile (int8, and 4-bit codes with a scale).
int matrix_kernel_block_rows(int head_dim, int value_codec) {
    if (head_dim == 256) return 32;
    if (head_dim == 128 && (value_codec == POLYKV_VALUES_INT8 || value_codec == POLYKV_VALUES_TQ4_SCALED)) return 32;
    return 64;
}

bool matrix_kernel_direct(const AttendPlan& plan) { return plan.nsplit == 1; }

template <int D, int NT, int VC, int KC, bool K16>
static hipError_t launch_one(dim3 grid, const uint8_t* storage, const AttendPlan& plan, const void* Q, float* ws_ml,
                             float* ws_o, float* out, int direct, hipStream_t s) {
    constexpr int kMergeBytes = 4 * 32 * NT * (D + 4) * (int)sizeof(float);
    auto kern = attend_mfma_kernel<D, NT, VC, KC, K16>;
    static std::once_flag configured;  // per instantiation: the limit is a property of the function
    static hipError_t config_result = hipSuccess;
    if (kMergeBytes > 48 * 1024)
        std::call_once(configured, [&]() {
            config_result = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, kMergeBytes);
        });
    if (config_result != hipSuccess) return config_result;
    launch_main_kernel(kern, grid, dim3(256), kMergeBytes, s, storage, (const __half*)Q, ws_ml, ws_o, out, plan, direct);
    return hipGetLastError();
}

// Row tiles per workgroup: two (64 rows) or one (32 rows), see matrix_kernel_block_rows().
template <int D, int VC, int KC, bool K16>
static hipError_t launch_dv(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml, float* ws_o,
                            float* out, hipStream_t s) {
    const uint8_t* storage = reinterpret_cast<const uint8_t*>(pool->storage);
    const int units = plan.layers * plan.H;
    const int direct = matrix_kernel_direct(plan) ? 1 : 0;
    constexpr bool two_tiles_fit = D == 64 || (D == 128 && VC != 2 && VC != 6);   // matrix_kernel_block_rows()
    if constexpr (two_tiles_fit) {
        if (plan.R > 32 && plan.block_rows == 64)
            return launch_one<D, 2, VC, KC, K16>(dim3(plan.nsplit, units, (plan.R + 63) / 64), storage, plan, Q, ws_ml, ws_o,
                                                 out, direct, s);
    }
    return launch_one<D, 1, VC, KC, K16>(dim3(plan.nsplit, units, (plan.R + 31) / 32), storage, plan, Q, ws_ml, ws_o, out,
                                         direct, s);
}

template <int D, int KC, bool K16>
static hipError_t launch_dk(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml, float* ws_o,
                            float* out, hipStream_t s) {
    switch (plan.vcodec) {
        case 1: return launch_dv<D, 1, KC, K16>(pool, plan, Q, ws_ml, ws_o, out, s);
        case 2:
            if constexpr (D == 256) return hipErrorInvalidValue;   // not built: matrix_kernel_supports() says no
            else return launch_dv<D, 2, KC, K16>(pool, plan, Q, ws_ml, ws_o, out, s);
        case 3: return launch_dv<D, 3, KC, K16>(pool, plan, Q, ws_ml, ws_o, out, s);
        case 4: return launch_dv<D, 4, KC, K16>(pool, plan, Q, ws_ml, ws_o, out, s);
        case 5: return launch_dv<D, 5, KC, K16>(pool, plan, Q, ws_ml, ws_o, out, s);
        case 6: return launch_dv<D, 6, KC, K16>(pool, plan, Q, ws_ml, ws_o, out, s);
        default: return launch_dv<D, 0, KC, K16>(pool, plan, Q, ws_ml, ws_o, out, s);
    }
}

template <int D>
static hipError_t launch_d(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml,
                           float* ws_o, float* out, hipStream_t s) {
    if (plan.kcodec == POLYKV_KEYS_Q8_TENSOR) return launch_dk<D, 1, false>(pool, plan, Q, ws_ml, ws_o, out, s);
    // keys rounded to fp16 once dequantized (the precision of the dense cache the paper's read path holds): only
    // for the paper's value codec at head_dim 64 / 128, the shapes this option is meant for
    if (plan.key_fp16) {
        if constexpr (D != 256) {
            if (plan.vcodec == POLYKV_VALUES_TQ3) return launch_dv<D, 0, 0, true>(pool, plan, Q, ws_ml, ws_o, out, s);
        }
    }
    return launch_dk<D, 0, false>(pool, plan, Q, ws_ml, ws_o, out, s);
}

hipError_t launch_attend_matrix(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml,
                                float* ws_o, float* out, hipStream_t s) {
    if (plan.D == 128) return launch_d<128>(pool, plan, Q, ws_ml, ws_o, out, s);
    if (plan.D == 256) return launch_d<256>(pool, plan, Q, ws_ml, ws_o, out, s);
    return launch_d<64>(pool, plan, Q, ws_ml, ws_o, out, s);
}

}  // namespace polykv
