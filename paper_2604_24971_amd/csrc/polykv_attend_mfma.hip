// Matrix-core decode attention over the packed pool (gfx950, v_mfma_f32_16x16x32_f16).
//
// One wave owns up to 64 query rows (NRT tiles of 16) of one KV head and streams 32-token tile
// records.  Per tile, with tokens as the MFMA M dimension and query rows as N:
//
//   staging  a lane's share of a record (its key-code runs, its tokens' scales, its value-code
//            triplets -- every wave load one contiguous run) is loaded into registers one step ahead
//            of its use, so each load has a whole step to land.
//   pipeline two tiles are in flight per wave: the scores of the next tile are computed on the matrix
//            cores while the vector ALUs run the softmax and value dequantization of the current one.
//   scores   S^T[t, r] = sum_j sum_{k in block j} (code[t,k] * s[t,j]) * q[r,k].  The dequantized key
//            code*s has up to 18 significant bits, so it is split exactly into two fp16 terms
//            hi = fp16(code*s), lo = code*s - hi (one packed fma), each fed to one MFMA per q8_0 block
//            (K = 32 = one block) with fp32 accumulation: key dequantization stays exact.
//   softmax  online, per row, in base-2 units; the reference maximum is only raised when a row
//            exceeds it by more than 2^8, so the accumulator rescale is rare; p <= 256 fits fp16.
//   PV       O^T[v, r] += sum_t c[code[t, v]] * p[t, r]   with the score tile's accumulator layout
//            feeding the B operand directly (the value codes are stored in that k-order), centroids
//            looked up with byte permutes.  A row of ones as an extra A operand yields the softmax
//            denominator from the very same fp16-rounded p.
//
// The accumulation stays in the rotated value domain; the inverse Walsh-Hadamard rotation is done
// once per output row (sections "Compression Scheme" / "TurboQuant", dequantization), in this kernel
// when one workgroup covers the whole token range and there are no private tails, else in the merge
// kernel.  The four waves of a workgroup take interleaved tiles and are merged through LDS.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "polykv_internal.hpp"
#include "polykv_layout.hpp"

namespace polykv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

union H8 {
    half8 h;
    uint32_t u[4];
};

__device__ __forceinline__ float xor16_max(float x) {
    const uint32_t xi = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_max(float x) {
    const uint32_t xi = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}


// ---- tile staging: global -> registers, one step ahead ------------------------------------------
// A lane's share of a tile record: its 16 bytes of every key block (the two 8-code A operands), the
// scales of its two tokens, and its value-code triplets.  Every load is one contiguous, fully
// coalesced run across the wave (the record is stored in exactly this order).
template <int D> struct RawK {
    uint2 k[2][D / 32];      // [mt][j]: codes of token 16mt + n, block j, elements 8grp .. 8grp+7
    uint32_t sc[2][D / 64];  // [mt]: fp16 scales of token 16mt + n, blocks 0..NB-1
};
template <int D> struct RawV {
    uint32_t w[D / 64][3];
};

template <int D> __device__ __forceinline__ uint2 load_kraw(const uint8_t* tile, int lane, int mt, int j) {
    return *reinterpret_cast<const uint2*>(tile + j * 1024 + lane * 16 + 8 * mt);
}
template <int D> __device__ __forceinline__ uint32_t load_sc(const uint8_t* tile, int n, int mt, int x) {
    return *reinterpret_cast<const uint32_t*>(tile + Layout<D>::kscales_off + (16 * mt + n) * (D / 32) * 2 + 4 * x);
}
template <int D> __device__ __forceinline__ void load_rawk(RawK<D>& r, const uint8_t* tile, int lane) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int x = 0; x < D / 64; ++x) r.sc[mt][x] = load_sc<D>(tile, lane & 15, mt, x);
#pragma unroll
        for (int j = 0; j < D / 32; ++j) r.k[mt][j] = load_kraw<D>(tile, lane, mt, j);
    }
}
template <int D> __device__ __forceinline__ void load_rawv(RawV<D>& r, const uint8_t* tile, int lane) {
#pragma unroll
    for (int q = 0; q < D / 64; ++q)
#pragma unroll
        for (int w = 0; w < 3; ++w)
            r.w[q][w] = *reinterpret_cast<const uint32_t*>(tile + Layout<D>::vcodes_off + q * 768 + lane * 12 + 4 * w);
}

__device__ __forceinline__ float max8(const float4v& a, const float4v& b) {
    float m = fmaxf(fmaxf(a[0], a[1]), a[2]);
    m = fmaxf(fmaxf(m, a[3]), b[0]);
    m = fmaxf(fmaxf(m, b[1]), b[2]);
    return fmaxf(m, b[3]);
}

// The pool's last tile when it crosses the end of the pool, read straight from memory: scores, softmax
// and PV one after the other, tokens >= T masked out.  Runs at most once per KV head.
template <int D, int NRT>
__device__ __forceinline__ void process_ragged_tile(const uint8_t* lt, int tile, int T, float qscale, float raise_thr,
                                                 int lane, const half8 (&qb)[NRT][D / 32], float4v (&O)[D / 16][NRT],
                                                 float4v (&Lacc)[NRT], float (&m_ref)[NRT], float (&m_thr)[NRT],
                                                 float (&mneg)[NRT]) {
    using LY = Layout<D>;
    constexpr int NB = D / 32, NG = D / 16, NTR = D / 64;
    const int grp = lane >> 4, n = lane & 15;
    H8 ones;
#pragma unroll
    for (int i = 0; i < 4; ++i) ones.u[i] = 0x3C003C00u;
    float4v S[NRT][2];
#pragma unroll
    for (int nt = 0; nt < NRT; ++nt) S[nt][0] = S[nt][1] = float4v{0, 0, 0, 0};
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const _Float16 sj = *reinterpret_cast<const _Float16*>(lt + LY::kscales_off + ((16 * mt + n) * NB + j) * 2);
            const uint2 kw = *reinterpret_cast<const uint2*>(lt + j * 1024 + lane * 16 + 8 * mt);
            H8 a;
            codes4_to_half(kw.x, a.u[0], a.u[1]);
            codes4_to_half(kw.y, a.u[2], a.u[3]);
            a.h = a.h - (_Float16)1152.0f;
            const half8 sv = (half8)(sj);
            const half8 hi = a.h * sv;
            const half8 lo = __builtin_elementwise_fma(a.h, sv, -hi);
#pragma unroll
            for (int nt = 0; nt < NRT; ++nt) {
                S[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(hi, qb[nt][j], S[nt][mt], 0, 0, 0);
                S[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(lo, qb[nt][j], S[nt][mt], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (tile * kTile + 16 * mt + 4 * grp + i >= T) {
#pragma unroll
                for (int nt = 0; nt < NRT; ++nt) S[nt][mt][i] = -INFINITY;
            }
    H8 pb[NRT];
#pragma unroll
    for (int nt = 0; nt < NRT; ++nt) {
        // this path always re-references: cheap here, and it needs no vote
        const float m_new = fmaxf(m_ref[nt], xor32_max(xor16_max(max8(S[nt][0], S[nt][1]))));
        const float alpha = __builtin_amdgcn_exp2f((m_ref[nt] - m_new) * qscale);
        m_ref[nt] = m_new;
        m_thr[nt] = m_new + raise_thr;
        mneg[nt] = -m_new * qscale;
        Lacc[nt] *= alpha;
#pragma unroll
        for (int g = 0; g < NG; ++g) O[g][nt] *= alpha;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                pb[nt].h[4 * mt + i] = (_Float16)__builtin_amdgcn_exp2f(fmaf(S[nt][mt][i], qscale, mneg[nt]));
    }
#pragma unroll
    for (int q = 0; q < NTR; ++q) {
        const uint32_t* vw = reinterpret_cast<const uint32_t*>(lt + LY::vcodes_off + q * 768 + lane * 12);
        const uint32_t w0 = vw[0], w1 = vw[1], w2 = vw[2];
#pragma unroll
        for (int gi = 0; gi < 4; ++gi) {
            uint32_t sel_a, sel_b;
            if (gi < 3) {
                const uint32_t w = gi == 0 ? w0 : gi == 1 ? w1 : w2;
                sel_a = w & 0x07070707u;
                sel_b = (w >> 3) & 0x07070707u;
            } else {
                sel_a = ((w0 >> 6) & 0x03030303u) | ((w1 >> 4) & 0x04040404u);
                sel_b = ((w2 >> 6) & 0x03030303u) | ((w1 >> 5) & 0x04040404u);
            }
            H8 va;
            lookup4(sel_a, va.u[0], va.u[1]);
            lookup4(sel_b, va.u[2], va.u[3]);
#pragma unroll
            for (int nt = 0; nt < NRT; ++nt)
                O[4 * q + gi][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, pb[nt].h, O[4 * q + gi][nt], 0, 0, 0);
        }
    }
#pragma unroll
    for (int nt = 0; nt < NRT; ++nt)
        Lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones.h, pb[nt].h, Lacc[nt], 0, 0, 0);
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
//   Sa         scores of tile A on entry, of tile B on exit; mloc / raise: per-lane row maxima of the
//              same tile and whether some row outgrew the reference
// Only full tiles go through here; a ragged last tile is handled by process_ragged_tile.
template <int D, int NRT, bool HAS_A, bool HAS_B>
__device__ __forceinline__ void pipeline_step(const RawV<D>& rv, const RawK<D>& rk, RawV<D>& rvN, RawK<D>& rkN,
                                              const uint8_t* nextK, const uint8_t* nextV, float qscale,
                                              float raise_thr, int lane, const half8 (&qb)[NRT][D / 32],
                                              float4v (&O)[D / 16][NRT], float4v (&Lacc)[NRT], float (&m_ref)[NRT],
                                              float (&m_thr)[NRT], float (&mneg)[NRT], float4v (&Sa)[NRT][2],
                                              float (&mloc)[NRT], bool& raise) {
    using LY = Layout<D>;
    constexpr int NB = D / 32, NG = D / 16, NTR = D / 64;
    const int n = lane & 15;
    const half8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    H8 ones;
#pragma unroll
    for (int i = 0; i < 4; ++i) ones.u[i] = 0x3C003C00u;
    float4v Sb[NRT][2];

    if (HAS_A && __builtin_expect(__any(raise), 0)) {
        // Rare: a row of tile A outgrew the softmax reference by more than 2^8.  The accumulators live
        // in accumulation registers that vector instructions cannot read; an MFMA with zero operands
        // (D = 0*0 + C) carries them to vector registers and back, so the hot path never copies them.
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) {
            const float m_new = fmaxf(m_ref[nt], xor32_max(xor16_max(mloc[nt])));
            const float alpha = __builtin_amdgcn_exp2f((m_ref[nt] - m_new) * qscale);
            m_ref[nt] = m_new;
            m_thr[nt] = m_new + raise_thr;
            mneg[nt] = -m_new * qscale;
            float4v x = __builtin_amdgcn_mfma_f32_16x16x32_f16(zero8, zero8, Lacc[nt], 0, 0, 0);
            x *= alpha;
            Lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(zero8, zero8, x, 0, 0, 0);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                float4v y = __builtin_amdgcn_mfma_f32_16x16x32_f16(zero8, zero8, O[g][nt], 0, 0, 0);
                y *= alpha;
                O[g][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(zero8, zero8, y, 0, 0, 0);
            }
        }
    }

    // The step is written as a sequence of slices.  Each slice pairs a batch of MFMAs whose operands
    // are ready with the vector work that prepares the operands of the NEXT batch, and is closed by a
    // scheduling barrier so that the compiler keeps the pairing; inside a slice the two streams are
    // interleaved one MFMA to a few vector instructions.
    constexpr int NQK = 2 * NB;     // key blocks of tile B: (mt, j)
    constexpr int NCH = 2 * NRT;    // probability chunks of tile A: 4 scores each
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

    // The next step's bytes are requested first thing, into the other set of registers, so that every
    // load has the whole step (and more, for all but the first key block) to land.
    if (HAS_B) load_rawk<D>(rkN, nextK, lane);
    load_rawv<D>(rvN, nextV, lane);
    __builtin_amdgcn_sched_barrier(0);

    H8 pb[NRT];
    half8 khi[2], klo[2];
    H8 va[2];
    auto exp_chunk = [&](int c) {  // probabilities of tile A: 4 of them, fp16, B operand of the PV products
        const int nt = c >> 1, mt = c & 1;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            pb[nt].h[4 * mt + i] = (_Float16)__builtin_amdgcn_exp2f(fmaf(Sa[nt][mt][i], qscale, mneg[nt]));
    };
    auto kdeq = [&](int k) {  // key block k of tile B: code * scale split exactly into hi + lo fp16 terms
        const int mt = k / NB, j = k % NB;
        H8 a;
        codes4_to_half(rk.k[mt][j].x, a.u[0], a.u[1]);
        codes4_to_half(rk.k[mt][j].y, a.u[2], a.u[3]);
        a.h = a.h - (_Float16)1152.0f;
        union {
            uint32_t u;
            _Float16 h[2];
        } s2;
        s2.u = rk.sc[mt][j >> 1];
        const half8 sv = (half8)(s2.h[j & 1]);
        khi[k & 1] = a.h * sv;
        klo[k & 1] = __builtin_elementwise_fma(a.h, sv, -khi[k & 1]);  // exact remainder of the product
    };
    auto qk = [&](int k) {
        const int mt = k / NB, j = k % NB;
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt)
            Sb[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(khi[k & 1], qb[nt][j], Sb[nt][mt], 0, 0, 0);
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt)
            Sb[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(klo[k & 1], qb[nt][j], Sb[nt][mt], 0, 0, 0);
    };
    auto vdeq = [&](int g) {  // value group g of tile A: eight 3-bit codes -> fp16 centroids (A operand)
        const int q = g >> 2, gi = g & 3;
        const uint32_t w0 = rv.w[q][0], w1 = rv.w[q][1], w2 = rv.w[q][2];
        uint32_t sel_a, sel_b;
        if (gi < 3) {
            const uint32_t w = gi == 0 ? w0 : gi == 1 ? w1 : w2;
            sel_a = w & 0x07070707u;
            sel_b = (w >> 3) & 0x07070707u;
        } else {
            sel_a = ((w0 >> 6) & 0x03030303u) | ((w1 >> 4) & 0x04040404u);
            sel_b = ((w2 >> 6) & 0x03030303u) | ((w1 >> 5) & 0x04040404u);
        }
        lookup4(sel_a, va[g & 1].u[0], va[g & 1].u[1]);
        lookup4(sel_b, va[g & 1].u[2], va[g & 1].u[3]);
    };
    auto pv = [&](int g) {
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt)
            O[g][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va[g & 1].h, pb[nt].h, O[g][nt], 0, 0, 0);
    };

    if (HAS_B) {
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) Sb[nt][0] = Sb[nt][1] = float4v{0, 0, 0, 0};
        // lead-in: vector work only, while the LDS reads land
        if (HAS_A) {
#pragma unroll
            for (int c = 0; c < NCH / NQK; ++c) exp_chunk(c);
        }
        kdeq(0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < NQK; ++k) {
            qk(k);
            if (k + 1 < NQK) kdeq(k + 1);
            if (HAS_A) {
                // spread the remaining probability chunks over the score slices
                const int c0 = NCH / NQK + (k * (NCH - NCH / NQK)) / NQK, c1 = NCH / NQK + ((k + 1) * (NCH - NCH / NQK)) / NQK;
#pragma unroll
                for (int c = c0; c < c1; ++c) exp_chunk(c);
                if (k + 1 == NQK) vdeq(0);
            }
            slice_end(integral_constant<int, 2 * NRT>{}, integral_constant<int, (HAS_A ? 28 : 16)>{});
        }
    } else if (HAS_A) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) exp_chunk(c);
        vdeq(0);
        __builtin_amdgcn_sched_barrier(0);
    }

    if (HAS_A) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            pv(g);
            if (g + 1 < NG) vdeq(g + 1);
            slice_end(integral_constant<int, NRT>{}, integral_constant<int, 16>{});
        }
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt)
            Lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones.h, pb[nt].h, Lacc[nt], 0, 0, 0);
    }

    // ---- row maxima of tile B for the next step's vote (no cross-lane reduction needed for the vote)
    if (HAS_B) {
        raise = false;
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) {
            // the scores are consumed by vector instructions only: have the MFMAs deliver them there
            asm volatile("" : "+v"(Sb[nt][0]), "+v"(Sb[nt][1]));
            mloc[nt] = max8(Sb[nt][0], Sb[nt][1]);
            raise |= mloc[nt] > m_thr[nt];  // also true while the reference is -inf
            Sa[nt][0] = Sb[nt][0];
            Sa[nt][1] = Sb[nt][1];
        }
    }
    if (HAS_A) slice_end(integral_constant<int, NRT>{}, integral_constant<int, 24>{});
}

template <int D, int NRT>
__global__ __launch_bounds__(256) void attend_mfma_kernel(const uint8_t* __restrict__ pool,
                                                          const __half* __restrict__ Q,
                                                          float* __restrict__ ws_ml, float* __restrict__ ws_o,
                                                          float* __restrict__ out, AttendPlan p, int direct) {
    using LY = Layout<D>;
    constexpr int NB = D / 32, NG = D / 16, ROWS = 16 * NRT;
    constexpr int OSTRIDE = D + 4;
    constexpr int TB = LY::tile_bytes;
    __shared__ float m_s[4][ROWS];
    __shared__ float l_s[2 * ROWS];
    extern __shared__ __align__(16) float o_s[];  // two merge buffers of ROWS x OSTRIDE floats

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: LDS bases go through M0
    const int grp = lane >> 4, n = lane & 15;
    const int usel = blockIdx.y, ls = usel / p.H, kvh = usel - ls * p.H;
    const int row0 = blockIdx.z * ROWS;
    const int split = blockIdx.x;
    const int tps = (p.tiles + p.nsplit - 1) / p.nsplit;
    const int t_begin = split * tps, t_end = min(p.tiles, t_begin + tps);
    const uint8_t* unit_base = pool + (size_t)((p.layer_begin + ls) * p.H + kvh) * p.tiles * TB;
    const float qscale = p.qscale;

    // this wave's tiles: t_begin + wave, +4, +8, ...; local index k <-> tile my_first + 4k
    const int my_first = t_begin + wave;
    const int my_count = my_first < t_end ? (t_end - my_first + 3) / 4 : 0;
    // pointer to local tile k; k past the end is clamped (the refill loads of the last steps then
    // fetch the wave's own last tile again, harmlessly, instead of needing a branch per load)
    auto tile_ptr = [&](int k) { return unit_base + (size_t)(my_first + 4 * min(k, max(my_count - 1, 0))) * TB; };
    RawK<D> rk;
    RawV<D> rv;
    if (my_count > 0) {
        load_rawk<D>(rk, tile_ptr(0), lane);
        load_rawv<D>(rv, tile_ptr(0), lane);
    }

    // ---- query rows as MFMA B operands: lane (n, grp) holds q[row 16nt+n][32j + 8grp .. +7]
    half8 qb[NRT][NB];
#pragma unroll
    for (int nt = 0; nt < NRT; ++nt) {
        const int r = row0 + 16 * nt + n;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            H8 t;
            uint4v raw = {0, 0, 0, 0};
            if (r < p.R) raw = *reinterpret_cast<const uint4v*>(Q + q_row_index(p, ls, kvh, r) * D + 32 * j + 8 * grp);
            t.u[0] = raw.x; t.u[1] = raw.y; t.u[2] = raw.z; t.u[3] = raw.w;
            qb[nt][j] = t.h;
            // The queries are only ever MFMA operands: park them in accumulation registers so that the
            // vector registers are left for the scores and the dequantization temporaries.
            asm volatile("" : "+a"(qb[nt][j]));
        }
    }

    float4v O[NG][NRT], Lacc[NRT];
    float m_ref[NRT], m_thr[NRT], mneg[NRT], mloc[NRT];
#pragma unroll
    for (int nt = 0; nt < NRT; ++nt) {
        m_ref[nt] = -INFINITY;
        m_thr[nt] = -INFINITY;
        mneg[nt] = 0.0f;
        mloc[nt] = -INFINITY;
        Lacc[nt] = float4v{0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < NG; ++g) O[g][nt] = float4v{0, 0, 0, 0};
    }
    const float raise_thr = 8.0f / qscale;  // raise the reference only when a row exceeds it by 2^8
    bool raise = false;
    float4v S[NRT][2];  // scores of the tile whose softmax comes next

    // Local tile k is "B" in step k-1 (scores) and "A" in step k (softmax, PV).  Only the pool's very
    // last tile can be ragged; it stays out of the pipeline and goes last.
    const bool last_ragged = my_count > 0 && (my_first + 4 * (my_count - 1)) * kTile + kTile > p.T;
    const int full_count = last_ragged ? my_count - 1 : my_count;
    if (full_count > 0) {
        // register sets: (rk, rv) and (rk2, rv2) alternate between "current" and "being loaded"
        RawK<D> rk2;
        RawV<D> rv2;
        // prologue: scores of tile 0 from rk; requests K of tile 1 and (again) V of tile 0 into set 2
        pipeline_step<D, NRT, false, true>(rv, rk, rv2, rk2, tile_ptr(1), tile_ptr(0), qscale, raise_thr, lane, qb, O, Lacc,
                                           m_ref, m_thr, mneg, S, mloc, raise);
        int s = 0;
        for (; s + 1 < full_count - 1; s += 2) {  // two steps per trip: the sets swap roles without copies
            pipeline_step<D, NRT, true, true>(rv2, rk2, rv, rk, tile_ptr(s + 2), tile_ptr(s + 1), qscale, raise_thr, lane, qb,
                                              O, Lacc, m_ref, m_thr, mneg, S, mloc, raise);
            pipeline_step<D, NRT, true, true>(rv, rk, rv2, rk2, tile_ptr(s + 3), tile_ptr(s + 2), qscale, raise_thr, lane, qb,
                                              O, Lacc, m_ref, m_thr, mneg, S, mloc, raise);
        }
        if (s < full_count - 1) {  // one step with a B tile left: current = set 2
            pipeline_step<D, NRT, true, true>(rv2, rk2, rv, rk, tile_ptr(s + 2), tile_ptr(s + 1), qscale, raise_thr, lane, qb,
                                              O, Lacc, m_ref, m_thr, mneg, S, mloc, raise);
            pipeline_step<D, NRT, true, false>(rv, rk, rv2, rk2, tile_ptr(s + 2), tile_ptr(s + 2), qscale, raise_thr, lane, qb,
                                               O, Lacc, m_ref, m_thr, mneg, S, mloc, raise);
        } else {
            pipeline_step<D, NRT, true, false>(rv2, rk2, rv, rk, tile_ptr(s + 1), tile_ptr(s + 1), qscale, raise_thr, lane, qb,
                                               O, Lacc, m_ref, m_thr, mneg, S, mloc, raise);
        }
    }
    if (last_ragged)
        process_ragged_tile<D, NRT>(tile_ptr(my_count - 1), my_first + 4 * (my_count - 1), p.T, qscale, raise_thr, lane, qb, O,
                                    Lacc, m_ref, m_thr, mneg);

    // ---- merge the four waves through LDS: waves 0 and 2 store their (rescaled) accumulators into
    // two buffers, waves 1 and 3 add theirs on top, the final pass sums the two buffers.  The order of
    // the additions is fixed, so the result is reproducible.
    if (grp == 0) {
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) m_s[wave][16 * nt + n] = m_ref[nt];
    }
    __syncthreads();
    float* obuf = o_s + (wave >> 1) * (ROWS * OSTRIDE);
    float* lbuf = l_s + (wave >> 1) * ROWS;
    for (int round = 0; round < 2; ++round) {
        if ((wave & 1) == round) {
#pragma unroll
            for (int nt = 0; nt < NRT; ++nt) {
                const int r = 16 * nt + n;
                const float M = fmaxf(fmaxf(m_s[0][r], m_s[1][r]), fmaxf(m_s[2][r], m_s[3][r]));
                const float f = m_ref[nt] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f((m_ref[nt] - M) * qscale);
                if (grp == 0) lbuf[r] = (round == 0 ? 0.0f : lbuf[r]) + Lacc[nt][0] * f;
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    float4* dst = reinterpret_cast<float4*>(&obuf[r * OSTRIDE + 16 * g + 4 * grp]);
                    float4 v = round == 0 ? make_float4(0.0f, 0.0f, 0.0f, 0.0f) : *dst;
                    v.x = fmaf(O[g][nt][0], f, v.x);
                    v.y = fmaf(O[g][nt][1], f, v.y);
                    v.z = fmaf(O[g][nt][2], f, v.z);
                    v.w = fmaf(O[g][nt][3], f, v.w);
                    *dst = v;
                }
            }
        }
        __syncthreads();
    }

    constexpr int EPL = D / 64;
    for (int rr = wave; rr < ROWS; rr += 4) {
        const int r = row0 + rr;
        if (r >= p.R) break;  // uniform over the wave
        const float Mr = fmaxf(fmaxf(m_s[0][rr], m_s[1][rr]), fmaxf(m_s[2][rr], m_s[3][rr]));
        const float l = l_s[rr] + l_s[ROWS + rr];
        float x[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i)
            x[i] = (o_s[rr * OSTRIDE + lane * EPL + i] + o_s[(ROWS + rr) * OSTRIDE + lane * EPL + i]) * kInvCentroidScale;
        if (direct) {
            const float inv = 1.0f / l;
#pragma unroll
            for (int i = 0; i < EPL; ++i) x[i] *= inv;
            wht_inlane<EPL>(x);
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                x[i] = wht_lane_stage<1>(x[i], lane);
                x[i] = wht_lane_stage<2>(x[i], lane);
                x[i] = wht_lane_stage<4>(x[i], lane);
                x[i] = wht_lane_stage<8>(x[i], lane);
                x[i] = wht_lane_stage<16>(x[i], lane);
                x[i] = wht_lane_stage<32>(x[i], lane);
                x[i] *= (D == 64 ? 0.125f : 0.08838834764831845f);
            }
            float* dst = out + q_row_index(p, ls, kvh, r) * D + lane * EPL;
#pragma unroll
            for (int i = 0; i < EPL; ++i) dst[i] = x[i];
        } else {
            const size_t prow = ((size_t)usel * p.nsplit + split) * p.R + r;
#pragma unroll
            for (int i = 0; i < EPL; ++i) ws_o[prow * D + lane * EPL + i] = x[i];
            if (lane == 0) {
                ws_ml[prow * 2] = Mr * qscale;
                ws_ml[prow * 2 + 1] = l;
            }
        }
    }
}

bool matrix_kernel_supports(int head_dim, int rows_per_kv_head) {
    return (head_dim == 64 || head_dim == 128) && rows_per_kv_head >= 1;
}

bool matrix_kernel_direct(const AttendPlan& plan) { return plan.nsplit == 1 && !plan.has_tails; }

template <int D, int NRT>
static hipError_t launch_one(dim3 grid, const uint8_t* storage, const AttendPlan& plan, const void* Q, float* ws_ml,
                             float* ws_o, float* out, int direct, hipStream_t s) {
    constexpr int kMergeBytes = 2 * 16 * NRT * (D + 4) * (int)sizeof(float);
    auto kern = attend_mfma_kernel<D, NRT>;
    static bool configured = false;  // per instantiation: the limit is a property of the function
    if (!configured && kMergeBytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMergeBytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kern<<<grid, 256, kMergeBytes, s>>>(storage, (const __half*)Q, ws_ml, ws_o, out, plan, direct);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml,
                           float* ws_o, float* out, hipStream_t s) {
    const uint8_t* storage = reinterpret_cast<const uint8_t*>(pool->storage);
    const int units = plan.layers * plan.H;
    const int direct = matrix_kernel_direct(plan) ? 1 : 0;
    if (plan.R <= 16) return launch_one<D, 1>(dim3(plan.nsplit, units, 1), storage, plan, Q, ws_ml, ws_o, out, direct, s);
    if (plan.R <= 32) return launch_one<D, 2>(dim3(plan.nsplit, units, 1), storage, plan, Q, ws_ml, ws_o, out, direct, s);
    return launch_one<D, 4>(dim3(plan.nsplit, units, (plan.R + 63) / 64), storage, plan, Q, ws_ml, ws_o, out, direct, s);
}

hipError_t launch_attend_matrix(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml,
                                float* ws_o, float* out, hipStream_t s) {
    if (plan.D == 128) return launch_d<128>(pool, plan, Q, ws_ml, ws_o, out, s);
    return launch_d<64>(pool, plan, Q, ws_ml, ws_o, out, s);
}

}  // namespace polykv
