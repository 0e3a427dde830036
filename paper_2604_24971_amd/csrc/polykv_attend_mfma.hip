// Matrix-core decode attention over the packed pool (gfx950, v_mfma_f32_16x16x32_f16).
//
// One wave owns up to 64 query rows (NRT tiles of 16) of one KV head and streams 32-token tile
// records.  Per tile, with tokens as the MFMA M dimension and query rows as N:
//
//   scores   S^T[t, r] = sum_j s[t, j] * (codes_j[t, :] . q_j[r, :])     one MFMA per q8_0 block j
//            (K = 32 = one block): int8 codes are exact in fp16, the product is accumulated in fp32
//            and multiplied by the block scale in fp32 afterwards, so key dequantization is exact.
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

// Centroids scaled by kCentroidScale and rounded to fp16.  The factor was searched in [1, 2) so that
// all four magnitudes land within 1.9e-5 (relative) of an fp16 value -- ten times closer than the
// unscaled centroids; it is divided out once per output row.
constexpr float kCentroidScale = 1.6146639585494995f;
constexpr float kInvCentroidScale = 0.6193239123875222f;
// fp16 bit patterns by code 0..7: C2F3 C057 BCE2 B655 3655 3CE2 4057 42F3, split into byte planes
constexpr uint32_t kTabLoA = 0x55E257F3u, kTabLoB = 0xF357E255u;  // low bytes of codes 0..3 / 4..7
constexpr uint32_t kTabHiA = 0xB6BCC0C2u, kTabHiB = 0x42403C36u;  // high bytes

// Four 3-bit codes sitting in the four bytes of `sel` -> four fp16 centroids (two dwords).
__device__ __forceinline__ void lookup4(uint32_t sel, uint32_t& out01, uint32_t& out23) {
    const uint32_t lo = __builtin_amdgcn_perm(kTabLoB, kTabLoA, sel);
    const uint32_t hi = __builtin_amdgcn_perm(kTabHiB, kTabHiA, sel);
    out01 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
    out23 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
}

// Four offset-binary key codes in a dword -> four exact fp16 integers: 0x6400 | b is 1024 + b.
__device__ __forceinline__ void codes4_to_half(uint32_t w, uint32_t& out01, uint32_t& out23) {
    out01 = __builtin_amdgcn_perm(0x64646464u, w, 0x04010400u);
    out23 = __builtin_amdgcn_perm(0x64646464u, w, 0x04030402u);
}

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

template <int D> struct RawTile {
    static constexpr int NB = D / 32, NTR = D / 64, SCV = NB / 2;  // SCV: 16-byte scale vectors per 16 tokens
    uint4v k[NB];
    union {
        uint4v v[2][SCV];
        _Float16 h[2][4 * NB];  // [mt][4 tokens x NB blocks]
    } sc;
    uint32_t v[NTR][3];
};

template <int D>
__device__ __forceinline__ void load_tile(RawTile<D>& rt, const uint8_t* tb, int lane, int grp) {
    using LY = Layout<D>;
    constexpr int NB = D / 32;
#pragma unroll
    for (int j = 0; j < NB; ++j) rt.k[j] = *reinterpret_cast<const uint4v*>(tb + j * 1024 + lane * 16);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int x = 0; x < RawTile<D>::SCV; ++x)
            rt.sc.v[mt][x] = *reinterpret_cast<const uint4v*>(tb + LY::kscales_off + (16 * mt + 4 * grp) * NB * 2 + 16 * x);
#pragma unroll
    for (int q = 0; q < RawTile<D>::NTR; ++q)
#pragma unroll
        for (int w = 0; w < 3; ++w)
            rt.v[q][w] = *reinterpret_cast<const uint32_t*>(tb + LY::vcodes_off + q * 768 + lane * 12 + 4 * w);
}

template <int D, int NRT>
__global__ __launch_bounds__(256) void attend_mfma_kernel(const uint8_t* __restrict__ pool,
                                                          const __half* __restrict__ Q,
                                                          float* __restrict__ ws_ml, float* __restrict__ ws_o,
                                                          float* __restrict__ out, AttendPlan p, int direct) {
    using LY = Layout<D>;
    constexpr int NB = D / 32, NG = D / 16, NTR = D / 64, ROWS = 16 * NRT;
    constexpr int OSTRIDE = D + 4;
    __shared__ float m_s[4][ROWS];
    __shared__ float l_s[ROWS];
    __shared__ __align__(16) float o_s[ROWS * OSTRIDE];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int grp = lane >> 4, n = lane & 15;
    const int usel = blockIdx.y, ls = usel / p.H, kvh = usel - ls * p.H;
    const int row0 = blockIdx.z * ROWS;
    const int split = blockIdx.x;
    const int tps = (p.tiles + p.nsplit - 1) / p.nsplit;
    const int t_begin = split * tps, t_end = min(p.tiles, t_begin + tps);
    const uint8_t* unit_base = pool + (size_t)((p.layer_begin + ls) * p.H + kvh) * p.tiles * LY::tile_bytes;
    const float qscale = p.qscale;

    for (int i = tid; i < ROWS * OSTRIDE; i += 256) o_s[i] = 0.0f;
    if (tid < ROWS) l_s[tid] = 0.0f;

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
        }
    }

    float4v O[NG][NRT], Lacc[NRT];
    float m_ref[NRT];
#pragma unroll
    for (int nt = 0; nt < NRT; ++nt) {
        m_ref[nt] = -INFINITY;
        Lacc[nt] = float4v{0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < NG; ++g) O[g][nt] = float4v{0, 0, 0, 0};
    }
    H8 ones;
#pragma unroll
    for (int i = 0; i < 4; ++i) ones.u[i] = 0x3C003C00u;
    const float raise_thr = 8.0f / qscale;  // raise the reference only when a row exceeds it by 2^8

    RawTile<D> cur, nxt;
    int tile = t_begin + wave;
    if (tile < t_end) load_tile<D>(cur, unit_base + (size_t)tile * LY::tile_bytes, lane, grp);

    for (; tile < t_end; tile += 4) {
        const int tile_n = tile + 4;
        if (tile_n < t_end) load_tile<D>(nxt, unit_base + (size_t)tile_n * LY::tile_bytes, lane, grp);

        // ---- scores
        float4v S[NRT][2];
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) S[nt][0] = S[nt][1] = float4v{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const uint32_t kw[4] = {cur.k[j].x, cur.k[j].y, cur.k[j].z, cur.k[j].w};
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                H8 a;
                codes4_to_half(kw[2 * mt], a.u[0], a.u[1]);
                codes4_to_half(kw[2 * mt + 1], a.u[2], a.u[3]);
                a.h = a.h - (_Float16)1152.0f;
#pragma unroll
                for (int nt = 0; nt < NRT; ++nt) {
                    const float4v X = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, qb[nt][j], float4v{0, 0, 0, 0}, 0, 0, 0);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        S[nt][mt][i] = fmaf(X[i], (float)cur.sc.h[mt][i * NB + j], S[nt][mt][i]);
                }
            }
        }
        if (tile * kTile + kTile > p.T) {  // ragged last tile: tokens past the end never score
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (tile * kTile + 16 * mt + 4 * grp + i >= p.T) {
#pragma unroll
                        for (int nt = 0; nt < NRT; ++nt) S[nt][mt][i] = -INFINITY;
                    }
        }

        // ---- online softmax
        float mx[NRT];
        bool raise = false;
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) {
            float m = fmaxf(fmaxf(S[nt][0][0], S[nt][0][1]), fmaxf(S[nt][0][2], S[nt][0][3]));
            m = fmaxf(m, fmaxf(fmaxf(S[nt][1][0], S[nt][1][1]), fmaxf(S[nt][1][2], S[nt][1][3])));
            m = xor32_max(xor16_max(m));
            mx[nt] = m;
            raise |= m > m_ref[nt] + raise_thr;   // also true while m_ref is -inf
        }
        if (__any(raise)) {
#pragma unroll
            for (int nt = 0; nt < NRT; ++nt) {
                const float m_new = fmaxf(m_ref[nt], mx[nt]);
                const float alpha = __builtin_amdgcn_exp2f((m_ref[nt] - m_new) * qscale);
                m_ref[nt] = m_new;
                Lacc[nt] *= alpha;
#pragma unroll
                for (int g = 0; g < NG; ++g) O[g][nt] *= alpha;
            }
        }
        H8 pb[NRT];
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) {
            const float mneg = -m_ref[nt] * qscale;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    pb[nt].h[4 * mt + i] = (_Float16)__builtin_amdgcn_exp2f(fmaf(S[nt][mt][i], qscale, mneg));
        }

        // ---- PV in the rotated domain
#pragma unroll
        for (int q = 0; q < NTR; ++q) {
            const uint32_t w0 = cur.v[q][0], w1 = cur.v[q][1], w2 = cur.v[q][2];
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

        cur = nxt;
    }

    // ---- merge the four waves through LDS
    if (grp == 0) {
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) m_s[wave][16 * nt + n] = m_ref[nt];
    }
    __syncthreads();
    // waves add their share one after the other, so the summation order (and the result) is fixed
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int nt = 0; nt < NRT; ++nt) {
                const int r = 16 * nt + n;
                const float M = fmaxf(fmaxf(m_s[0][r], m_s[1][r]), fmaxf(m_s[2][r], m_s[3][r]));
                const float f = m_ref[nt] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f((m_ref[nt] - M) * qscale);
                if (grp == 0) l_s[r] += Lacc[nt][0] * f;
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    float4* dst = reinterpret_cast<float4*>(&o_s[r * OSTRIDE + 16 * g + 4 * grp]);
                    float4 v = *dst;
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
        const float l = l_s[rr];
        float x[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) x[i] = o_s[rr * OSTRIDE + lane * EPL + i] * kInvCentroidScale;
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

template <int D>
static hipError_t launch_d(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml,
                           float* ws_o, float* out, hipStream_t s) {
    const uint8_t* storage = reinterpret_cast<const uint8_t*>(pool->storage);
    const int units = plan.layers * plan.H;
    const int direct = matrix_kernel_direct(plan) ? 1 : 0;
    if (plan.R <= 16) {
        dim3 grid(plan.nsplit, units, 1);
        attend_mfma_kernel<D, 1><<<grid, 256, 0, s>>>(storage, (const __half*)Q, ws_ml, ws_o, out, plan, direct);
    } else if (plan.R <= 32) {
        dim3 grid(plan.nsplit, units, 1);
        attend_mfma_kernel<D, 2><<<grid, 256, 0, s>>>(storage, (const __half*)Q, ws_ml, ws_o, out, plan, direct);
    } else {
        dim3 grid(plan.nsplit, units, (plan.R + 63) / 64);
        attend_mfma_kernel<D, 4><<<grid, 256, 0, s>>>(storage, (const __half*)Q, ws_ml, ws_o, out, plan, direct);
    }
    return hipGetLastError();
}

hipError_t launch_attend_matrix(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml,
                                float* ws_o, float* out, hipStream_t s) {
    if (plan.D == 128) return launch_d<128>(pool, plan, Q, ws_ml, ws_o, out, s);
    return launch_d<64>(pool, plan, Q, ws_ml, ws_o, out, s);
}

}  // namespace polykv
