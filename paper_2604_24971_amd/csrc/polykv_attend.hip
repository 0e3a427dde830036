// Decode attention of all agents' query rows over the packed pool (gfx950): vector (VALU) kernel,
// private-tail kernel and the merge / inverse-rotation kernel.
//
// The pool part is accumulated in the ROTATED value domain: acc[r,:] = sum_t p[r,t] * c[code[t,:]].
// Because the inverse rotation is linear, it is applied once per output row in the merge kernel
// instead of once per pool token (sections "Compression Scheme" / "TurboQuant", dequantization).
// Scores are kept in base-2 units (q is pre-multiplied by scale*log2 e) so exp2 is the only
// transcendental.  Every split of the token range emits a partial (m, l, acc) per row; the merge
// kernel combines them with log-sum-exp weights, rotates back, and folds in the agent's private
// tail partial, which lives in the un-rotated domain.
#include <hip/hip_fp16.h>

#include "polykv_internal.hpp"
#include "polykv_layout.hpp"

namespace polykv {

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
}

constexpr int kRB = 4;  // query rows per pass of the vector kernels

template <int N> struct __attribute__((aligned(2 * N))) HalfVecN { __half h[N]; };

// ---------------------------------------------------------------------------- vector kernel ---
// One wave = one token-range split of one (layer, kv head, block of kRB rows).  Per 64 tokens:
//   scores  lane = token: the lane dequantizes its key (code * block scale, exact in fp32) and dots
//           it with each row's query (LDS broadcast);
//   softmax running max / sum per row across the wave;
//   PV      lane = (half h, coordinate m) exactly as the value codes are stored: the lane owns the
//           codes of 16 of the tile's tokens for coordinates 32*g + m and accumulates its share;
//           the two lane halves are added once at the end.
template <int D, int VC, int KC>
__global__ __launch_bounds__(256) void attend_vector_kernel(const uint8_t* __restrict__ pool,
                                                            const __half* __restrict__ Q,
                                                            float* __restrict__ ws_ml,
                                                            float* __restrict__ ws_o, AttendPlan p) {
    using LY = Layout<D, VC, KC>;
    constexpr int VB = vc_bits(VC);
    constexpr bool VS = LY::has_vscales, V8 = VB == 8;
    constexpr int MT = D / 32;
    __shared__ __align__(16) float q_s[kRB][D];
    __shared__ __align__(16) float p_s[4][kRB][64];
    __shared__ float ctab[16];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int usel = blockIdx.y;  // selected unit: ls * H + kvh
    const int ls = usel / p.H, kvh = usel - ls * p.H;
    const int r0 = blockIdx.z * kRB;
    const int sp = blockIdx.x * 4 + wave;

    for (int i = tid; i < kRB * D; i += 256) {
        const int r = i / D, jj = i - r * D;
        float v = 0.0f;
        if (r0 + r < p.R)
            v = bits16_to_float(reinterpret_cast<const uint16_t*>(Q)[q_row_index(p, ls, kvh, r0 + r) * D + jj], p.io_bf16) *
                p.qscale;
        q_s[r][jj] = v;
    }
    if (VB == 3 && tid < 8) ctab[tid] = centroid_of(tid);
    if ((VB == 2 || VB == 4) && tid < (1 << VB)) ctab[tid] = centroid_signmag(VB, tid);  // sign-magnitude codes
    __syncthreads();

    const int nchunks = (p.tiles + 1) / 2;
    const int cps = (nchunks + p.nsplit - 1) / p.nsplit;
    const int c_begin = sp * cps, c_end = min(nchunks, c_begin + cps);
    const uint8_t* unit_base = pool + (size_t)((p.layer_begin + ls) * p.H + kvh) * p.tiles_cap * LY::tile_bytes;

    float m_run[kRB], l_run[kRB], acc[kRB][MT];
#pragma unroll
    for (int r = 0; r < kRB; ++r) {
        m_run[r] = -INFINITY;
        l_run[r] = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[r][mt] = 0.0f;
    }
    const int hh = lane >> 5, cc = lane & 31;   // scores: which tile of the pair, token in the tile
    const int vh = lane >> 5, mm = lane & 31;   // PV: position of the lane in the value-code layout

    for (int ch = c_begin; ch < c_end; ++ch) {
        // ---- scores, lane = token
        {
            const int tile = ch * 2 + hh, tl = cc;
            const bool valid = tile < p.tiles && tile * kTile + tl < p.T;
            const uint8_t* tb = unit_base + (size_t)min(tile, p.tiles - 1) * LY::tile_bytes;
            float k[D];
            const __half* sc = reinterpret_cast<const __half*>(tb + LY::kscales_off) + tl * LY::NB;
            const float s_tensor = KC == 1 ? (float)tensor_key_scale(p.kmax[p.layer_begin + ls]) : 0.0f;
            // codecs with a per-vector value scale: it rides on the token's probability in the P.V sum
            const float vscale = VS ? __half2float(reinterpret_cast<const __half*>(tb + LY::vscales_off)[tl]) : 1.0f;
#pragma unroll
            for (int j = 0; j < LY::NB; ++j) {
                const float s = KC == 1 ? s_tensor : __half2float(sc[j]);
#pragma unroll
                for (int g8 = 0; g8 < 4; ++g8) {
                    const uint2 raw = *reinterpret_cast<const uint2*>(tb + kcode_run_offset(tl, j, g8));
                    const uint32_t w[2] = {raw.x, raw.y};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        k[32 * j + 8 * g8 + e] = (float)((int)((w[e >> 2] >> (8 * (e & 3))) & 0xFF) - 128) * s;
                }
            }
#pragma unroll
            for (int r = 0; r < kRB; ++r) {
                float s = 0.0f;
#pragma unroll
                for (int jj = 0; jj < D; jj += 4) {
                    const float4 qv = *reinterpret_cast<const float4*>(&q_s[r][jj]);
                    s = fmaf(qv.x, k[jj], s);
                    s = fmaf(qv.y, k[jj + 1], s);
                    s = fmaf(qv.z, k[jj + 2], s);
                    s = fmaf(qv.w, k[jj + 3], s);
                }
                s = valid ? s : -INFINITY;
                const float m_new = fmaxf(m_run[r], wave_max(s));  // finite: every chunk has a valid token
                const float alpha = exp2f(m_run[r] - m_new);
                const float pr = exp2f(s - m_new);
                l_run[r] = l_run[r] * alpha + wave_sum(pr);
                m_run[r] = m_new;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[r][mt] *= alpha;
                p_s[wave][r][lane] = VS ? pr * vscale : pr;
            }
        }
        // ---- PV, lane = (h, c) of the stored value codes; p_s is private to the wave
        for (int sub = 0; sub < 2; ++sub) {
            const int tile = ch * 2 + sub;
            if (tile >= p.tiles) break;
            const uint32_t* vreg = reinterpret_cast<const uint32_t*>(unit_base + (size_t)tile * LY::tile_bytes + LY::vcodes_off);
            if (V8) {
                // int8 values: the lane's 16 bytes of coordinate group g, token 16ks + 8*e4 + 4*vh + e3 at byte 8ks + 4e4 + e3
#pragma unroll
                for (int g = 0; g < MT; ++g) {
                    const uint4 raw = *reinterpret_cast<const uint4*>(vreg + g * 256 + lane * 4);
                    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                    for (int x = 0; x < 4; ++x) {  // x = 2*ks + e4
                        float cv[4];
#pragma unroll
                        for (int e3 = 0; e3 < 4; ++e3) cv[e3] = (float)((int)((w[x] >> (8 * e3)) & 0xFF) - 128);
                        const int tk = sub * 32 + 8 * x + 4 * vh;  // tokens tk .. tk+3
#pragma unroll
                        for (int r = 0; r < kRB; ++r) {
                            const float4 pv = *reinterpret_cast<const float4*>(&p_s[wave][r][tk]);
                            acc[r][g] = fmaf(pv.x, cv[0], acc[r][g]);
                            acc[r][g] = fmaf(pv.y, cv[1], acc[r][g]);
                            acc[r][g] = fmaf(pv.z, cv[2], acc[r][g]);
                            acc[r][g] = fmaf(pv.w, cv[3], acc[r][g]);
                        }
                    }
                }
                continue;
            }
            if (VB == 2 || VB == 4) {
#pragma unroll
                for (int G = 0; G < D / 16; ++G) {
                    const uint32_t w = VB == 4 ? vreg[lane * (D / 16) + G] : vreg[lane * (D / 32) + (G >> 1)];
                    const int g = G >> 1;
#pragma unroll
                    for (int e4 = 0; e4 < 2; ++e4) {
                        float cv[4];
#pragma unroll
                        for (int e3 = 0; e3 < 4; ++e3) {
                            const int code = VB == 4 ? (w >> (8 * e3 + 4 * e4)) & 15 : (w >> (8 * e3 + 2 * (2 * (G & 1) + e4))) & 3;
                            cv[e3] = ctab[code];
                        }
                        const int tk = sub * 32 + vcode_token(G, lane, 4 * e4);  // tokens tk .. tk+3
#pragma unroll
                        for (int r = 0; r < kRB; ++r) {
                            const float4 pv = *reinterpret_cast<const float4*>(&p_s[wave][r][tk]);
                            acc[r][g] = fmaf(pv.x, cv[0], acc[r][g]);
                            acc[r][g] = fmaf(pv.y, cv[1], acc[r][g]);
                            acc[r][g] = fmaf(pv.z, cv[2], acc[r][g]);
                            acc[r][g] = fmaf(pv.w, cv[3], acc[r][g]);
                        }
                    }
                }
                continue;
            }
#pragma unroll
            for (int q = 0; q < LY::NT; ++q) {
                uint32_t w[3];
#pragma unroll
                for (int i = 0; i < 3; ++i) w[i] = vreg[q * 192 + lane * 3 + i];
#pragma unroll
                for (int gi = 0; gi < 4; ++gi) {
                    const int G = 4 * q + gi, g = G >> 1;
#pragma unroll
                    for (int e4 = 0; e4 < 2; ++e4) {
                        float cv[4];
#pragma unroll
                        for (int e3 = 0; e3 < 4; ++e3) {
                            int code;
                            if (gi < 3) code = (w[gi] >> (8 * e3 + 3 * e4)) & 7;
                            else if (e4 == 0) code = ((w[0] >> (8 * e3 + 6)) & 3) | (((w[1] >> (8 * e3 + 6)) & 1) << 2);
                            else code = ((w[2] >> (8 * e3 + 6)) & 3) | (((w[1] >> (8 * e3 + 7)) & 1) << 2);
                            cv[e3] = ctab[code];
                        }
                        const int tk = sub * 32 + vcode_token(G, lane, 4 * e4);  // tokens tk .. tk+3
#pragma unroll
                        for (int r = 0; r < kRB; ++r) {
                            const float4 pv = *reinterpret_cast<const float4*>(&p_s[wave][r][tk]);
                            acc[r][g] = fmaf(pv.x, cv[0], acc[r][g]);
                            acc[r][g] = fmaf(pv.y, cv[1], acc[r][g]);
                            acc[r][g] = fmaf(pv.z, cv[2], acc[r][g]);
                            acc[r][g] = fmaf(pv.w, cv[3], acc[r][g]);
                        }
                    }
                }
            }
        }
    }

    // ---- emit the split's partial
#pragma unroll
    for (int r = 0; r < kRB; ++r) {
        if (r0 + r >= p.R) break;
        const size_t prow = ((size_t)usel * p.nsplit + sp) * p.R + r0 + r;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float v = acc[r][mt];
            v += __shfl_xor(v, 32, 64);
            if (vh == 0) ws_o[prow * D + 32 * mt + mm] = v;
        }
        if (lane == 0) {
            ws_ml[prow * 2] = m_run[r];
            ws_ml[prow * 2 + 1] = l_run[r];
        }
    }
}

// ------------------------------------------------------------------------------ tail kernel ---
// Dense 16-bit attention of one agent's rows over its private, uncompressed continuation.
// One wave per (selected layer, kv head, agent, block of kRB rows); emits (m, l, o) in the original domain.
// The loops over a block's loads and pieces are unrolled in full: the compiler then keeps a block's key row and
// the query pieces in registers (all 256 at head_dim 128, one wave per SIMD plus what the 19 KB of LDS allow) and
// has every load of a block in flight at once.  Held under 128 registers for more waves per SIMD the kernel is
// 2 % faster on 64-token tails of all layers and 4 % slower on one layer's 32-token tails (measured); the
// unrolled form stays.  Per block of 64 tokens:
//   scores  the 64 key rows are fetched with coalesced loads and staged in LDS; lane = token then walks its
//           row in 16-byte pieces; the products with the raw 16-bit queries (LDS broadcast) are packed dot
//           products with fp32 accumulation, the softmax scale is applied to the sum;
//   P.V     lane = (token slot, 8 coordinates): one 16-byte load covers a lane's 8 coordinates of a token,
//           D/8 lanes a whole value row, so a wave load covers 512/D tokens of consecutive rows; every lane
//           accumulates its slot's tokens, the slots are added once at the very end.
typedef _Float16 tail_h2 __attribute__((ext_vector_type(2)));
typedef short tail_s2 __attribute__((ext_vector_type(2)));
template <bool BF> __device__ __forceinline__ float tail_dot2(uint32_t a, uint32_t b, float c) {
    if constexpr (BF) {
        union { uint32_t u; tail_s2 v; } x, y;
        x.u = a, y.u = b;
        return __builtin_amdgcn_fdot2_f32_bf16(x.v, y.v, c, false);
    } else {
        union { uint32_t u; tail_h2 v; } x, y;
        x.u = a, y.u = b;
        return __builtin_amdgcn_fdot2(x.v, y.v, c, false);
    }
}

template <int D, bool BF>
__global__ __launch_bounds__(64) void attend_tail_kernel(const __half* __restrict__ Q, TailPtrs tails,
                                                            float* __restrict__ tail_ml,
                                                            float* __restrict__ tail_o, AttendPlan p) {
    constexpr int LPR = D / 8;       // lanes per value row
    constexpr int TPL = 64 / LPR;    // tokens per wave load (token slots)
    constexpr int NLD = 64 / TPL;    // wave loads per 64 tokens
    __shared__ __align__(16) uint16_t q_s[kRB][D];     // the raw 16-bit queries
    __shared__ __align__(16) float p_s[64][kRB];       // probabilities, [token][row]
    __shared__ uint4 k_s[64][LPR + 1];                 // 64 key rows (one spare piece per row rotates the banks)
    const int lane = threadIdx.x;
    const int usel = blockIdx.y, ls = usel / p.H, kvh = usel - ls * p.H;
    const int a = blockIdx.x;
    const int rows_a = p.nq * p.G;  // rows of this agent within the KV head, contiguous
    const int r0 = a * rows_a + blockIdx.z * kRB;
    const int r_end = min((a + 1) * rows_a, r0 + kRB);
    if (r0 >= r_end) return;
    const int len = tails.len[a];
    // tokens each of the wave's rows may see: all of them, or, for a causal multi-token step, one less for
    // every query position before the agent's last (row r0 + r is query (r0 + r - a * rows_a) / G)
    int len_r[kRB];
#pragma unroll
    for (int r = 0; r < kRB; ++r) {
        const int qi = (r0 + r - a * rows_a) / p.G;
        len_r[r] = p.tail_causal ? max(0, len - (p.nq - 1 - min(qi, p.nq - 1))) : len;
    }
    const size_t head_off = ((size_t)(p.layer_begin + ls) * p.H + kvh) * p.tail_capacity * D;
    const uint16_t* Kt = reinterpret_cast<const uint16_t*>(tails.K[a]) + head_off;
    const uint16_t* Vt = reinterpret_cast<const uint16_t*>(tails.V[a]) + head_off;

    // queries: 16-byte loads, D/8 lanes to a row; rows past the agent's last are zero
    for (int i = lane; i < kRB * LPR; i += 64) {
        const int r = i / LPR, piece = i - r * LPR;
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (r0 + r < r_end) raw = *reinterpret_cast<const uint4*>(Q + q_row_index(p, ls, kvh, r0 + r) * D + 8 * piece);
        *reinterpret_cast<uint4*>(&q_s[r][8 * piece]) = raw;
    }
    __syncthreads();

    const int slot = lane / LPR, piece = lane - slot * LPR;
    float m_run[kRB], l_run[kRB], acc[kRB][8];
#pragma unroll
    for (int r = 0; r < kRB; ++r) {
        m_run[r] = -INFINITY;
        l_run[r] = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[r][c] = 0.0f;
    }

    for (int t0 = 0; t0 < len; t0 += 64) {
        const int cnt = min(64, len - t0);
        // ---- the 64 key rows come in with fully coalesced loads (lane = (token slot, piece), as for the
        // values below) and go through LDS, where every lane then walks the row of its own token
        // (rows past the end are copies of the last token; their scores become -inf)
#pragma unroll
        for (int b0 = 0; b0 < NLD; b0 += 8) {
            uint4 kin[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                kin[u] = *reinterpret_cast<const uint4*>(Kt + (size_t)(t0 + min((b0 + u) * TPL + slot, cnt - 1)) * D + 8 * piece);
#pragma unroll
            for (int u = 0; u < 8; ++u) k_s[(b0 + u) * TPL + slot][piece] = kin[u];
        }
        __syncthreads();
        const uint4* krow = &k_s[lane][0];
        float sc[kRB];
#pragma unroll
        for (int r = 0; r < kRB; ++r) sc[r] = 0.0f;
#pragma unroll
        for (int i0 = 0; i0 < LPR; i0 += 4) {   // four 16-byte pieces of the key row at a time
            uint4 kraw[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) kraw[u] = krow[i0 + u];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int r = 0; r < kRB; ++r) {
                    const uint4 qv = *reinterpret_cast<const uint4*>(&q_s[r][8 * (i0 + u)]);
                    sc[r] = tail_dot2<BF>(kraw[u].x, qv.x, sc[r]);
                    sc[r] = tail_dot2<BF>(kraw[u].y, qv.y, sc[r]);
                    sc[r] = tail_dot2<BF>(kraw[u].z, qv.z, sc[r]);
                    sc[r] = tail_dot2<BF>(kraw[u].w, qv.w, sc[r]);
                }
        }
        float alpha[kRB];
#pragma unroll
        for (int r = 0; r < kRB; ++r) {
            const float sv = t0 + lane < len_r[r] ? sc[r] * p.qscale : -INFINITY;
            const float m_new = fmaxf(m_run[r], wave_max(sv));
            // a row that has seen no token yet keeps m = -inf: nothing to rescale, every weight 0
            alpha[r] = m_new == -INFINITY ? 1.0f : exp2f(m_run[r] - m_new);
            const float pr = m_new == -INFINITY ? 0.0f : exp2f(sv - m_new);
            l_run[r] = l_run[r] * alpha[r] + wave_sum(pr);
            m_run[r] = m_new;
            p_s[lane][r] = pr;
        }
        __syncthreads();
        // ---- P.V, lane = (token slot, 8 coordinates)
#pragma unroll
        for (int r = 0; r < kRB; ++r)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[r][c] *= alpha[r];
#pragma unroll
        for (int b0 = 0; b0 < NLD; b0 += 8) {   // eight wave loads at a time
            uint4 vraw[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = min((b0 + u) * TPL + slot, cnt - 1);   // past the end: a re-read with weight 0
                vraw[u] = *reinterpret_cast<const uint4*>(Vt + (size_t)(t0 + t) * D + 8 * piece);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = (b0 + u) * TPL + slot;
                const float4 pr4 = *reinterpret_cast<const float4*>(&p_s[t][0]);
                const float pr[4] = {pr4.x, pr4.y, pr4.z, pr4.w};
                const uint32_t w[4] = {vraw[u].x, vraw[u].y, vraw[u].z, vraw[u].w};
#pragma unroll
                for (int c2 = 0; c2 < 4; ++c2) {
                    const float2 f = pair16_to_float2(w[c2], BF);
#pragma unroll
                    for (int r = 0; r < kRB; ++r) {
                        acc[r][2 * c2] = fmaf(pr[r], f.x, acc[r][2 * c2]);
                        acc[r][2 * c2 + 1] = fmaf(pr[r], f.y, acc[r][2 * c2 + 1]);
                    }
                }
            }
        }
        __syncthreads();
    }
    // ---- the token slots' shares are added (lanes piece + LPR * slot), slot 0 stores
#pragma unroll
    for (int r = 0; r < kRB; ++r)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float v = acc[r][c];
#pragma unroll
            for (int m = LPR; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
            acc[r][c] = v;
        }
#pragma unroll
    for (int r = 0; r < kRB; ++r) {
        if (r0 + r >= r_end) break;
        const size_t prow = (size_t)usel * p.R + r0 + r;
        if (slot == 0) {
            float4* dst = reinterpret_cast<float4*>(tail_o + prow * D + 8 * piece);
            dst[0] = make_float4(acc[r][0], acc[r][1], acc[r][2], acc[r][3]);
            dst[1] = make_float4(acc[r][4], acc[r][5], acc[r][6], acc[r][7]);
        }
        if (lane == 0) {
            tail_ml[prow * 2] = m_run[r];
            tail_ml[prow * 2 + 1] = l_run[r];
        }
    }
}

// ----------------------------------------------------------------------------- merge kernel ---
// One wave per query row: log-sum-exp merge of the split partials, o = H (acc / l) / sqrt(d),
// then the tail partial (already in the original domain), then the fp32 store.
template <int D>
__global__ __launch_bounds__(256) void attend_merge_kernel(const float* __restrict__ ws_ml,
                                                           const float* __restrict__ ws_o,
                                                           const float* __restrict__ tail_ml,
                                                           const float* __restrict__ tail_o,
                                                           float* __restrict__ out, AttendPlan p) {
    constexpr int EPL = D / 64;
    const int lane = threadIdx.x & 63;
    const long row_global = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long nrows = (long)p.layers * p.H * p.R;
    const bool active = row_global < nrows;  // no early return: the butterflies need the whole wave
    const long rg = active ? row_global : 0;
    const int usel = (int)(rg / p.R), r = (int)(rg - (long)usel * p.R);
    const int ls = usel / p.H, kvh = usel - ls * p.H;

    // Every split wrote its partial (zeros with m = -inf, l = 0 where it had no tokens), so nothing here
    // is conditional: the lanes fetch the (m, l) pairs of 64 splits at a time, the weights
    // w_s = 2^(m_s - M) are handed out with readlane, and the loads of the partial rows are independent
    // of each other (eight in flight per lane).
    const size_t row0 = (size_t)usel * p.nsplit * p.R + r;     // partial row of split 0; split stride p.R rows
    // the tail partial is requested now and used last
    float tail_m = -INFINITY, tail_l = 0.0f, tail_x[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) tail_x[i] = 0.0f;
    if (p.has_tails) {
        const size_t prow = (size_t)usel * p.R + r;
        tail_m = tail_ml[prow * 2];
        tail_l = tail_ml[prow * 2 + 1];
#pragma unroll
        for (int i = 0; i < EPL; ++i) tail_x[i] = tail_o[prow * D + lane * EPL + i];
    }
    float M = -INFINITY;
    for (int s = lane; s < p.nsplit; s += 64) M = fmaxf(M, ws_ml[(row0 + (size_t)s * p.R) * 2]);
    M = wave_max(M);
    float Lsum = 0.0f, x[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) x[i] = 0.0f;
    for (int s0 = 0; s0 < p.nsplit; s0 += 64) {
        const int s_mine = s0 + lane, cnt = min(64, p.nsplit - s0);
        float w = 0.0f;
        if (s_mine < p.nsplit) {
            const float2 ml = *reinterpret_cast<const float2*>(ws_ml + (row0 + (size_t)s_mine * p.R) * 2);
            w = ml.y > 0.0f ? exp2f(ml.x - M) : 0.0f;
            Lsum = fmaf(ml.y, w, Lsum);
        }
        const float* src = ws_o + (row0 + (size_t)s0 * p.R) * D + lane * EPL;
        const size_t stride = (size_t)p.R * D;
        int k = 0;
        for (; k + 8 <= cnt; k += 8) {
            float v[8][EPL];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < EPL; ++i) v[u][i] = src[(size_t)(k + u) * stride + i];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float wu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), k + u));
#pragma unroll
                for (int i = 0; i < EPL; ++i) x[i] = fmaf(v[u][i], wu, x[i]);
            }
        }
        for (; k < cnt; ++k) {
            const float wu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), k));
#pragma unroll
            for (int i = 0; i < EPL; ++i) x[i] = fmaf(src[(size_t)k * stride + i], wu, x[i]);
        }
    }
    Lsum = wave_sum(Lsum);
    const float invL = 1.0f / Lsum;
#pragma unroll
    for (int i = 0; i < EPL; ++i) x[i] *= invL;
    // Walsh-Hadamard over D = 64*EPL coordinates, coordinate = lane*EPL + i (int8 values were never rotated)
    if (p.vcodec != POLYKV_VALUES_INT8) wht_inlane<EPL>(x);
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        if (p.vcodec == POLYKV_VALUES_INT8) break;
        x[i] = wht_lane_stage<1>(x[i], lane);
        x[i] = wht_lane_stage<2>(x[i], lane);
        x[i] = wht_lane_stage<4>(x[i], lane);
        x[i] = wht_lane_stage<8>(x[i], lane);
        x[i] = wht_lane_stage<16>(x[i], lane);
        x[i] = wht_lane_stage<32>(x[i], lane);
        x[i] *= (D == 64 ? 0.125f : D == 128 ? 0.08838834764831845f : 0.0625f);
    }
    if (p.signs.on && p.vcodec != POLYKV_VALUES_INT8)  // rotation variant H.D: coordinates lane*EPL ..
        flip_signs<EPL>(x, sign_word(p.signs, (lane * EPL) >> 5) >> ((lane * EPL) & 31));
    if (tail_l > 0.0f) {
        const float M2 = fmaxf(M, tail_m);
        const float wa = exp2f(M - M2) * Lsum, wb = exp2f(tail_m - M2);
        const float inv = 1.0f / (wa + wb * tail_l);
#pragma unroll
        for (int i = 0; i < EPL; ++i) x[i] = (wa * x[i] + wb * tail_x[i]) * inv;
    }
    if (active) {
        float* dst = out + q_row_index(p, ls, kvh, r) * D + lane * EPL;
#pragma unroll
        for (int i = 0; i < EPL; ++i) dst[i] = x[i];
    }
}

// --------------------------------------------------------------------------------- launcher ---
hipError_t launch_attend(const polykv_pool* pool, const AttendPlan& plan, const void* Q, void* out,
                         const TailPtrs* tails, void* workspace, hipStream_t s) {
    char* ws = reinterpret_cast<char*>(workspace);
    float* ws_ml = reinterpret_cast<float*>(ws + plan.off_ml);
    float* ws_o = reinterpret_cast<float*>(ws + plan.off_o);
    float* tail_ml = reinterpret_cast<float*>(ws + plan.off_tail_ml);
    float* tail_o = reinterpret_cast<float*>(ws + plan.off_tail_o);
    const uint8_t* storage = reinterpret_cast<const uint8_t*>(pool->storage);
    const int units = plan.layers * plan.H;
    hipError_t err;

    // The private tails go first: their partials are independent of the pool's, and where the matrix-core kernel
    // writes the final output itself it takes them in (through its ws_ml / ws_o arguments, which it does not
    // otherwise use then) instead of leaving them to the merge kernel.
    if (plan.has_tails) {
        dim3 grid(plan.A, units, (plan.nq * plan.G + kRB - 1) / kRB);
        using TailKern = decltype(&attend_tail_kernel<128, false>);
        static const TailKern tail_table[3][2] = {{attend_tail_kernel<64, false>, attend_tail_kernel<64, true>},
                                                  {attend_tail_kernel<128, false>, attend_tail_kernel<128, true>},
                                                  {attend_tail_kernel<256, false>, attend_tail_kernel<256, true>}};
        tail_table[plan.D == 64 ? 0 : plan.D == 128 ? 1 : 2][plan.io_bf16 ? 1 : 0]<<<grid, 64, 0, s>>>(
            (const __half*)Q, *tails, tail_ml, tail_o, plan);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    if (plan.kernel == POLYKV_KERNEL_MATRIX) {
        const bool direct = matrix_kernel_direct(plan);
        err = launch_attend_matrix(pool, plan, Q, direct && plan.has_tails ? tail_ml : ws_ml,
                                   direct && plan.has_tails ? tail_o : ws_o, (float*)out, s);
        if (err != hipSuccess) return err;
        if (direct) return hipSuccess;
    } else {
        dim3 grid(plan.nsplit / 4, units, (plan.R + kRB - 1) / kRB);
        using Kern = decltype(&attend_vector_kernel<128, 0, 0>);
#define POLYKV_VEC_ROW(D, KC)                                                                                   \
    {attend_vector_kernel<D, 0, KC>, attend_vector_kernel<D, 1, KC>, attend_vector_kernel<D, 2, KC>,            \
     attend_vector_kernel<D, 3, KC>, attend_vector_kernel<D, 4, KC>, attend_vector_kernel<D, 5, KC>,            \
     attend_vector_kernel<D, 6, KC>}
        static const Kern table[2][3][kNumValueCodecs] = {
            {POLYKV_VEC_ROW(64, 0), POLYKV_VEC_ROW(128, 0), POLYKV_VEC_ROW(256, 0)},
            {POLYKV_VEC_ROW(64, 1), POLYKV_VEC_ROW(128, 1), POLYKV_VEC_ROW(256, 1)}};
#undef POLYKV_VEC_ROW
        auto kern = table[plan.kcodec][plan.D == 64 ? 0 : plan.D == 128 ? 1 : 2][plan.vcodec];
        launch_main_kernel(kern, grid, dim3(256), 0, s, storage, (const __half*)Q, ws_ml, ws_o, plan);
        if ((err = hipGetLastError()) != hipSuccess) return err;
    }
    const long nrows = (long)units * plan.R;
    dim3 mgrid((unsigned)((nrows + 3) / 4));
    if (plan.D == 128)
        attend_merge_kernel<128><<<mgrid, 256, 0, s>>>(ws_ml, ws_o, tail_ml, tail_o, (float*)out, plan);
    else if (plan.D == 64)
        attend_merge_kernel<64><<<mgrid, 256, 0, s>>>(ws_ml, ws_o, tail_ml, tail_o, (float*)out, plan);
    else
        attend_merge_kernel<256><<<mgrid, 256, 0, s>>>(ws_ml, ws_o, tail_ml, tail_o, (float*)out, plan);
    return hipGetLastError();
}

}  // namespace polykv
