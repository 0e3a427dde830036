// Encode / decode / export kernels of the packed pool (gfx950).
//
// One workgroup of 256 threads handles one tile (32 tokens) of one KV head.  Thread (t, c) owns D/8
// head_dim elements of token t -- in decode, and in encode at head_dim 256, every eighth 8-element piece
// (8i + c), which makes every access instruction to the dense tensors cover whole cache lines; in encode
// at head_dim 64 and 128 the consecutive ones c*D/8 .., where that does not pay -- so a
// dense row is read or written by 8 lanes and a wave covers 8 whole rows.  The Walsh-Hadamard transform
// is log2(D/8) in-register stages plus three one-instruction DPP stages across those 8 lanes.  Both
// kernels are written to stay under the HBM time in vector instructions: conversions are fused with
// multiplies, the key codes are rounded with one magic-number add, the value quantizer compares the
// magnitude against three thresholds, and all bit (un)packing works on dwords.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "polykv_internal.hpp"
#include "polykv_layout.hpp"

// The quantizers take rounding decisions that must match the definition operation by operation
// (product rounded to fp32, then rounded to an integer): no fused multiply-adds unless written out.
#pragma clang fp contract(off)

namespace polykv {

// The dense output of pool_decode is written once and read by some later kernel, 537 MB of it at the Llama shape:
// it is stored with the non-temporal hint, so that it streams to memory instead of sitting in the last-level
// cache as dirty lines whose write-back the NEXT kernels would pay for (measured: whatever followed pool_decode
// ran 9-10 us longer; decode itself takes 2-3 us more this way).  Every store instruction of a wave covers whole
// cache lines (see decode_kernel), which is what makes streaming stores cheap here.  The packed pool that
// pool_encode writes keeps ordinary stores: it is what the next kernels read, and streaming it cost 3 us.
typedef uint32_t StreamQuad __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void stream_store16(void* dst, uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    const StreamQuad q = {a, b, c, d};
    __builtin_nontemporal_store(q, reinterpret_cast<StreamQuad*>(dst));
}

template <int D> __device__ __forceinline__ constexpr float inv_sqrt_d() {
    return D == 64 ? 0.125f : D == 128 ? 0.08838834764831845f : 0.0625f;
}
template <int D> __device__ __forceinline__ constexpr float sqrt_d() {
    return D == 64 ? 8.0f : D == 128 ? 11.313708498984761f : 16.0f;
}

union Half2Bits {
    uint32_t u;
    _Float16 h[2];
};

// Thread -> (token of the tile, chunk) for the codec kernels; see wht_cross_chunks().
struct CodecThread {
    int t, c;
    __device__ __forceinline__ explicit CodecThread(int tid)
        : t((tid >> 6) * 8 + codec_token_in_wave(tid & 63)), c(codec_chunk(tid & 63)) {}
};

// ------------------------------------------------------------------------------------ encode ---
// Key quantization and value quantization of section "Compression Scheme", fused in one pass.
// VC = 1, the scaled-values codec: each value vector also stores g = fp16(min(rms, 128)), rms = |v|/sqrt(D),
// and its rotated coordinates are quantized in units of g, which gives the codebook the unit-variance
// input that the analysis of section "TurboQuant" assumes.
// VC = 2, int8 values: no rotation; the key formula on the whole vector with one scale per vector,
// s = fp16(min(max|v|/127, 128)) (the uniform int8 ablation proposed in sections "Discussion" and
// "Future Work").
// BF: K and V are bfloat16 instead of fp16 (the bit patterns are passed as __half all the same).
// KC = 1: one key scale per layer tensor, from the layer's max|k| in kmax[] (found by kamax_kernel); H = KV
// heads per layer.
template <int D, int VC, bool BF, int KC>
__global__ __launch_bounds__(256) void encode_kernel(const __half* __restrict__ K,
                                                     const __half* __restrict__ V,
                                                     uint8_t* __restrict__ pool, int in_tokens, int tok_begin,
                                                     int tok_end, int tiles_cap, SignBits signs,
                                                     const uint32_t* __restrict__ kmax, int H) {
    // K, V hold in_tokens = tok_end - tok_begin tokens per (layer, KV head); they become pool tokens
    // [tok_begin, tok_end).  blockIdx.x counts tiles from the first one touched.  Tokens of that tile that
    // lie before tok_begin were encoded earlier and are carried over; tokens from tok_end on are padding
    // and are encoded as zeros.
    using LY = Layout<D, VC, KC>;
    constexpr int VB = vc_bits(VC);  // bits per value code
    constexpr bool V8 = VB == 8, VS = vc_has_scale(VC) && !V8;
    constexpr int EPT = D / 8;
    constexpr int KBYTES = LY::vcodes_off;  // key codes (+ key scales) (+ value scales)
    constexpr int VST = kTile + 4;          // bytes per rotated coordinate in the code staging area
    __shared__ __align__(16) uint8_t kimg[KBYTES];
    __shared__ __align__(16) uint8_t vstage[D * VST];  // value codes as bytes, [coordinate][token]

    const int tile = tok_begin / kTile + blockIdx.x, unit = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63;
    const CodecThread th(tid);
    const int t = th.t, c = th.c;
    const int tok = tile * kTile + t;
    const bool old_token = tok < tok_begin;              // keep what the record holds
    const bool valid = !old_token && tok < tok_end;      // read from K, V
    const bool has_old = tile * kTile < tok_begin;       // uniform over the workgroup
    // At head_dim 256 a thread's share is every eighth 8-element piece (8 rr + c, as in decode_kernel): with
    // four pieces per thread the 8 lanes of a token then read whole cache lines per load instruction, which is
    // worth a tenth of the kernel's time there (and nothing at 128, where the consecutive share stays).
    constexpr bool PIECES = D == 256;
    const size_t row = ((size_t)unit * in_tokens + (valid ? tok - tok_begin : 0)) * D + (PIECES ? 0 : c * EPT);
    const int e0 = c * EPT, j = e0 >> 5, g8 = (e0 >> 3) & 3;  // (consecutive share)
    // element i of the thread's share is head_dim coordinate coord(i)
    auto coord = [&](int i) { return PIECES ? 8 * (8 * (i >> 3) + c) + (i & 7) : e0 + i; };
    uint8_t* rec = pool + ((size_t)unit * tiles_cap + tile) * LY::tile_bytes;

    uint4 kraw[EPT / 8], vraw[EPT / 8];
#pragma unroll
    for (int i = 0; i < EPT / 8; ++i) {
        const int piece = PIECES ? 8 * i + c : i;
        kraw[i] = valid ? reinterpret_cast<const uint4*>(K + row)[piece] : make_uint4(0, 0, 0, 0);
        vraw[i] = valid ? reinterpret_cast<const uint4*>(V + row)[piece] : make_uint4(0, 0, 0, 0);
    }

    if (has_old) {
        // carry the earlier tokens over: their key bytes and scales go back into the record image, their
        // value codes are unpacked into the byte staging area (whole dwords: the slots of the new tokens
        // are overwritten below)
        const uint4* src = reinterpret_cast<const uint4*>(rec);
        for (int i = tid; i < KBYTES / 16; i += 256) reinterpret_cast<uint4*>(kimg)[i] = src[i];
        if (V8) {
            for (int g = tid >> 6; g < LY::NB; g += 4) {
                const uint4 w = *reinterpret_cast<const uint4*>(rec + LY::vcodes_off + g * 1024 + lane * 16);
                uint8_t* dst = vstage + (32 * g + (lane & 31)) * VST + 4 * (lane >> 5);  // tokens 4h.., 8+4h.., 16+4h.., 24+4h..
                *reinterpret_cast<uint32_t*>(dst) = w.x;
                *reinterpret_cast<uint32_t*>(dst + 8) = w.y;
                *reinterpret_cast<uint32_t*>(dst + 16) = w.z;
                *reinterpret_cast<uint32_t*>(dst + 24) = w.w;
            }
        } else if (VB == 4 || VB == 2) {
            if (tid < LY::NT * 64) {  // work item (q, lane): groups 4q .. 4q+3
                const int q = tid >> 6;
#pragma unroll
                for (int gi = 0; gi < 4; ++gi) {
                    const int G = 4 * q + gi;
                    uint32_t lo, hi;
                    if (VB == 4) {
                        const uint32_t w = reinterpret_cast<const uint32_t*>(rec + LY::vcodes_off)[lane * (D / 16) + G];
                        lo = w & 0x0F0F0F0Fu;
                        hi = (w >> 4) & 0x0F0F0F0Fu;
                    } else {
                        const uint32_t w = reinterpret_cast<const uint32_t*>(rec + LY::vcodes_off)[lane * (D / 32) + (G >> 1)];
                        lo = (w >> (4 * (G & 1))) & 0x03030303u;
                        hi = (w >> (4 * (G & 1) + 2)) & 0x03030303u;
                    }
                    uint8_t* dst = vstage + vcode_coord(G, lane) * VST + vcode_token(G, lane, 0);
                    *reinterpret_cast<uint32_t*>(dst) = lo;
                    *reinterpret_cast<uint32_t*>(dst + 8) = hi;
                }
            }
        } else if (tid < LY::NT * 64) {  // NT <= 4: one wave per triplet
            const int q = tid >> 6;
            const uint32_t* w = reinterpret_cast<const uint32_t*>(rec + LY::vcodes_off + q * 768 + lane * 12);
            const uint32_t w0 = w[0], w1 = w[1], w2 = w[2];
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                const int G = 4 * q + gi;
                uint32_t lo, hi;
                vcode_selectors(w0, w1, w2, gi, lo, hi);
                uint8_t* dst = vstage + vcode_coord(G, lane) * VST + vcode_token(G, lane, 0);
                *reinterpret_cast<uint32_t*>(dst) = lo;
                *reinterpret_cast<uint32_t*>(dst + 8) = hi;
            }
        }
        __syncthreads();
    }

    // ---- keys: block absmax -> fp16 scale -> codes with the stored scale
    if constexpr (!PIECES) {
        // max|k| on the raw 16-bit patterns: magnitudes of fp16 (and of bfloat16) order like unsigned integers
        typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
        union {
            uint32_t u;
            ushort2v v;
        } mx;
        mx.u = 0;
#pragma unroll
        for (int i = 0; i < EPT / 2; ++i) {
            union {
                uint32_t u;
                ushort2v v;
            } w;
            w.u = reinterpret_cast<const uint32_t*>(kraw)[i] & 0x7FFF7FFFu;
            mx.v = __builtin_elementwise_max(mx.v, w.v);
        }
        float amax = bits16_to_float((uint16_t)max(mx.u & 0xFFFFu, mx.u >> 16), BF);
        // a q8_0 block of 32 elements spans 32 / EPT lanes
        if (EPT <= 16) amax = fmaxf(amax, lane_xor<1>(amax));
        if (EPT == 8) amax = fmaxf(amax, lane_xor<2>(amax));
        // bfloat16 keys can exceed what an fp16 scale holds: it saturates at the fp16 maximum
        const float sraw = __fdiv_rn(amax, 127.0f);
        __half s16 = __float2half_rn(BF ? fminf(sraw, 65504.0f) : sraw);
        if (KC == 1) s16 = (__half)tensor_key_scale(kmax[unit / H]);
        const float sf = __half2float(s16);
        const float inv = sf > 0.0f ? __fdiv_rn(1.0f, sf) : 0.0f;
        // round(k * inv) + 128 in the low byte of a float: adding 1.5 * 2^23 + 128 rounds the product
        // to an integer (nearest, ties to even) in the low mantissa bits; the clamp keeps the byte valid
        // when a subnormal scale lets |k * inv| exceed 127.
        constexpr float kMagic = 12582912.0f + 128.0f;
        uint32_t r[EPT];
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            // two roundings, product then sum (contraction is off in this file); for fp16 input the
            // conversion rides on the multiply (one fma-mix instruction, the product rounded once)
            const uint32_t pair = reinterpret_cast<const uint32_t*>(kraw)[i >> 1];
            float prod;
            if (BF) {
                prod = __uint_as_float((i & 1) ? pair & 0xFFFF0000u : pair << 16) * inv;
            } else {
                Half2Bits hb;
                hb.u = pair;
                prod = __builtin_fmaf((float)hb.h[i & 1], inv, 0.0f);
            }
            const float q = prod + kMagic;
            r[i] = __float_as_uint(__builtin_amdgcn_fmed3f(q, kMagic - 128.0f, kMagic + 127.0f));
        }
#pragma unroll
        for (int rr = 0; rr < EPT / 8; ++rr) {
            if (old_token) break;
            uint2 w;
            const uint32_t a01 = __builtin_amdgcn_perm(r[8 * rr + 1], r[8 * rr + 0], 0x0c0c0400u);
            const uint32_t a23 = __builtin_amdgcn_perm(r[8 * rr + 3], r[8 * rr + 2], 0x04000c0cu);
            const uint32_t b01 = __builtin_amdgcn_perm(r[8 * rr + 5], r[8 * rr + 4], 0x0c0c0400u);
            const uint32_t b23 = __builtin_amdgcn_perm(r[8 * rr + 7], r[8 * rr + 6], 0x04000c0cu);
            w.x = a01 | a23;
            w.y = b01 | b23;
            *reinterpret_cast<uint2*>(kimg + LY::kcodes_off + kcode_run_offset(t, j, g8 + rr)) = w;
        }
        if (KC == 0 && (e0 & 31) == 0 && !old_token)
            reinterpret_cast<__half*>(kimg + LY::kscales_off)[t * LY::NB + j] = s16;
    } else {
        // Interleaved pieces: piece rr of the thread lies in block 2 rr + c / 4, which the four lanes of a quad
        // share (c % 4 = the piece's place in the block).  Lane q of the quad works out the scale of piece q's
        // block; a quad broadcast hands every lane the four scales.
        typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
        constexpr int NP = EPT / 8;
        static_assert(NP == 4, "one piece per lane of a quad");
        float amax_p[NP];
#pragma unroll
        for (int rr = 0; rr < NP; ++rr) {
            union {
                uint32_t u;
                ushort2v v;
            } mx, w;
            mx.u = 0;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                w.u = reinterpret_cast<const uint32_t*>(&kraw[rr])[x] & 0x7FFF7FFFu;
                mx.v = __builtin_elementwise_max(mx.v, w.v);
            }
            float am = bits16_to_float((uint16_t)max(mx.u & 0xFFFFu, mx.u >> 16), BF);
            am = fmaxf(am, lane_xor<1>(am));
            amax_p[rr] = fmaxf(am, lane_xor<2>(am));
        }
        const int q = c & 3;
        const float amax = q == 0 ? amax_p[0] : q == 1 ? amax_p[1] : q == 2 ? amax_p[2] : amax_p[3];
        const float sraw = __fdiv_rn(amax, 127.0f);
        __half s16 = __float2half_rn(BF ? fminf(sraw, 65504.0f) : sraw);
        if (KC == 1) s16 = (__half)tensor_key_scale(kmax[unit / H]);
        const float sf = __half2float(s16);
        const float inv = sf > 0.0f ? __fdiv_rn(1.0f, sf) : 0.0f;
        float sf_p[NP], inv_p[NP];
        {
            const int si = __float_as_int(sf), ii = __float_as_int(inv);
            sf_p[0] = __int_as_float(__builtin_amdgcn_update_dpp(si, si, 0x00, 0xF, 0xF, false));   // quad_perm [0,0,0,0]
            sf_p[1] = __int_as_float(__builtin_amdgcn_update_dpp(si, si, 0x55, 0xF, 0xF, false));   // [1,1,1,1]
            sf_p[2] = __int_as_float(__builtin_amdgcn_update_dpp(si, si, 0xAA, 0xF, 0xF, false));   // [2,2,2,2]
            sf_p[3] = __int_as_float(__builtin_amdgcn_update_dpp(si, si, 0xFF, 0xF, 0xF, false));   // [3,3,3,3]
            inv_p[0] = __int_as_float(__builtin_amdgcn_update_dpp(ii, ii, 0x00, 0xF, 0xF, false));
            inv_p[1] = __int_as_float(__builtin_amdgcn_update_dpp(ii, ii, 0x55, 0xF, 0xF, false));
            inv_p[2] = __int_as_float(__builtin_amdgcn_update_dpp(ii, ii, 0xAA, 0xF, 0xF, false));
            inv_p[3] = __int_as_float(__builtin_amdgcn_update_dpp(ii, ii, 0xFF, 0xF, 0xF, false));
        }
        constexpr float kMagic = 12582912.0f + 128.0f;  // as above: the low byte is round(k * inv) + 128
#pragma unroll
        for (int rr = 0; rr < NP; ++rr) {
            uint32_t r[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t pair = reinterpret_cast<const uint32_t*>(&kraw[rr])[i >> 1];
                float prod;
                if (BF) {
                    prod = __uint_as_float((i & 1) ? pair & 0xFFFF0000u : pair << 16) * inv_p[rr];
                } else {
                    Half2Bits hb;
                    hb.u = pair;
                    prod = __builtin_fmaf((float)hb.h[i & 1], inv_p[rr], 0.0f);
                }
                const float qv = prod + kMagic;
                r[i] = __float_as_uint(__builtin_amdgcn_fmed3f(qv, kMagic - 128.0f, kMagic + 127.0f));
            }
            if (!old_token) {
                uint2 w;
                w.x = __builtin_amdgcn_perm(r[1], r[0], 0x0c0c0400u) | __builtin_amdgcn_perm(r[3], r[2], 0x04000c0cu);
                w.y = __builtin_amdgcn_perm(r[5], r[4], 0x0c0c0400u) | __builtin_amdgcn_perm(r[7], r[6], 0x04000c0cu);
                *reinterpret_cast<uint2*>(kimg + LY::kcodes_off + kcode_run_offset(t, 2 * rr + (c >> 2), q)) = w;
                if (KC == 0 && q == 0)  // exact: the value is an fp16 number
                    reinterpret_cast<__half*>(kimg + LY::kscales_off)[t * LY::NB + 2 * rr + (c >> 2)] = __float2half_rn(sf_p[rr]);
            }
        }
    }

    // ---- values, int8 codec: vector absmax -> fp16 scale -> codes with the stored scale, staged as bytes
    if (V8) {
        float v[EPT];
#pragma unroll
        for (int i = 0; i < EPT / 2; ++i) {
            const float2 f = pair16_to_float2(reinterpret_cast<const uint32_t*>(vraw)[i], BF);
            v[2 * i] = f.x;
            v[2 * i + 1] = f.y;
        }
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < EPT; i += 2) amax = fmaxf(fmaxf(fabsf(v[i]), fabsf(v[i + 1])), amax);
        amax = fmaxf(amax, lane_xor<1>(amax));
        amax = fmaxf(amax, lane_xor<2>(amax));
        amax = fmaxf(amax, lane_xor<8>(amax));
        const __half s16 = __float2half_rn(fminf(__fdiv_rn(amax, 127.0f), 128.0f));
        const float sf = __half2float(s16);
        const float inv = sf > 0.0f ? __fdiv_rn(1.0f, sf) : 0.0f;
        constexpr float kMagic = 12582912.0f + 128.0f;  // as for the keys: the low byte is round(v * inv) + 128
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const float q = v[i] * inv + kMagic;
            const uint32_t r = __float_as_uint(__builtin_amdgcn_fmed3f(q, kMagic - 128.0f, kMagic + 127.0f));
            if (!old_token) vstage[coord(i) * VST + t] = (uint8_t)r;
        }
        if (c == 0 && !old_token) reinterpret_cast<__half*>(kimg + LY::vscales_off)[t] = s16;
    }
    // ---- values: rotate, nearest centroid, stage the codes as bytes [coordinate][token]
    if (!V8) {
        const float eps = codec_entry_sign(lane);
        float y[EPT];
#pragma unroll
        for (int i = 0; i < EPT / 2; ++i) {
            if (BF) {
                const float2 f = pair16_to_float2(reinterpret_cast<const uint32_t*>(vraw)[i], true);
                y[2 * i] = f.x * eps;
                y[2 * i + 1] = f.y * eps;
            } else {
                Half2Bits b;
                b.u = reinterpret_cast<const uint32_t*>(vraw)[i];
                y[2 * i] = __builtin_fmaf((float)b.h[0], eps, 0.0f);  // conversion and sign in one fma-mix
                y[2 * i + 1] = __builtin_fmaf((float)b.h[1], eps, 0.0f);
            }
        }
        // y = sqrt(D) * v_rot after the transform; the thresholds are scaled instead of the values.  The
        // code is the number of thresholds below v_rot: 4 + n for positive values, 3 - n otherwise, with
        // n the number of positive thresholds below |v_rot|.
        float t1 = POLYKV_T1 * sqrt_d<D>(), t2 = POLYKV_T2 * sqrt_d<D>(), t3 = POLYKV_T3 * sqrt_d<D>();
        float zref = 0.0f;  // what "positive" is measured against
        float tscale = sqrt_d<D>();  // factor on the thresholds (2- and 4-bit codes)
        if (VS) {
            // |v|^2 over the 8 lanes of the token (the signs do not matter); every lane gets the same sum
            float ss = 0.0f;
#pragma unroll
            for (int i = 0; i < EPT; ++i) ss = __builtin_fmaf(y[i], y[i], ss);
            ss += lane_xor<1>(ss);
            ss += lane_xor<2>(ss);
            ss += __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(ss), __float_as_int(ss), 0x128, 0xF, 0xF,
                                                               false));  // row_ror:8 = lane ^ 8
            const float rms = __fsqrt_rn(ss * (1.0f / D));
            const __half g16 = __float2half_rn(fminf(rms, 128.0f));
            const float g = __half2float(g16);
            t1 = t1 * g;
            t2 = t2 * g;
            t3 = t3 * g;
            tscale = tscale * g;
            // a scale of zero stores the zero vector, the code of zero everywhere: nothing counts as positive
            // and no magnitude exceeds a threshold
            if (!(g > 0.0f)) {
                zref = INFINITY;
                t1 = t2 = t3 = INFINITY;
                tscale = INFINITY;
            }
            if (c == 0 && !old_token) reinterpret_cast<__half*>(kimg + LY::vscales_off)[t] = g16;
        }
        if (signs.on) {  // rotation H.D: D first
            if constexpr (PIECES) {
#pragma unroll
                for (int rr = 0; rr < EPT / 8; ++rr) {
                    const int p = 8 * rr + c;
                    float(&y8)[8] = *reinterpret_cast<float(*)[8]>(&y[8 * rr]);
                    flip_signs<8>(y8, sign_word(signs, p >> 2) >> (8 * (p & 3)));
                }
            } else {
                flip_signs<EPT>(y, sign_word(signs, e0 >> 5) >> (e0 & 31));
            }
        }
        wht_cross_chunks<EPT>(y, lane);
        wht_inlane<EPT>(y);
        // the thresholds are operands of every element's compare block: pin them to registers once (as
        // constants the compiler would load them again in front of each block)
        asm volatile("" : "+v"(t1), "+v"(t2), "+v"(t3), "+v"(zref), "+v"(tscale));
        uint8_t codes[EPT];
        if (VB != 3) {
            // 2 and 4 bits: sign and magnitude, magnitude = number of positive thresholds below |v_rot|
            constexpr int NTH = (1 << (VB - 1)) - 1;
            float th[NTH];
#pragma unroll
            for (int k = 0; k < NTH; ++k) th[k] = threshold_mag(VB, k) * tscale;  // inf * t = inf for a zero scale
            if constexpr (VB == 4) {
                // Sign, then a three-level binary search over the seven thresholds: per element four compares
                // into scalar masks, four selects of the next threshold and four add-with-carry steps that
                // shift the decisions into the code (code = 2 code + decision).  Two elements go in lockstep
                // so that every mask is read two or more instructions after the compare that wrote it.
#pragma unroll
                for (int i = 0; i < EPT; i += 2) {
                    int n0, n1;
                    float ta, tb, aa, ab, ba, bb;
                    unsigned long long ma0, ma1, mb0, mb1;
                    asm("v_cmp_nlt_f32_e64 %8, %21, %12\n\t"
                        "v_cmp_nlt_f32_e64 %9, %21, %13\n\t"
                        "v_cmp_gt_f32_e64 %10, |%12|, %17\n\t"
                        "v_cmp_gt_f32_e64 %11, |%13|, %17\n\t"
                        "v_addc_co_u32_e64 %0, vcc, 0, 0, %8\n\t"
                        "v_addc_co_u32_e64 %1, vcc, 0, 0, %9\n\t"
                        "v_cndmask_b32_e64 %2, %15, %19, %10\n\t"
                        "v_cndmask_b32_e64 %3, %15, %19, %11\n\t"
                        "v_cndmask_b32_e64 %4, %14, %18, %10\n\t"
                        "v_cndmask_b32_e64 %5, %14, %18, %11\n\t"
                        "v_cndmask_b32_e64 %6, %16, %20, %10\n\t"
                        "v_cndmask_b32_e64 %7, %16, %20, %11\n\t"
                        "v_cmp_gt_f32_e64 %8, |%12|, %2\n\t"
                        "v_cmp_gt_f32_e64 %9, |%13|, %3\n\t"
                        "v_addc_co_u32_e64 %0, vcc, %0, %0, %10\n\t"
                        "v_addc_co_u32_e64 %1, vcc, %1, %1, %11\n\t"
                        "v_cndmask_b32_e64 %2, %4, %6, %8\n\t"
                        "v_cndmask_b32_e64 %3, %5, %7, %9\n\t"
                        "v_cmp_gt_f32_e64 %10, |%12|, %2\n\t"
                        "v_cmp_gt_f32_e64 %11, |%13|, %3\n\t"
                        "v_addc_co_u32_e64 %0, vcc, %0, %0, %8\n\t"
                        "v_addc_co_u32_e64 %1, vcc, %1, %1, %9\n\t"
                        "v_addc_co_u32_e64 %0, vcc, %0, %0, %10\n\t"
                        "v_addc_co_u32_e64 %1, vcc, %1, %1, %11"
                        : "=&v"(n0), "=&v"(n1), "=&v"(ta), "=&v"(tb), "=&v"(aa), "=&v"(ab), "=&v"(ba), "=&v"(bb),
                          "=&s"(ma0), "=&s"(ma1), "=&s"(mb0), "=&s"(mb1)
                        : "v"(y[i]), "v"(y[i + 1]), "v"(th[0]), "v"(th[1]), "v"(th[2]), "v"(th[3]), "v"(th[4]), "v"(th[5]),
                          "v"(th[6]), "v"(zref)
                        : "vcc");
                    codes[i] = (uint8_t)n0;
                    codes[i + 1] = (uint8_t)n1;
                }
            } else {
#pragma unroll
                for (int i = 0; i < EPT; ++i) {
                    const float ay = fabsf(y[i]);
                    int n = 0;
#pragma unroll
                    for (int k = 0; k < NTH; ++k) n += ay > th[k];
                    codes[i] = (uint8_t)((y[i] > zref ? 0 : (1 << (VB - 1))) | n);
                }
            }
        }
#pragma unroll
        for (int i = 0; VB == 3 && i < EPT; ++i) {
            // Four compares into scalar masks, then a select and an add-with-carry chain.  On this target a
            // vector instruction may read a scalar mask only two or more instructions after the compare
            // that wrote it; the order below keeps that distance without padding.
            int n, m;
            unsigned long long sp, s1, s2, s3;
            asm("v_cmp_lt_f32_e64 %2, %10, %6\n\t"
                "v_cmp_gt_f32_e64 %3, |%6|, %7\n\t"
                "v_cmp_gt_f32_e64 %4, |%6|, %8\n\t"
                "v_cmp_gt_f32_e64 %5, |%6|, %9\n\t"
                "v_cndmask_b32_e64 %1, 3, 4, %2\n\t"
                "v_addc_co_u32_e64 %0, vcc, 0, 0, %3\n\t"
                "v_addc_co_u32_e64 %0, vcc, 0, %0, %4\n\t"
                "v_addc_co_u32_e64 %0, vcc, 0, %0, %5\n\t"
                "v_xor_b32_e32 %0, %0, %1"
                : "=&v"(n), "=&v"(m), "=&s"(sp), "=&s"(s1), "=&s"(s2), "=&s"(s3)
                : "v"(y[i]), "v"(t1), "v"(t2), "v"(t3), "v"(zref)
                : "vcc");
            codes[i] = (uint8_t)n;
        }
        if (!old_token) {
#pragma unroll
            for (int i = 0; i < EPT; ++i) vstage[coord(i) * VST + t] = codes[i];
        }
    }
    __syncthreads();

    // ---- int8 values: one lane's 16 bytes of a coordinate group per thread, in P.V operand order
    if (V8) {
        for (int g = tid >> 6; g < LY::NB; g += 4) {
            const uint8_t* src = vstage + (32 * g + (lane & 31)) * VST + 4 * (lane >> 5);
            uint4 w;
            w.x = *reinterpret_cast<const uint32_t*>(src);
            w.y = *reinterpret_cast<const uint32_t*>(src + 8);
            w.z = *reinterpret_cast<const uint32_t*>(src + 16);
            w.w = *reinterpret_cast<const uint32_t*>(src + 24);
            *reinterpret_cast<uint4*>(rec + LY::vcodes_off + g * 1024 + lane * 16) = w;
        }
    } else if (VB == 4 || VB == 2) {
        // ---- 4 / 2 bits: work item (q, lane) packs groups 4q .. 4q+3 into four / two dwords
        if (tid < LY::NT * 64) {
            const int q = tid >> 6;
            uint32_t lo[4], hi[4];
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                const int G = 4 * q + gi;
                const uint8_t* src = vstage + vcode_coord(G, lane) * VST + vcode_token(G, lane, 0);
                lo[gi] = *reinterpret_cast<const uint32_t*>(src);
                hi[gi] = *reinterpret_cast<const uint32_t*>(src + 8);
            }
            if (VB == 4) {
                uint4 w = make_uint4(lo[0] | (hi[0] << 4), lo[1] | (hi[1] << 4), lo[2] | (hi[2] << 4), lo[3] | (hi[3] << 4));
                *reinterpret_cast<uint4*>(rec + LY::vcodes_off + lane * (D / 4) + 16 * q) = w;
            } else {
                uint2 w = make_uint2(lo[0] | (hi[0] << 2) | (lo[1] << 4) | (hi[1] << 6),
                                     lo[2] | (hi[2] << 2) | (lo[3] << 4) | (hi[3] << 6));
                *reinterpret_cast<uint2*>(rec + LY::vcodes_off + lane * (D / 8) + 8 * q) = w;
            }
        }
    } else if (tid < LY::NT * 64) {
        // ---- bit-pack the value codes: one lane triplet (three dwords, four coordinate groups) per thread
        const int q = tid >> 6;
        uint32_t lo[4], hi[4];  // codes e = 0..3 and e = 4..7 of each group, one per byte (consecutive tokens)
#pragma unroll
        for (int gi = 0; gi < 4; ++gi) {
            const int G = 4 * q + gi;
            const uint8_t* src = vstage + vcode_coord(G, lane) * VST + vcode_token(G, lane, 0);
            lo[gi] = *reinterpret_cast<const uint32_t*>(src);
            hi[gi] = *reinterpret_cast<const uint32_t*>(src + 8);
        }
        uint32_t w0 = lo[0] | (hi[0] << 3), w1 = lo[1] | (hi[1] << 3), w2 = lo[2] | (hi[2] << 3);
        w0 |= (lo[3] & 0x03030303u) << 6;
        w2 |= (hi[3] & 0x03030303u) << 6;
        w1 |= ((lo[3] & 0x04040404u) << 4) | ((hi[3] & 0x04040404u) << 5);
        uint32_t* out = reinterpret_cast<uint32_t*>(rec + LY::vcodes_off + q * 768 + lane * 12);
        out[0] = w0;
        out[1] = w1;
        out[2] = w2;
    }
    // ---- key codes and scales: 16-byte coalesced stores
    uint4* out = reinterpret_cast<uint4*>(rec);
    const uint4* src = reinterpret_cast<const uint4*>(kimg);
    for (int i = tid; i < KBYTES / 16; i += 256) out[i] = src[i];
}

// ------------------------------------------------------------------------------------ decode ---
template <int D, int VC, int KC>
__device__ __forceinline__ void stage_tile(uint8_t* img, const uint8_t* pool, int unit, int tiles,
                                           int tile, int tid) {
    using LY = Layout<D, VC, KC>;
    const uint4* src = reinterpret_cast<const uint4*>(pool + ((size_t)unit * tiles + tile) * LY::tile_bytes);
    uint4* dst = reinterpret_cast<uint4*>(img);
    for (int i = tid; i < LY::tile_bytes / 16; i += 256) dst[i] = src[i];
    __syncthreads();
}

template <typename OutT, int N> struct RowStore;
template <int N> struct RowStore<__half, N> {
    // N fp32 values -> N halves, 16-byte stores
    static __device__ __forceinline__ void store(__half* dst, const float (&x)[N]) {
#pragma unroll
        for (int i = 0; i < N / 8; ++i) {
            uint32_t w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                Half2Bits b;
                b.h[0] = (_Float16)x[8 * i + 2 * k];
                b.h[1] = (_Float16)x[8 * i + 2 * k + 1];
                w[k] = b.u;
            }
            stream_store16(reinterpret_cast<uint4*>(dst) + i, w[0], w[1], w[2], w[3]);
        }
    }
};
struct Bf16Out {  // output element type: a bfloat16 bit pattern
    uint16_t bits;
};
template <int N> struct RowStore<Bf16Out, N> {
    // N fp32 values -> N bfloat16 (round to nearest even; inputs are finite), 16-byte stores
    static __device__ __forceinline__ uint32_t rne(float x) {
        const uint32_t u = __float_as_uint(x);
        return u + 0x7FFFu + ((u >> 16) & 1u);
    }
    static __device__ __forceinline__ void store(Bf16Out* dst, const float (&x)[N]) {
#pragma unroll
        for (int i = 0; i < N / 8; ++i) {
            uint32_t w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)  // high halves of the two rounded words
                w[k] = __builtin_amdgcn_perm(rne(x[8 * i + 2 * k + 1]), rne(x[8 * i + 2 * k]), 0x07060302u);
            stream_store16(reinterpret_cast<uint4*>(dst) + i, w[0], w[1], w[2], w[3]);
        }
    }
};
template <int N> struct RowStore<float, N> {
    static __device__ __forceinline__ void store(float* dst, const float (&x)[N]) {
#pragma unroll
        for (int i = 0; i < N / 4; ++i)
            stream_store16(reinterpret_cast<float4*>(dst) + i, __float_as_uint(x[4 * i]), __float_as_uint(x[4 * i + 1]),
                           __float_as_uint(x[4 * i + 2]), __float_as_uint(x[4 * i + 3]));
    }
};

// K = code * s and V = H c[code] / sqrt(d)  (sections "Compression Scheme" and "TurboQuant",
// dequantization; the inverse of the normalized rotation is the same normalized transform); times the
// vector's scale in the scaled-values codec (VC = 1).  Int8 values (VC = 2): V = code * s, no rotation.
template <int D, int VC, typename OutT, int KC>
__global__ __launch_bounds__(256) void decode_kernel(const uint8_t* __restrict__ pool,
                                                     OutT* __restrict__ K_out, OutT* __restrict__ V_out,
                                                     int T, int tiles, SignBits signs,
                                                     const uint32_t* __restrict__ kmax, int H) {
    using LY = Layout<D, VC, KC>;
    constexpr int EPT = D / 8;
    constexpr int KBYTES = LY::vcodes_off;
    constexpr int VB = vc_bits(VC);
    constexpr bool VS = LY::has_vscales, V8 = VB == 8;
    constexpr int CS = D + 8;  // halves per token row of the centroid staging area (16-byte aligned rows)
    constexpr int VST = kTile + 4;  // int8 values: bytes per coordinate of the code staging area
    __shared__ __align__(16) uint8_t kimg[KBYTES];
    // 3-bit codecs: fp16 centroids (scaled), [token][coordinate]; int8 codec: code bytes, [coordinate][token]
    __shared__ __align__(16) uint8_t vbuf[V8 ? D * VST : kTile * CS * 2];
    _Float16* cent = reinterpret_cast<_Float16*>(vbuf);

    const int tile = blockIdx.x, unit = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint8_t* rec = pool + ((size_t)unit * tiles + tile) * LY::tile_bytes;
    const CodecThread th(tid);
    const int t = th.t, c = th.c;

    float vscale = 1.0f;
    if (VS && V_out != nullptr) vscale = (float)reinterpret_cast<const _Float16*>(rec + LY::vscales_off)[t];
    if (K_out != nullptr) {
        const uint4* src = reinterpret_cast<const uint4*>(rec);
        uint4* dst = reinterpret_cast<uint4*>(kimg);
        for (int i = tid; i < KBYTES / 16; i += 256) dst[i] = src[i];
    }
    if (V8) {
        for (int g = tid >> 6; V_out != nullptr && g < LY::NB; g += 4) {
            const uint4 w = *reinterpret_cast<const uint4*>(rec + LY::vcodes_off + g * 1024 + lane * 16);
            uint8_t* dst = vbuf + (32 * g + (lane & 31)) * VST + 4 * (lane >> 5);
            *reinterpret_cast<uint32_t*>(dst) = w.x;
            *reinterpret_cast<uint32_t*>(dst + 8) = w.y;
            *reinterpret_cast<uint32_t*>(dst + 16) = w.z;
            *reinterpret_cast<uint32_t*>(dst + 24) = w.w;
        }
    } else if (V_out != nullptr) {
      for (int x = tid; x < LY::NT * 128; x += 256) {
        // work item (half, q, lane): two of the four coordinate groups of one lane triplet
        const int half = x / (LY::NT * 64), ql = x - half * (LY::NT * 64);
        const int q = ql >> 6;
        uint32_t w0 = 0, w1 = 0, w2 = 0;
        if (VB == 3) {
            const uint32_t* w = reinterpret_cast<const uint32_t*>(rec + LY::vcodes_off + q * 768 + lane * 12);
            w0 = w[0], w1 = w[1], w2 = w[2];
        }
#pragma unroll
        for (int gg = 0; gg < 2; ++gg) {
            const int G = 4 * q + 2 * half + gg;
            Half2Bits c01, c23, c45, c67;
            if (VB == 3) {
                uint32_t sel_a, sel_b;
                if (half == 0)
                    vcode_selectors(w0, w1, w2, gg, sel_a, sel_b);
                else
                    vcode_selectors(w0, w1, w2, 2 + gg, sel_a, sel_b);
                lookup4(sel_a, c01.u, c23.u);
                lookup4(sel_b, c45.u, c67.u);
            } else {
                uint32_t o[4];
                if (VB == 4)
                    group8_b4(reinterpret_cast<const uint32_t*>(rec + LY::vcodes_off)[lane * (D / 16) + G], o);
                else
                    group8_b2(reinterpret_cast<const uint32_t*>(rec + LY::vcodes_off)[lane * (D / 32) + (G >> 1)], G & 1, o);
                c01.u = o[0], c23.u = o[1], c45.u = o[2], c67.u = o[3];
            }
            _Float16* col = cent + vcode_token(G, lane, 0) * CS + vcode_coord(G, lane);  // codes e: rows +0..3, +8..11
            col[0 * CS] = c01.h[0];
            col[1 * CS] = c01.h[1];
            col[2 * CS] = c23.h[0];
            col[3 * CS] = c23.h[1];
            col[8 * CS] = c45.h[0];
            col[9 * CS] = c45.h[1];
            col[10 * CS] = c67.h[0];
            col[11 * CS] = c67.h[1];
        }
      }
    }
    __syncthreads();

    // A thread's share of its token's row is every eighth 8-element piece: piece p = 8 * rr + c for rr = 0 ..
    // EPT/8 - 1.  The eight threads of a token then write one contiguous run per store instruction, and the
    // rotation does not care which index bits are in-lane and which are cross-lane.
    const int tok = tile * kTile + t;
    const bool valid = tok < T;
    const size_t row = ((size_t)unit * T + (valid ? tok : 0)) * D;
    constexpr int NP = EPT / 8;
    auto piece_of = [&](const float (&x)[EPT], int rr) -> const float(&)[8] {
        return *reinterpret_cast<const float(*)[8]>(&x[8 * rr]);
    };

    if (K_out != nullptr) {
        float k[EPT];
#pragma unroll
        for (int rr = 0; rr < NP; ++rr) {
            const int p = 8 * rr + c, j = p >> 2, g8 = p & 3;
            const _Float16 s16 = KC == 1 ? tensor_key_scale(kmax[unit / H])
                                         : reinterpret_cast<const _Float16*>(kimg + LY::kscales_off)[t * LY::NB + j];
            const uint2 raw = *reinterpret_cast<const uint2*>(kimg + LY::kcodes_off + kcode_run_offset(t, j, g8));
            Half2Bits h[4];
            codes4_to_half(raw.x, h[0].u, h[1].u);
            codes4_to_half(raw.y, h[2].u, h[3].u);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // (1024 + b) - 1152 = code, exact in fp16; code * s is exact in fp32
                k[8 * rr + 2 * i] = (float)(h[i].h[0] - (_Float16)1152.0f) * (float)s16;
                k[8 * rr + 2 * i + 1] = (float)(h[i].h[1] - (_Float16)1152.0f) * (float)s16;
            }
        }
        if (valid) {
#pragma unroll
            for (int rr = 0; rr < NP; ++rr) RowStore<OutT, 8>::store(K_out + row + 8 * (8 * rr + c), piece_of(k, rr));
        }
    }
    if (V8) {
        if (V_out != nullptr) {
            float y[EPT];
#pragma unroll
            for (int i = 0; i < EPT; ++i)  // exact in fp32
                y[i] = (float)((int)vbuf[(8 * (8 * (i >> 3) + c) + (i & 7)) * VST + t] - 128) * vscale;
            if (valid) {
#pragma unroll
                for (int rr = 0; rr < NP; ++rr) RowStore<OutT, 8>::store(V_out + row + 8 * (8 * rr + c), piece_of(y, rr));
            }
        }
    } else if (V_out != nullptr) {
        // the centroid scale, 1/sqrt(D) and the entry sign of the cross-lane stages ride on the conversion
        const float f = codec_entry_sign(lane) * (inv_centroid_scale<VB>() * inv_sqrt_d<D>()) * vscale;
        float y[EPT];
#pragma unroll
        for (int rr = 0; rr < NP; ++rr) {
            const uint4 raw = *reinterpret_cast<const uint4*>(cent + t * CS + 8 * (8 * rr + c));
            const uint32_t* w = reinterpret_cast<const uint32_t*>(&raw);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                Half2Bits b;
                b.u = w[k];
                y[8 * rr + 2 * k] = __builtin_fmaf((float)b.h[0], f, 0.0f);
                y[8 * rr + 2 * k + 1] = __builtin_fmaf((float)b.h[1], f, 0.0f);
            }
        }
        wht_cross_chunks<EPT>(y, lane);
        wht_inlane<EPT>(y);
        if (signs.on) {  // inverse of H.D: D last
#pragma unroll
            for (int rr = 0; rr < NP; ++rr) {
                const int p = 8 * rr + c;
                float(&y8)[8] = *reinterpret_cast<float(*)[8]>(&y[8 * rr]);
                flip_signs<8>(y8, sign_word(signs, p >> 2) >> (8 * (p & 3)));
            }
        }
        if (valid) {
#pragma unroll
            for (int rr = 0; rr < NP; ++rr) RowStore<OutT, 8>::store(V_out + row + 8 * (8 * rr + c), piece_of(y, rr));
        }
    }
}

// ------------------------------------------------------------------------------------ export ---
template <int D, int VC, int KC>
__global__ __launch_bounds__(256) void export_kernel(const uint8_t* __restrict__ pool,
                                                     int8_t* __restrict__ k_codes,
                                                     __half* __restrict__ k_scales,
                                                     uint8_t* __restrict__ v_packed,
                                                     __half* __restrict__ v_scales, int T, int tiles,
                                                     const uint32_t* __restrict__ kmax, int H) {
    using LY = Layout<D, VC, KC>;
    constexpr int VB = vc_bits(VC);
    constexpr bool VS = LY::has_vscales, V8 = VB == 8;
    constexpr int EPT = D / 8;
    __shared__ __align__(16) uint8_t img[LY::tile_bytes];
    const int tile = blockIdx.x, unit = blockIdx.y;
    const int tid = threadIdx.x, t = tid >> 3, c = tid & 7;
    stage_tile<D, VC, KC>(img, pool, unit, tiles, tile, tid);
    if (KC == 1 && k_scales != nullptr && tile == 0 && unit % H == 0 && tid == 0)  // one scale per layer
        k_scales[unit / H] = (__half)tensor_key_scale(kmax[unit / H]);
    const int tok = tile * kTile + t;
    if (tok >= T) return;
    const size_t vec = (size_t)unit * T + tok;
    const int e0 = c * EPT, j = e0 >> 5, g8 = (e0 >> 3) & 3;
    if (k_codes != nullptr) {
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const uint8_t* codes = img + LY::kcodes_off + kcode_run_offset(t, j, g8 + (i >> 3));
            k_codes[vec * D + e0 + i] = (int8_t)((int)codes[i & 7] - 128);
        }
    }
    if (KC == 0 && k_scales != nullptr && c < LY::NB)
        k_scales[vec * LY::NB + c] = reinterpret_cast<const __half*>(img + LY::kscales_off)[t * LY::NB + c];
    if (VS && v_scales != nullptr && c == 0)
        v_scales[vec] = reinterpret_cast<const __half*>(img + LY::vscales_off)[t];
    if (V8) {
        if (v_packed != nullptr) {  // int8 codes, [head_dim] per vector
#pragma unroll
            for (int i = 0; i < EPT; ++i)
                v_packed[vec * D + e0 + i] = (uint8_t)((int)img[LY::vcodes_off + v8_byte_offset(t, e0 + i)] - 128);
        }
    } else if (VB != 3) {
        if (v_packed != nullptr) {  // canonical codes (ascending over all centroids), VB bits each, LSB first
            const uint32_t* vreg = reinterpret_cast<const uint32_t*>(img + LY::vcodes_off);
            constexpr int half = 1 << (VB - 1), PER = 8 / VB;
            uint8_t* dst = v_packed + vec * (VB * D / 8) + VB * e0 / 8;
#pragma unroll
            for (int b = 0; b < EPT / PER; ++b) {
                uint32_t byte = 0;
#pragma unroll
                for (int i = 0; i < PER; ++i) {
                    const int sm = VB == 4 ? vcode_extract_b4(vreg, D, t, e0 + b * PER + i) : vcode_extract_b2(vreg, D, t, e0 + b * PER + i);
                    const int code = (sm & half) ? half - 1 - (sm & (half - 1)) : half + sm;
                    byte |= (uint32_t)code << (VB * i);
                }
                dst[b] = (uint8_t)byte;
            }
        }
    } else if (v_packed != nullptr) {
        const uint32_t* vreg = reinterpret_cast<const uint32_t*>(img + LY::vcodes_off);
        uint8_t* dst = v_packed + vec * (3 * D / 8) + 3 * e0 / 8;
#pragma unroll
        for (int g8 = 0; g8 < EPT / 8; ++g8) {
            uint32_t bits = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) bits |= (uint32_t)vcode_extract(vreg, t, e0 + g8 * 8 + i) << (3 * i);
            dst[g8 * 3 + 0] = bits & 0xFF;
            dst[g8 * 3 + 1] = (bits >> 8) & 0xFF;
            dst[g8 * 3 + 2] = (bits >> 16) & 0xFF;
        }
    }
}

// ---------------------------------------------------------------- per-tensor key scale: max|k| ---
__global__ void zero_u32_kernel(uint32_t* __restrict__ p, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0u;
}

// max|k| of every layer tensor, first pass of the key formula with one scale per tensor (section
// "Compression Scheme", key quantization).  Same thread -> (token, chunk) map as the encode kernel; a
// workgroup strides over the tiles of its KV head and issues one atomic at the end (non-negative floats
// order like their bit patterns), so a layer's maximum sees a few thousand atomics, not one per tile.
template <int D, bool BF>
__global__ __launch_bounds__(256) void kamax_kernel(const __half* __restrict__ K, uint32_t* __restrict__ kmax, int T,
                                                    int H) {
    constexpr int EPT = D / 8;
    __shared__ float wmax[4];
    const int unit = blockIdx.y, tid = threadIdx.x;
    const CodecThread th(tid);
    float amax = 0.0f;
    for (int tok = blockIdx.x * kTile + th.t; tok < T; tok += gridDim.x * kTile) {
        const uint4* src = reinterpret_cast<const uint4*>(K + ((size_t)unit * T + tok) * D + th.c * EPT);
#pragma unroll
        for (int i = 0; i < EPT / 8; ++i) {
            const uint4 raw = src[i];
            const uint32_t* w = reinterpret_cast<const uint32_t*>(&raw);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float2 f = pair16_to_float2(w[k], BF);
                amax = fmaxf(amax, fmaxf(fabsf(f.x), fabsf(f.y)));
            }
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m, 64));
    if ((tid & 63) == 0) wmax[tid >> 6] = amax;
    __syncthreads();
    if (tid == 0) {
        const float m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
        atomicMax(&kmax[unit / H], __float_as_uint(m));
    }
}

// ---------------------------------------------------------------------------------- launchers ---
// Calls f(integral_constant<int, D>, integral_constant<int, VC>, integral_constant<int, KC>) for the pool's
// head_dim, value codec and key codec.
template <typename F> static void for_pool_shape(const polykv_pool* p, F&& f) {
    using std::integral_constant;
    auto with_dv = [&](auto d, auto vc) {
        if (p->key_codec == POLYKV_KEYS_Q8_TENSOR)
            f(d, vc, integral_constant<int, POLYKV_KEYS_Q8_TENSOR>{});
        else
            f(d, vc, integral_constant<int, POLYKV_KEYS_Q8_BLOCK32>{});
    };
    auto with_d = [&](auto d) {
        switch (p->value_codec) {
            case 1: with_dv(d, integral_constant<int, 1>{}); break;
            case 2: with_dv(d, integral_constant<int, 2>{}); break;
            case 3: with_dv(d, integral_constant<int, 3>{}); break;
            case 4: with_dv(d, integral_constant<int, 4>{}); break;
            case 5: with_dv(d, integral_constant<int, 5>{}); break;
            case 6: with_dv(d, integral_constant<int, 6>{}); break;
            default: with_dv(d, integral_constant<int, 0>{}); break;
        }
    };
    if (p->head_dim == 128)
        with_d(integral_constant<int, 128>{});
    else if (p->head_dim == 64)
        with_d(integral_constant<int, 64>{});
    else
        with_d(integral_constant<int, 256>{});
}

// The layers' max|k| inside the pool's storage (POLYKV_KEYS_Q8_TENSOR), else nullptr.
static uint32_t* kmax_of(const polykv_pool* p) {
    return p->key_codec == POLYKV_KEYS_Q8_TENSOR ? reinterpret_cast<uint32_t*>((char*)p->storage + p->kmax_off) : nullptr;
}

hipError_t launch_encode(const polykv_pool* p, const void* K, const void* V, int in_dtype, int begin, int count,
                         hipStream_t s) {
    const int end = begin + count;
    const int units = p->layers * p->kv_heads;
    dim3 grid(tiles_of(end) - begin / kTile, units);
    uint32_t* kmax = kmax_of(p);
    for_pool_shape(p, [&](auto d, auto vs, auto kc) {
        constexpr int D = decltype(d)::value, VC = decltype(vs)::value, KC = decltype(kc)::value;
        if (KC == 1) {  // first pass of the per-tensor key formula: the layers' max|k| (begin is 0 here)
            zero_u32_kernel<<<1, 256, 0, s>>>(kmax, p->layers);
            const dim3 mgrid(min(tiles_of(count), 8), units);
            if (in_dtype == POLYKV_BF16)
                kamax_kernel<D, true><<<mgrid, 256, 0, s>>>((const __half*)K, kmax, count, p->kv_heads);
            else
                kamax_kernel<D, false><<<mgrid, 256, 0, s>>>((const __half*)K, kmax, count, p->kv_heads);
        }
        if (in_dtype == POLYKV_BF16)
            launch_main_kernel(encode_kernel<D, VC, true, KC>, grid, dim3(256), 0, s, (const __half*)K, (const __half*)V,
                               (uint8_t*)p->storage, count, begin, end, p->tiles, p->signs, (const uint32_t*)kmax,
                               p->kv_heads);
        else
            launch_main_kernel(encode_kernel<D, VC, false, KC>, grid, dim3(256), 0, s, (const __half*)K, (const __half*)V,
                               (uint8_t*)p->storage, count, begin, end, p->tiles, p->signs, (const uint32_t*)kmax,
                               p->kv_heads);
    });
    return hipGetLastError();
}

hipError_t launch_decode(const polykv_pool* p, void* K_out, void* V_out, int dtype, int layer_begin, int layer_end,
                         hipStream_t s) {
    dim3 grid(tiles_of(p->length), (layer_end - layer_begin) * p->kv_heads);  // the tokens encoded so far
    const uint8_t* pool = (const uint8_t*)p->storage + (size_t)layer_begin * p->kv_heads * p->tiles * p->tile_bytes;
    const uint32_t* kmax = kmax_of(p) ? kmax_of(p) + layer_begin : nullptr;
    for_pool_shape(p, [&](auto d, auto vs, auto kc) {
        constexpr int D = decltype(d)::value, VC = decltype(vs)::value, KC = decltype(kc)::value;
        if (dtype == POLYKV_BF16)
            launch_main_kernel(decode_kernel<D, VC, Bf16Out, KC>, grid, dim3(256), 0, s, pool, (Bf16Out*)K_out,
                               (Bf16Out*)V_out, p->length, p->tiles, p->signs, kmax, p->kv_heads);
        else if (dtype == POLYKV_F32)
            launch_main_kernel(decode_kernel<D, VC, float, KC>, grid, dim3(256), 0, s, pool, (float*)K_out, (float*)V_out,
                               p->length, p->tiles, p->signs, kmax, p->kv_heads);
        else
            launch_main_kernel(decode_kernel<D, VC, __half, KC>, grid, dim3(256), 0, s, pool, (__half*)K_out,
                               (__half*)V_out, p->length, p->tiles, p->signs, kmax, p->kv_heads);
    });
    return hipGetLastError();
}

hipError_t launch_export(const polykv_pool* p, void* kc_out, void* ks, void* vp, void* vs_out, hipStream_t s) {
    dim3 grid(tiles_of(p->length), p->layers * p->kv_heads);  // the tokens encoded so far
    const uint8_t* pool = (const uint8_t*)p->storage;
    const uint32_t* kmax = kmax_of(p);
    for_pool_shape(p, [&](auto d, auto vs, auto kc) {
        export_kernel<decltype(d)::value, decltype(vs)::value, decltype(kc)::value><<<grid, 256, 0, s>>>(
            pool, (int8_t*)kc_out, (__half*)ks, (uint8_t*)vp, (__half*)vs_out, p->length, p->tiles, kmax, p->kv_heads);
    });
    return hipGetLastError();
}

}  // namespace polykv
