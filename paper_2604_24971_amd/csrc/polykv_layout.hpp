// In-HBM layout of the packed pool and small device helpers shared by the kernels.
//
// The pool is an array of tile records, [layer*kv_head][tile], one tile = 32 consecutive tokens of
// one KV head (the last tile is zero-padded).  A record is laid out for the matrix-core attention
// kernel (v_mfma_f32_32x32x16_f16) so that every wave load is one contiguous, fully coalesced run and
// lands in registers in MFMA operand order.  "lane" below is a wave lane 0..63 = 32*h + m.
//
//   K codes   NB x 1024 B    NB = head_dim/32 q8_0 blocks.  Byte j*1024 + lane*16 + 8*s + e holds
//                            code(token m, element 32j + 16s + 8h + e) + 128 (offset binary),
//                            j < NB, s < 2, e < 8: the lane's 16 bytes of block j are the A operands
//                            (8 k-values each) of the block's two K=16 MFMA slices, M = token.
//   K scales  32 x NB fp16   scale(token t, block j) at index t*NB + j.
//   V codes   NT x 768 B     NT = head_dim/64 triplets.  Triplet q, lane: three dwords at byte
//                            q*768 + lane*12.  They carry four groups of eight 3-bit codes, group
//                            G = 4q + {0,1,2,3}; group G belongs to rotated coordinate 32*(G/2) + m and
//                            its code e (0..7) to token 16*(G%2) + 8*(e/4) + 4*h + e%4: the k-order in
//                            which a 32x32 score tile leaves the MFMA accumulators, so the
//                            probabilities feed the P.V products without any data movement.
//                            Groups 4q+0..2 sit in dword 0..2: code e at bit 8*(e%4) + 3*(e/4).
//                            Group 4q+3 uses the two spare top bits of every byte:
//                              code e<4 : bits 1:0 = dword0 bits 8e+7:8e+6, bit 2 = dword1 bit 8e+6
//                              code e>=4: bits 1:0 = dword2 bits 8(e-4)+7:8(e-4)+6, bit 2 = dword1 bit 8(e-4)+7
//
//
// Value codecs with a per-vector scale (VC = 1, 2) put a region of 32 fp16 scales, one per token,
// between the key scales and the value codes:
//   V scales  32 fp16        scale(token t) at index t.
// The int8 value codec (VC = 2) stores, instead of the 3-bit triplets,
//   V codes   NB x 1024 B    byte g*1024 + lane*16 + 8*ks + e holds code(coordinate 32g + m, token
//                            16ks + 8*(e/4) + 4h + e%4) + 128, g < NB, ks < 2, e < 8: the lane's 16 bytes of
//                            coordinate group g are the A operands of that group's two P.V products, in the
//                            same token order as above.
//
// With one key scale per layer tensor (KC = 1) the K-scales region is absent; the layer maxima live in a
// small array behind all records (see polykv_pool::kmax_off).
//
// Per token and KV head this is head_dim + head_dim/16 + 3*head_dim/8 bytes: 184 (d=128), 92 (d=64),
// plus 2 with value scales; 2*head_dim + head_dim/16 + 2 with int8 values; head_dim/16 less with KC = 1.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace polykv {

constexpr int kTile = 32;  // tokens per tile record

// Value codecs, numbered as POLYKV_VALUES_* in the ABI header: 0 the paper's 3-bit codes, 1 the same with a
// per-vector scale, 2 int8 codes with a per-vector scale, 3 / 4 two-bit codes without / with the scale,
// 5 / 6 four-bit codes without / with it.
constexpr int vc_bits(int vc) { return vc == 2 ? 8 : (vc == 3 || vc == 4) ? 2 : (vc == 5 || vc == 6) ? 4 : 3; }
constexpr bool vc_has_scale(int vc) { return vc == 1 || vc == 2 || vc == 4 || vc == 6; }
constexpr int kNumValueCodecs = 7;

// The 2-bit and 4-bit codes are stored as sign and magnitude: top bit set = negative, the other bits = the
// number of positive thresholds below |v_rot| (the canonical code, ascending over all centroids, is
// half - 1 - magnitude for negative and half + magnitude for positive values, half = 2^(bits-1)).  Per lane
// and coordinate group G (as for the 3-bit codes: coordinate 32*(G/2) + m, code e = token
// 16*(G%2) + 8*(e/4) + 4h + e%4):
//   4 bits   one dword per G, the lane's D/16 dwords contiguous at byte lane*(D/4) + 4G: code e < 4 in the low
//            nibble of byte e, code e >= 4 in the high nibble of byte e - 4;
//   2 bits   half a dword per G, the lane's D/32 dwords contiguous at byte lane*(D/8) + 4*(G/2): code e of
//            group G at bit 8*(e%4) + 2*(2*(G%2) + e/4).
// VC: value codec.
// KC: key codec, POLYKV_KEYS_* (0 q8_0 blocks of 32 with a scale each, 1 one scale per layer tensor).
template <int D, int VC = 0, int KC = 0> struct Layout {
    static constexpr int NB = D / 32;             // q8_0 blocks per vector
    static constexpr int NT = D / 64;             // value-code triplets per lane
    static constexpr bool has_vscales = vc_has_scale(VC);
    static constexpr int vbits = vc_bits(VC);
    static constexpr bool has_kscales = KC == 0;
    static constexpr int kcodes_off = 0;
    static constexpr int kscales_off = NB * 1024;                     // present only if has_kscales
    static constexpr int vscales_off = kscales_off + (has_kscales ? kTile * NB * 2 : 0);  // only if has_vscales
    static constexpr int vcodes_off = vscales_off + (has_vscales ? kTile * 2 : 0);
    static constexpr int tile_bytes =
        vcodes_off + (vbits == 8 ? NB * 1024 : vbits == 3 ? NT * 768 : vbits == 4 ? D * 16 : D * 8);
};

__host__ __device__ inline int tiles_of(int tokens) { return (tokens + kTile - 1) / kTile; }

// Lloyd-Max codebook for N(0,1), 8 levels: the converged fixed point of Lloyd's iteration
// (thresholds = midpoints of neighbouring centroids, centroids = conditional means of their cells),
// rounded to fp32.  They agree to three decimals with the values printed in the paper's section
// "TurboQuant".
#define POLYKV_C0 0.24509418f
#define POLYKV_C1 0.75600528f
#define POLYKV_C2 1.34390928f
#define POLYKV_C3 2.15194570f
#define POLYKV_T1 0.50054973f
#define POLYKV_T2 1.04995728f
#define POLYKV_T3 1.74792749f

__device__ __forceinline__ float centroid_of(int code) {
    // code 0..7 ascending; symmetric table
    const int m = (code & 4) ? (code & 3) : (3 - code);
    float c = (m == 0) ? POLYKV_C0 : (m == 1) ? POLYKV_C1 : (m == 2) ? POLYKV_C2 : POLYKV_C3;
    return (code & 4) ? c : -c;
}

// Number of thresholds strictly below x (thresholds -T3,-T2,-T1,0,T1,T2,T3).
__device__ __forceinline__ int quantize3(float x) {
    int n = 0;
    n += x > -POLYKV_T3;
    n += x > -POLYKV_T2;
    n += x > -POLYKV_T1;
    n += x > 0.0f;
    n += x > POLYKV_T1;
    n += x > POLYKV_T2;
    n += x > POLYKV_T3;
    return n;
}

// Byte offset (inside the K-code region of a tile) of the 8-byte run holding elements
// 32j + 8*g8 .. +7 of token t (g8 = 0..3).
__device__ __forceinline__ int kcode_run_offset(int t, int j, int g8) {
    return j * 1024 + (32 * (g8 & 1) + t) * 16 + (g8 >> 1) * 8;
}

// Value-code group G of a lane: its rotated coordinate, and the token (within the tile) of its code e.
__device__ __forceinline__ int vcode_coord(int G, int lane) { return 32 * (G >> 1) + (lane & 31); }
__device__ __forceinline__ int vcode_token(int G, int lane, int e) {
    return 16 * (G & 1) + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
}

// int8 value codec: byte offset (inside the V-code region of a tile) of the code of (token t of the tile,
// coordinate dv).
__device__ __forceinline__ int v8_byte_offset(int t, int dv) {
    const int ks = t >> 4, e = (((t >> 3) & 1) << 2) | (t & 3), lane = 32 * ((t >> 2) & 1) + (dv & 31);
    return (dv >> 5) * 1024 + lane * 16 + 8 * ks + e;
}

// Extract the 3-bit value code of (token t of the tile, rotated coordinate dv) from the V-code
// region `v` (dword view) of a tile.
__device__ __forceinline__ int vcode_extract(const uint32_t* v, int t, int dv) {
    const int G = 2 * (dv >> 5) + (t >> 4), q = G >> 2, gi = G & 3;
    const int e = (((t >> 3) & 1) << 2) | (t & 3), lane = 32 * ((t >> 2) & 1) + (dv & 31);
    const uint32_t* w = v + q * 192 + lane * 3;
    if (gi < 3) return (w[gi] >> (8 * (e & 3) + 3 * (e >> 2))) & 7;
    if (e < 4) return ((w[0] >> (8 * e + 6)) & 3) | (((w[1] >> (8 * e + 6)) & 1) << 2);
    return ((w[2] >> (8 * (e - 4) + 6)) & 3) | (((w[1] >> (8 * (e - 4) + 7)) & 1) << 2);
}

// One key scale per layer tensor: the layer's max|k| (fp32 bits, kept behind the records) -> the fp16
// scale max|k| / 127, saturating at the fp16 maximum; the same expression in every kernel.
__device__ __forceinline__ _Float16 tensor_key_scale(uint32_t amax_bits) {
    return (_Float16)fminf(__fdiv_rn(__uint_as_float(amax_bits), 127.0f), 65504.0f);
}

// ---- sign diagonal of the rotation variant (struct SignBits: bit i set = coordinate i negated) ---
// The 32-bit word holding coordinates 32*idx .. 32*idx+31; idx may differ between lanes.
template <typename S> __device__ __forceinline__ uint32_t sign_word(const S& s, int idx) {
    uint32_t r = s.w[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) r = idx == k ? s.w[k] : r;
    return r;
}
// Negates y[i] where bit i of `bits` is set (y[i] = coordinate e0 + i, bits = sign_word(e0 / 32) >> (e0 % 32)).
template <int N> __device__ __forceinline__ void flip_signs(float (&y)[N], uint32_t bits) {
    static_assert(N <= 32, "");
#pragma unroll
    for (int i = 0; i < N; ++i) y[i] = __uint_as_float(__float_as_uint(y[i]) ^ ((bits << (31 - i)) & 0x80000000u));
}

// ---- 16-bit floating-point inputs: fp16, or bfloat16 (the top half of an fp32) ------------------
// Two packed 16-bit values -> fp32; `bf` is uniform over the wave.
__device__ __forceinline__ float2 pair16_to_float2(uint32_t w, bool bf) {
    if (bf) return make_float2(__uint_as_float(w << 16), __uint_as_float(w & 0xFFFF0000u));
    union {
        uint32_t u;
        _Float16 h[2];
    } b;
    b.u = w;
    return make_float2((float)b.h[0], (float)b.h[1]);
}
__device__ __forceinline__ float bits16_to_float(uint16_t bits, bool bf) {
    if (bf) return __uint_as_float((uint32_t)bits << 16);
    union {
        uint16_t u;
        _Float16 h;
    } b;
    b.u = bits;
    return (float)b.h;
}

// ---- register-level dequantization helpers shared by the decode and attention kernels ---------
// Centroids scaled by 1.6146639585494995 and rounded to fp16.  The factor was searched in [1, 2) so
// that all four magnitudes land within 1.9e-5 (relative) of an fp16 value -- ten times closer than the
// unscaled centroids; its inverse is applied once per output row.
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

// ---- 2-bit and 4-bit codebooks (Lloyd-Max for N(0,1), positive half; rounded to fp32) -------------------
__device__ __host__ inline float centroid_mag(int bits, int i) {
    constexpr float c2[2] = {0.452780038f, 1.51041758f};
    constexpr float c3[4] = {POLYKV_C0, POLYKV_C1, POLYKV_C2, POLYKV_C3};
    constexpr float c4[8] = {0.128395036f, 0.388048291f, 0.656759143f, 0.942340434f,
                             1.25623119f,  1.6180464f,   2.06901717f,  2.73258948f};
    return bits == 2 ? c2[i] : bits == 4 ? c4[i] : c3[i];
}
__device__ __host__ inline float threshold_mag(int bits, int i) {  // the i-th positive threshold
    constexpr float t2[1] = {0.981598794f};
    constexpr float t3[3] = {POLYKV_T1, POLYKV_T2, POLYKV_T3};
    constexpr float t4[7] = {0.258221656f, 0.522403717f, 0.799549758f, 1.09928584f, 1.4371388f, 1.84353185f, 2.40080333f};
    return bits == 2 ? t2[i] : bits == 4 ? t4[i] : t3[i];
}
// Centroid of a sign-magnitude code (2 or 4 bits).
__device__ __forceinline__ float centroid_signmag(int bits, int code) {
    const int half = 1 << (bits - 1);
    const float c = centroid_mag(bits, code & (half - 1));
    return (code & half) ? -c : c;
}
// As for the 3-bit table: magnitudes times a factor searched in [1, 2) so that they land close to fp16 values
// (4 bits: 1.3338515, within 9.3e-5; 2 bits: 1.9810335, within 2.7e-7); the inverse goes on the output row.
template <int BITS> __device__ __host__ constexpr float inv_centroid_scale() {
    return BITS == 4 ? 0.7497086444780398f : BITS == 2 ? 0.5047870215218471f : kInvCentroidScale;
}
// fp16 patterns of the scaled magnitudes, byte planes.  4 bits: 317B 3824 3B02 3D07 3EB4 4051 4185 434A.
constexpr uint32_t kTab4LoA = 0x0702247Bu, kTab4LoB = 0x4A8551B4u, kTab4HiA = 0x3D3B3831u, kTab4HiB = 0x4341403Eu;
// 2 bits: 3B2D 41FC.
constexpr uint32_t kTab2Lo = 0x0000FC2Du, kTab2Hi = 0x0000413Bu;

// Four 4-bit sign-magnitude codes: magnitudes in the bytes of `sel` (0..7), `sign` = 0x80 in the bytes of the
// negative ones -> four fp16 centroids.
__device__ __forceinline__ void lookup4_b4(uint32_t sel, uint32_t sign, uint32_t& out01, uint32_t& out23) {
    const uint32_t lo = __builtin_amdgcn_perm(kTab4LoB, kTab4LoA, sel);
    const uint32_t hi = __builtin_amdgcn_perm(kTab4HiB, kTab4HiA, sel) | sign;
    out01 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
    out23 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
}
// The same for 2-bit codes: magnitudes 0..1 in the bytes of `sel`.
__device__ __forceinline__ void lookup4_b2(uint32_t sel, uint32_t sign, uint32_t& out01, uint32_t& out23) {
    const uint32_t lo = __builtin_amdgcn_perm(0u, kTab2Lo, sel);
    const uint32_t hi = __builtin_amdgcn_perm(0u, kTab2Hi, sel) | sign;
    out01 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
    out23 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
}
// Eight codes of coordinate group G from the lane's dword `w` -> eight fp16 centroids (four dwords, codes e
// in order).  4 bits: w is the group's dword; 2 bits: w is the dword of the pair G/2 and `odd` = G % 2.
__device__ __forceinline__ void group8_b4(uint32_t w, uint32_t (&out)[4]) {
    lookup4_b4(w & 0x07070707u, (w << 4) & 0x80808080u, out[0], out[1]);
    lookup4_b4((w >> 4) & 0x07070707u, w & 0x80808080u, out[2], out[3]);
}
__device__ __forceinline__ void group8_b2(uint32_t w, int odd, uint32_t (&out)[4]) {
    const uint32_t v = odd ? w >> 4 : w;   // slots 2*odd and 2*odd + 1 now sit at bits 0..1 and 2..3 of every byte
    lookup4_b2(v & 0x01010101u, (v << 6) & 0x80808080u, out[0], out[1]);
    lookup4_b2((v >> 2) & 0x01010101u, (v << 4) & 0x80808080u, out[2], out[3]);
}
// The sign-magnitude code of (token t of the tile, rotated coordinate dv) from the V-code region (dword view).
__device__ __forceinline__ int vcode_extract_b4(const uint32_t* v, int D, int t, int dv) {
    const int G = 2 * (dv >> 5) + (t >> 4), e = (((t >> 3) & 1) << 2) | (t & 3), lane = 32 * ((t >> 2) & 1) + (dv & 31);
    return (v[lane * (D / 16) + G] >> (8 * (e & 3) + 4 * (e >> 2))) & 15;
}
__device__ __forceinline__ int vcode_extract_b2(const uint32_t* v, int D, int t, int dv) {
    const int G = 2 * (dv >> 5) + (t >> 4), e = (((t >> 3) & 1) << 2) | (t & 3), lane = 32 * ((t >> 2) & 1) + (dv & 31);
    return (v[lane * (D / 32) + (G >> 1)] >> (8 * (e & 3) + 2 * (2 * (G & 1) + (e >> 2)))) & 3;
}

// Value-code selectors of one lane's triplet (w0, w1, w2): group gi (0..3) -> the codes of its eight
// tokens, e = 0..3 in the bytes of sel_a and e = 4..7 in the bytes of sel_b.  m7, m3, m4 are the byte masks
// 0x07070707, 0x03030303 and 0x04040404: a caller whose loop is bound by instruction fetch keeps them in
// registers (as literals they would double the size of the instructions that use them).
__device__ __forceinline__ void vcode_selectors(uint32_t w0, uint32_t w1, uint32_t w2, int gi, uint32_t m7, uint32_t m3,
                                                uint32_t m4, uint32_t& sel_a, uint32_t& sel_b) {
    if (gi < 3) {
        const uint32_t w = gi == 0 ? w0 : gi == 1 ? w1 : w2;
        sel_a = w & m7;
        sel_b = (w >> 3) & m7;
    } else {
        sel_a = ((w0 >> 6) & m3) | ((w1 >> 4) & m4);
        sel_b = ((w2 >> 6) & m3) | ((w1 >> 5) & m4);
    }
}
__device__ __forceinline__ void vcode_selectors(uint32_t w0, uint32_t w1, uint32_t w2, int gi, uint32_t& sel_a,
                                                uint32_t& sel_b) {
    vcode_selectors(w0, w1, w2, gi, 0x07070707u, 0x03030303u, 0x04040404u, sel_a, sel_b);
}

// ---- Walsh-Hadamard stages across the 8 lanes that share a token in the codec kernels ----------
// Codec thread layout: lane bits 0, 1 and 3 carry the chunk index c (c = b0 + 2*b1 + 4*b3), the other
// lane bits and the wave index carry the token.  Each of the three partner exchanges (lane ^ 1,
// lane ^ 2, lane ^ 8) is then a single DPP pattern, and a butterfly stage is ONE instruction per
// element:  y += kappa * y[partner]  (v_fmac_f32 with a DPP source).  That computes the true stage
// output up to a per-lane sign; the signs of the three stages multiply to codec_entry_sign(), which
// the caller applies when it converts its inputs to fp32 (for free, in the conversion's multiply),
// so that what comes out is exactly H applied over the chunk index bits.
__device__ __forceinline__ int codec_chunk(int lane) { return (lane & 3) | ((lane >> 1) & 4); }
__device__ __forceinline__ int codec_token_in_wave(int lane) { return ((lane >> 2) & 1) | ((lane >> 3) & 6); }
__device__ __forceinline__ float codec_entry_sign(int lane) {
    return (__builtin_popcount(lane & 0xB) & 1) ? -1.0f : 1.0f;
}
// kappa of the stage over lane bit `bit`: +1 where the bit is set, -1 where it is clear
__device__ __forceinline__ float codec_kappa(int lane, int bit) { return (lane >> bit) & 1 ? 1.0f : -1.0f; }

// The three cross-lane stages on N values per lane.  On entry y holds codec_entry_sign() * x.
template <int N> __device__ __forceinline__ void wht_cross_chunks(float (&y)[N], int lane) {
    static_assert(N % 8 == 0, "");
    const float k0 = codec_kappa(lane, 0), k1 = codec_kappa(lane, 1), k3 = codec_kappa(lane, 3);
#pragma unroll
    for (int b = 0; b < N; b += 8) {
        // A DPP source must not have been written by the two preceding instructions: the leading
        // s_nop covers the block entry, inside the block every register is reused 8 instructions later.
        asm volatile(
            "s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %0, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %1, %1, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %2, %2, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %3, %3, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %4, %4, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %5, %5, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %6, %6, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %7, %7, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %0, %0, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %1, %1, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %2, %2, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %3, %3, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %4, %4, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %5, %5, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %6, %6, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %7, %7, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %0, %0, %10 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %1, %1, %10 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %2, %2, %10 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %3, %3, %10 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %4, %4, %10 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %5, %5, %10 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %6, %6, %10 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %7, %7, %10 row_ror:8 row_mask:0xf bank_mask:0xf"
            : "+v"(y[b]), "+v"(y[b + 1]), "+v"(y[b + 2]), "+v"(y[b + 3]), "+v"(y[b + 4]), "+v"(y[b + 5]),
              "+v"(y[b + 6]), "+v"(y[b + 7])
            : "v"(k0), "v"(k1), "v"(k3));
    }
}

// The same one-instruction butterfly for vectors spread over the four lanes of a quad (lane bits 0
// and 1 carry the two top index bits).  On entry y holds quad_entry_sign() * x.
__device__ __forceinline__ float quad_entry_sign(int lane) { return (__builtin_popcount(lane & 3) & 1) ? -1.0f : 1.0f; }
template <int N> __device__ __forceinline__ void wht_cross_quad(float (&y)[N], int lane) {
    static_assert(N % 8 == 0, "");
    const float k0 = codec_kappa(lane, 0), k1 = codec_kappa(lane, 1);
#pragma unroll
    for (int b = 0; b < N; b += 8) {
        asm volatile(
            "s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %0, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %1, %1, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %2, %2, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %3, %3, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %4, %4, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %5, %5, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %6, %6, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %7, %7, %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %0, %0, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %1, %1, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %2, %2, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %3, %3, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %4, %4, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %5, %5, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %6, %6, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %7, %7, %9 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
            : "+v"(y[b]), "+v"(y[b + 1]), "+v"(y[b + 2]), "+v"(y[b + 3]), "+v"(y[b + 4]), "+v"(y[b + 5]),
              "+v"(y[b + 6]), "+v"(y[b + 7])
            : "v"(k0), "v"(k1));
    }
}

// ---- cross-lane butterflies -------------------------------------------------------------------
// Partner exchange lane ^ MASK with DPP where a single control word exists, ds_bpermute otherwise.
template <int MASK> __device__ __forceinline__ float lane_xor(float x) {
    int xi = __float_as_int(x), r;
    if constexpr (MASK == 1) {
        r = __builtin_amdgcn_update_dpp(xi, xi, 0xB1, 0xF, 0xF, false);  // quad_perm [1,0,3,2]
    } else if constexpr (MASK == 2) {
        r = __builtin_amdgcn_update_dpp(xi, xi, 0x4E, 0xF, 0xF, false);  // quad_perm [2,3,0,1]
    } else if constexpr (MASK == 4) {
        int y = __builtin_amdgcn_update_dpp(xi, xi, 0x1B, 0xF, 0xF, false);  // quad_perm [3,2,1,0]: ^3
        r = __builtin_amdgcn_update_dpp(y, y, 0x141, 0xF, 0xF, false);       // row_half_mirror: ^7
    } else if constexpr (MASK == 8) {
        int y = __builtin_amdgcn_update_dpp(xi, xi, 0x141, 0xF, 0xF, false);  // ^7
        r = __builtin_amdgcn_update_dpp(y, y, 0x140, 0xF, 0xF, false);        // row_mirror: ^15
    } else {
        r = __builtin_amdgcn_ds_bpermute((((int)threadIdx.x & 63) ^ MASK) << 2, xi);
    }
    return __int_as_float(r);
}

// One Walsh-Hadamard stage across lanes: lanes with bit MASK clear get a+b, the others a-b where
// a is the value held by the lane with the bit clear.
template <int MASK> __device__ __forceinline__ float wht_lane_stage(float x, int lane) {
    const float p = lane_xor<MASK>(x);
    return (lane & MASK) ? (p - x) : (x + p);
}

// In-register Walsh-Hadamard transform of N consecutive coordinates (natural order).
template <int N> __device__ __forceinline__ void wht_inlane(float (&x)[N]) {
#pragma unroll
    for (int h = 1; h < N; h <<= 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if ((i & h) == 0) {
                const float a = x[i], b = x[i | h];
                x[i] = a + b;
                x[i | h] = a - b;
            }
        }
    }
}

}  // namespace polykv
