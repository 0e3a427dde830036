// Encode / decode / export kernels of the packed pool (gfx950).
//
// One workgroup of 256 threads handles one tile (32 tokens) of one KV head.  Thread (t, c), t =
// tid/8, c = tid%8, owns the D/8 consecutive head_dim elements c*D/8 .. of token t, so a dense fp16
// row is read (or written) by 8 neighbouring lanes with 16- or 32-byte accesses, and the Walsh-
// Hadamard butterflies need log2(D/8) in-register stages plus three DPP stages across those 8 lanes.
// The tile record is assembled in LDS and streamed out with 16-byte coalesced stores.
#include <hip/hip_fp16.h>

#include "polykv_internal.hpp"
#include "polykv_layout.hpp"

namespace polykv {

template <int N> struct HalfVec { __half v[N]; };

template <int N>
__device__ __forceinline__ void load_halfs(const __half* p, bool valid, float (&x)[N]) {
    static_assert(N % 8 == 0, "");
#pragma unroll
    for (int i = 0; i < N / 8; ++i) {
        uint4 raw = valid ? reinterpret_cast<const uint4*>(p)[i] : make_uint4(0, 0, 0, 0);
        const __half2* h2 = reinterpret_cast<const __half2*>(&raw);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float2 f = __half22float2(h2[k]);
            x[i * 8 + 2 * k] = f.x;
            x[i * 8 + 2 * k + 1] = f.y;
        }
    }
}

// Walsh-Hadamard transform of a D-vector spread over 8 lanes (lane c holds elements c*N..c*N+N-1).
template <int N> __device__ __forceinline__ void wht_8lanes(float (&x)[N], int lane) {
    wht_inlane<N>(x);
#pragma unroll
    for (int i = 0; i < N; ++i) {
        x[i] = wht_lane_stage<1>(x[i], lane);
        x[i] = wht_lane_stage<2>(x[i], lane);
        x[i] = wht_lane_stage<4>(x[i], lane);
    }
}

template <int D> __device__ __forceinline__ constexpr float inv_sqrt_d() {
    return D == 64 ? 0.125f : 0.08838834764831845f;
}

// ------------------------------------------------------------------------------------ encode ---
// Key quantization and value quantization of section "Compression Scheme", fused in one pass.
template <int D>
__global__ __launch_bounds__(256) void encode_kernel(const __half* __restrict__ K,
                                                     const __half* __restrict__ V,
                                                     uint8_t* __restrict__ pool, int T, int tiles) {
    using LY = Layout<D>;
    constexpr int EPT = D / 8;
    __shared__ __align__(16) uint8_t img[LY::tile_bytes];
    constexpr int VS = D + 4;  // row stride of the code staging area: +4 bytes rotates the LDS bank per token
    __shared__ __align__(16) uint8_t vstage[kTile * VS];

    const int tile = blockIdx.x, unit = blockIdx.y;
    const int tid = threadIdx.x, t = tid >> 3, c = tid & 7;
    const int tok = tile * kTile + t;
    const bool valid = tok < T;
    const size_t row = ((size_t)unit * T + (valid ? tok : 0)) * D + c * EPT;
    const int e0 = c * EPT, j = e0 >> 5, g8 = (e0 >> 3) & 3;

    // ---- keys: block absmax -> fp16 scale -> codes with the stored scale
    {
        float k[EPT];
        load_halfs<EPT>(K + row, valid, k);
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < EPT; ++i) amax = fmaxf(amax, fabsf(k[i]));
        amax = fmaxf(amax, lane_xor<1>(amax));
        if (EPT == 8) amax = fmaxf(amax, lane_xor<2>(amax));
        const __half s16 = __float2half_rn(__fdiv_rn(amax, 127.0f));
        const float sf = __half2float(s16);
        const float inv = sf > 0.0f ? __fdiv_rn(1.0f, sf) : 0.0f;
        uint32_t packed[EPT / 4];
#pragma unroll
        for (int i = 0; i < EPT / 4; ++i) {
            uint32_t w = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                float q = rintf(__fmul_rn(k[i * 4 + b], inv));
                q = fminf(fmaxf(q, -128.0f), 127.0f);
                w |= (uint32_t)((int)q + 128) << (8 * b);
            }
            packed[i] = w;
        }
#pragma unroll
        for (int rr = 0; rr < EPT / 8; ++rr) {
            uint32_t* dst = reinterpret_cast<uint32_t*>(img + LY::kcodes_off + kcode_run_offset(t, j, g8 + rr));
            dst[0] = packed[2 * rr];
            dst[1] = packed[2 * rr + 1];
        }
        if ((e0 & 31) == 0)
            reinterpret_cast<__half*>(img + LY::kscales_off)[t * LY::NB + j] = s16;
    }

    // ---- values: rotate, nearest centroid, stage codes as bytes [t][dv]
    {
        float x[EPT];
        load_halfs<EPT>(V + row, valid, x);
        wht_8lanes<EPT>(x, tid);
        uint32_t* dst = reinterpret_cast<uint32_t*>(vstage + t * VS + e0);
#pragma unroll
        for (int i = 0; i < EPT / 4; ++i) {
            uint32_t w = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b)
                w |= (uint32_t)quantize3(__fmul_rn(x[i * 4 + b], inv_sqrt_d<D>())) << (8 * b);
            dst[i] = w;
        }
    }
    __syncthreads();

    // ---- bit-pack the value codes into the tile record
    for (int idx = tid; idx < LY::NT * 192; idx += 256) {
        const int q = idx / 192, rem = idx - q * 192;
        const int lane = rem / 3, w = rem - lane * 3;
        const int grp = lane >> 4, m = lane & 15;
        const int dv = 16 * (4 * q + w) + m;
        const int dv3 = 16 * (4 * q + 3) + m;  // group 4q+3 lives in the spare bits
        uint32_t word = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int tk = vcode_token(grp, e);
            word |= (uint32_t)vstage[tk * VS + dv] << (8 * (e & 3) + 3 * (e >> 2));
            const uint32_t c3 = vstage[tk * VS + dv3];
            if (w == 0 && e < 4) word |= (c3 & 3) << (8 * e + 6);
            if (w == 2 && e >= 4) word |= (c3 & 3) << (8 * (e - 4) + 6);
            if (w == 1) word |= (c3 >> 2) << (e < 4 ? 8 * e + 6 : 8 * (e - 4) + 7);
        }
        reinterpret_cast<uint32_t*>(img + LY::vcodes_off)[idx] = word;
    }
    __syncthreads();

    uint4* out = reinterpret_cast<uint4*>(pool + ((size_t)unit * tiles + tile) * LY::tile_bytes);
    const uint4* src = reinterpret_cast<const uint4*>(img);
    for (int i = tid; i < LY::tile_bytes / 16; i += 256) out[i] = src[i];
}

// ------------------------------------------------------------------------------------ decode ---
template <typename OutT> __device__ __forceinline__ OutT to_out(float x);
template <> __device__ __forceinline__ float to_out<float>(float x) { return x; }
template <> __device__ __forceinline__ __half to_out<__half>(float x) { return __float2half_rn(x); }

template <int D>
__device__ __forceinline__ void stage_tile(uint8_t* img, const uint8_t* pool, int unit, int tiles,
                                           int tile, int tid) {
    using LY = Layout<D>;
    const uint4* src = reinterpret_cast<const uint4*>(pool + ((size_t)unit * tiles + tile) * LY::tile_bytes);
    uint4* dst = reinterpret_cast<uint4*>(img);
    for (int i = tid; i < LY::tile_bytes / 16; i += 256) dst[i] = src[i];
    __syncthreads();
}

// K = code * s and V = H c[code] / sqrt(d)  (sections "Compression Scheme" and "TurboQuant",
// dequantization; the inverse of the normalized rotation is the same normalized transform).
template <int D, typename OutT>
__global__ __launch_bounds__(256) void decode_kernel(const uint8_t* __restrict__ pool,
                                                     OutT* __restrict__ K_out, OutT* __restrict__ V_out,
                                                     int T, int tiles) {
    using LY = Layout<D>;
    constexpr int EPT = D / 8;
    __shared__ __align__(16) uint8_t img[LY::tile_bytes];
    const int tile = blockIdx.x, unit = blockIdx.y;
    const int tid = threadIdx.x, t = tid >> 3, c = tid & 7;
    stage_tile<D>(img, pool, unit, tiles, tile, tid);
    const int tok = tile * kTile + t;
    const bool valid = tok < T;
    const size_t row = ((size_t)unit * T + (valid ? tok : 0)) * D + c * EPT;
    const int e0 = c * EPT, j = e0 >> 5, g8 = (e0 >> 3) & 3;

    if (K_out != nullptr) {
        const float s = __half2float(reinterpret_cast<const __half*>(img + LY::kscales_off)[t * LY::NB + j]);
        if (valid) {
#pragma unroll
            for (int i = 0; i < EPT; ++i) {
                const uint8_t* codes = img + LY::kcodes_off + kcode_run_offset(t, j, g8 + (i >> 3));
                K_out[row + i] = to_out<OutT>((float)((int)codes[i & 7] - 128) * s);
            }
        }
    }
    if (V_out != nullptr) {
        const uint32_t* vreg = reinterpret_cast<const uint32_t*>(img + LY::vcodes_off);
        float x[EPT];
#pragma unroll
        for (int i = 0; i < EPT; ++i) x[i] = centroid_of(vcode_extract(vreg, t, e0 + i));
        wht_8lanes<EPT>(x, tid);
        if (valid) {
#pragma unroll
            for (int i = 0; i < EPT; ++i) V_out[row + i] = to_out<OutT>(x[i] * inv_sqrt_d<D>());
        }
    }
}

// ------------------------------------------------------------------------------------ export ---
template <int D>
__global__ __launch_bounds__(256) void export_kernel(const uint8_t* __restrict__ pool,
                                                     int8_t* __restrict__ k_codes,
                                                     __half* __restrict__ k_scales,
                                                     uint8_t* __restrict__ v_packed, int T, int tiles) {
    using LY = Layout<D>;
    constexpr int EPT = D / 8;
    __shared__ __align__(16) uint8_t img[LY::tile_bytes];
    const int tile = blockIdx.x, unit = blockIdx.y;
    const int tid = threadIdx.x, t = tid >> 3, c = tid & 7;
    stage_tile<D>(img, pool, unit, tiles, tile, tid);
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
    if (k_scales != nullptr && c < LY::NB)
        k_scales[vec * LY::NB + c] = reinterpret_cast<const __half*>(img + LY::kscales_off)[t * LY::NB + c];
    if (v_packed != nullptr) {
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

// ---------------------------------------------------------------------------------- launchers ---
hipError_t launch_encode(const polykv_pool* p, const void* K, const void* V, hipStream_t s) {
    dim3 grid(p->tiles, p->layers * p->kv_heads);
    if (p->head_dim == 128)
        encode_kernel<128><<<grid, 256, 0, s>>>((const __half*)K, (const __half*)V, (uint8_t*)p->storage,
                                                p->tokens, p->tiles);
    else
        encode_kernel<64><<<grid, 256, 0, s>>>((const __half*)K, (const __half*)V, (uint8_t*)p->storage,
                                               p->tokens, p->tiles);
    return hipGetLastError();
}

hipError_t launch_decode(const polykv_pool* p, void* K_out, void* V_out, int dtype, hipStream_t s) {
    dim3 grid(p->tiles, p->layers * p->kv_heads);
    const uint8_t* pool = (const uint8_t*)p->storage;
    if (p->head_dim == 128) {
        if (dtype == POLYKV_F32)
            decode_kernel<128, float><<<grid, 256, 0, s>>>(pool, (float*)K_out, (float*)V_out, p->tokens, p->tiles);
        else
            decode_kernel<128, __half><<<grid, 256, 0, s>>>(pool, (__half*)K_out, (__half*)V_out, p->tokens, p->tiles);
    } else {
        if (dtype == POLYKV_F32)
            decode_kernel<64, float><<<grid, 256, 0, s>>>(pool, (float*)K_out, (float*)V_out, p->tokens, p->tiles);
        else
            decode_kernel<64, __half><<<grid, 256, 0, s>>>(pool, (__half*)K_out, (__half*)V_out, p->tokens, p->tiles);
    }
    return hipGetLastError();
}

hipError_t launch_export(const polykv_pool* p, void* kc, void* ks, void* vp, hipStream_t s) {
    dim3 grid(p->tiles, p->layers * p->kv_heads);
    const uint8_t* pool = (const uint8_t*)p->storage;
    if (p->head_dim == 128)
        export_kernel<128><<<grid, 256, 0, s>>>(pool, (int8_t*)kc, (__half*)ks, (uint8_t*)vp, p->tokens, p->tiles);
    else
        export_kernel<64><<<grid, 256, 0, s>>>(pool, (int8_t*)kc, (__half*)ks, (uint8_t*)vp, p->tokens, p->tiles);
    return hipGetLastError();
}

}  // namespace polykv
