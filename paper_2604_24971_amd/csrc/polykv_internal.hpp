// Host-side declarations shared by the translation units of libpolykv (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/polykv.h"

// Sign diagonal D of the rotation variant H.D: bit i of w[] set = coordinate i is negated; on = any set.
struct SignBits {
    uint32_t w[8];
    uint32_t on;
};

struct polykv_pool {
    int layers, kv_heads, head_dim, tokens;
    int value_codec;    // POLYKV_VALUES_*
    int key_codec;      // POLYKV_KEYS_*
    size_t kmax_off;    // POLYKV_KEYS_Q8_TENSOR: byte offset in storage of the layers' max|k| (uint32 fp32 bits each)
    int tiles;          // ceil(tokens / 32): tile records per (layer, KV head), the record stride
    size_t tile_bytes;  // bytes of one tile record
    size_t bytes;       // layers * kv_heads * tiles * tile_bytes
    void* storage;      // device, caller-owned
    int length;         // tokens encoded so far (0 = nothing to read yet), <= tokens
    SignBits signs;     // all zero: the plain transform
};

namespace polykv {

void set_error(const char* fmt, ...);

// Everything pool_attend needs after validation; passed by value to the kernels.
struct AttendPlan {
    int D, T, tiles, H;          // pool shape: T tokens encoded so far, in `tiles` tiles
    int vcodec;                  // the pool's value codec, POLYKV_VALUES_*
    int kcodec;                  // the pool's key codec, POLYKV_KEYS_*
    const uint32_t* kmax;        // POLYKV_KEYS_Q8_TENSOR: the layers' max|k| (device), indexed by pool layer
    int tiles_cap;               // tile records per (layer, KV head) in storage (the pool's capacity)
    int layer_begin, layers;     // selected layer range
    int A, nq, q_heads, G, R;    // R = A * nq * G query rows per KV head
    float qscale;                // softmax scale * log2(e): scores are kept in base-2 units
    int kernel;                  // POLYKV_KERNEL_VECTOR / _MATRIX (resolved)
    int nsplit;                  // token-range splits per KV head
    int block_rows;              // matrix-core kernel: query rows per workgroup, 64 or 32
    int has_tails, tail_capacity, tail_causal;
    int io_bf16;                 // 1: Q and the tails are bfloat16, 0: fp16
    int key_fp16;                // 1: scores over the dequantized keys rounded to fp16 (POLYKV_KEY_PRECISION_FP16)
    SignBits signs;              // the pool's sign diagonal
    // workspace carving (byte offsets from the 256-aligned workspace base)
    size_t off_ml, off_o, off_tail_ml, off_tail_o, total;
};

struct TailPtrs {
    const void* K[POLYKV_MAX_TAIL_AGENTS];
    const void* V[POLYKV_MAX_TAIL_AGENTS];
    int len[POLYKV_MAX_TAIL_AGENTS];
};

// Encodes dense tokens [0, count) of K, V ([layers, kv_heads, count, head_dim]) as pool tokens
// [begin, begin + count); tokens of the first touched tile that lie before `begin` are kept.
hipError_t launch_encode(const polykv_pool* p, const void* K, const void* V, int in_dtype, int begin, int count,
                         hipStream_t s);
hipError_t launch_decode(const polykv_pool* p, void* K_out, void* V_out, int dtype, int layer_begin, int layer_end,
                         hipStream_t s);
hipError_t launch_export(const polykv_pool* p, void* kc, void* ks, void* vp, void* vs, hipStream_t s);
hipError_t launch_attend(const polykv_pool* p, const AttendPlan& plan, const void* Q, void* out,
                         const TailPtrs* tails, void* workspace, hipStream_t s);

// Events armed by polykv_time_next_kernel() for the calling thread; taking them disarms the hook.
struct KernelEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
KernelEvents take_kernel_events();

// Launch of a call's main kernel: through hipExtLaunchKernelGGL when the caller asked for the kernel's own
// start / stop timestamps, as a plain launch otherwise.
template <typename... Params, typename... Args>
inline void launch_main_kernel(void (*kern)(Params...), dim3 grid, dim3 block, size_t shmem, hipStream_t s,
                               Args... args) {
    const KernelEvents ev = take_kernel_events();
    if (ev.start != nullptr || ev.stop != nullptr)
        hipExtLaunchKernelGGL(kern, grid, block, (uint32_t)shmem, s, ev.start, ev.stop, 0, static_cast<Params>(args)...);
    else
        kern<<<grid, block, shmem, s>>>(static_cast<Params>(args)...);
}

// True if the matrix-core attention kernel supports this shape.
bool matrix_kernel_supports(int head_dim, int rows_per_kv_head, int value_codec);
// Query rows one workgroup of the matrix-core kernel covers.
int matrix_kernel_block_rows(int head_dim, int value_codec);
// True if the matrix-core kernel writes the final output itself (no merge kernel needed).
bool matrix_kernel_direct(const AttendPlan& plan);
hipError_t launch_attend_matrix(const polykv_pool* pool, const AttendPlan& plan, const void* Q, float* ws_ml,
                                float* ws_o, float* out, hipStream_t s);

// Query row r of KV head kvh in selected layer ls -> index (in vectors of head_dim) into Q / out.
// Rows of a KV head are ordered (agent, query, head-in-group): r = (a * nq + i) * G + g.
__host__ __device__ inline size_t q_row_index(const AttendPlan& p, int ls, int kvh, int r) {
    const int g = r % p.G, ai = r / p.G;
    return ((size_t)ls * p.A * p.nq + ai) * p.q_heads + kvh * p.G + g;
}

}  // namespace polykv
