/*
 * polykv.h -- C ABI of the PolyKV shared-pool hot path for AMD MI355X (gfx950).
 *
 * One pool holds the KV cache of a shared context, written once and read by any number of
 * agents (paper: section "PolyKV Architecture", the SharedKVPool abstraction).  Keys are stored
 * as q8_0 (int8 codes, one fp16 scale = absmax/127 per 32 consecutive head_dim elements; section
 * "Compression Scheme", key quantization), values as a normalized Walsh-Hadamard rotation
 * followed by 3-bit Lloyd-Max codes for N(0,1), bit-packed (section "Compression Scheme", value
 * quantization; codebook of section "TurboQuant").
 *
 * Conventions for every call
 *   - "dev" pointers are device (HBM) addresses on the current HIP device; everything else is
 *     host memory.  The library allocates no device memory and never synchronizes: work is
 *     enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - All device buffers are owned by the caller and must stay valid until the enqueued work
 *     has finished.  A pool handle owns only a small host descriptor.
 *   - Return value: POLYKV_OK (0) or a negative polykv_status; polykv_last_error() then returns
 *     a thread-local description.  No call aborts or throws.  NaN/Inf inputs are not checked and
 *     give unspecified values (never out-of-bounds accesses).
 *   - Tensor layouts are row-major.  K/V caches: [layers, kv_heads, tokens, head_dim]
 *     (the paper's [batch=1, heads, seq_len, head_dim] per layer, stacked over layers).
 */
#ifndef POLYKV_H
#define POLYKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct polykv_pool polykv_pool;

typedef enum {
    POLYKV_OK = 0,
    POLYKV_EINVAL = -1,  /* NULL pointer, bad enum value                                   */
    POLYKV_ESHAPE = -2,  /* unsupported or inconsistent dimensions                         */
    POLYKV_ESTATE = -3,  /* storage not bound, or read before the pool was encoded         */
    POLYKV_ENOMEM = -4,  /* caller-provided storage / workspace too small                  */
    POLYKV_EHIP = -5     /* a HIP launch failed                                            */
} polykv_status;

/* Element types of dense tensors.  POLYKV_BF16 is bfloat16, the type of the paper's Llama-3-8B cache (section
 * "Experimental Setup"); everything is computed exactly as for fp16 after the (exact) widening to fp32. */
enum { POLYKV_F16 = 0, POLYKV_F32 = 1, POLYKV_BF16 = 2 };
enum { POLYKV_MAX_TAIL_AGENTS = 64 };

/* Attention kernel selection.  AUTO picks by shape: the matrix-core kernel when it supports the
 * shape, else the vector kernel.  The explicit values exist for tests and profiling. */
enum { POLYKV_KERNEL_AUTO = 0, POLYKV_KERNEL_VECTOR = 1, POLYKV_KERNEL_MATRIX = 2 };
enum { POLYKV_KEY_PRECISION_EXACT = 0, POLYKV_KEY_PRECISION_FP16 = 1 };

/* Value codecs.
 *   POLYKV_VALUES_TQ3         the paper's: rotate, 3-bit Lloyd-Max codes for N(0,1) applied to the rotated
 *                             coordinates as they are (section "Compression Scheme", value quantization).
 *   POLYKV_VALUES_TQ3_SCALED  a variant: each vector also stores g = fp16(min(|v|_2 / sqrt(head_dim), 128)) and
 *                             its rotated coordinates are quantized in units of g (code = number of
 *                             thresholds t_k with t_k * g strictly below v_rot; all codes 3 if g = 0), so the
 *                             codebook sees the unit-variance coordinates that the analysis cited in section
 *                             "TurboQuant" assumes; V = g * H_d c[code] / sqrt(d).  Two more bytes per vector.
 *   POLYKV_VALUES_INT8        uniform int8 without rotation, the ablation proposed in sections "Discussion" and
 *                             "Future Work": the key formula on each value vector with one scale per vector,
 *                             s = fp16(min(max|v| / 127, 128)), code = clip(rint(v / s), -128, 127) formed with the
 *                             stored s, V = code * s.  head_dim + 2 bytes per vector.
 *   POLYKV_VALUES_TQ2, _TQ4   the paper's codec at 2 and 4 bits per coordinate (section "TurboQuant" states the
 *   (and their _SCALED forms) quantizer for b bits; the paper uses b = 3): the Lloyd-Max codebook of N(0,1) with
 *                             4 and 16 levels, code = number of thresholds strictly below v_rot, head_dim/4 and
 *                             head_dim/2 bytes per vector. */
enum {
    POLYKV_VALUES_TQ3 = 0,
    POLYKV_VALUES_TQ3_SCALED = 1,
    POLYKV_VALUES_INT8 = 2,
    POLYKV_VALUES_TQ2 = 3,
    POLYKV_VALUES_TQ2_SCALED = 4,
    POLYKV_VALUES_TQ4 = 5,
    POLYKV_VALUES_TQ4_SCALED = 6
};

/* Key codecs.
 *   POLYKV_KEYS_Q8_BLOCK32  q8_0: one fp16 scale per block of 32 consecutive head_dim elements (the default).
 *   POLYKV_KEYS_Q8_TENSOR   the key formula as section "Compression Scheme" prints it: ONE scale per layer tensor
 *                           [kv_heads, tokens, head_dim], s = fp16(max|K| / 127).  No per-block scales are stored
 *                           (head_dim + 3*head_dim/8 bytes per token and KV head, the paper's 16/5.5 ratio), and
 *                           the attention kernel needs no per-block dequantization.  The maximum must be known
 *                           before any code is formed: such a pool is filled by one pool_encode (two passes over
 *                           K); pool_append returns POLYKV_ESTATE. */
enum { POLYKV_KEYS_Q8_BLOCK32 = 0, POLYKV_KEYS_Q8_TENSOR = 1 };

/* Host descriptor for a pool of `layers` x `kv_heads` x `tokens` vectors of `head_dim` elements.
 * head_dim must be 64, 128 or 256; all other dimensions >= 1, layers * kv_heads <= 65535, and the packed
 * records of one KV head (pool_bytes / (layers * kv_heads)) at most 4 GiB, about 23 million tokens at
 * head_dim 128; POLYKV_ESHAPE otherwise.  (SharedKVPool, section "PolyKV Architecture".)  *out receives the
 * handle; release it with pool_destroy. */
int pool_create(int layers, int kv_heads, int head_dim, int tokens, polykv_pool** out);
/* The same with a choice of value codec (POLYKV_VALUES_*); pool_create uses POLYKV_VALUES_TQ3. */
int pool_create_codec(int layers, int kv_heads, int head_dim, int tokens, int value_codec, polykv_pool** out);
/* ... and of key codec (POLYKV_KEYS_*). */
int pool_create_codecs(int layers, int kv_heads, int head_dim, int tokens, int key_codec, int value_codec,
                       polykv_pool** out);
/* Rotation variant: v_rot = H_d D v / sqrt(d) with D a fixed diagonal of pseudorandom signs (the randomized
 * Hadamard rotation of the rotation-based quantizers discussed in section "Related Work"), which keeps
 * structured vectors from piling onto a few rotated coordinates; dequantization applies D H_d / sqrt(d).
 * Coordinate i is negated iff output i of the SplitMix64 generator started at `seed` is odd; seed 0 (the
 * default) is the paper's plain transform.  Call before any token is encoded (POLYKV_ESTATE otherwise, and for
 * a POLYKV_VALUES_INT8 pool, whose values are not rotated). */
int pool_set_sign_seed(polykv_pool* pool, uint64_t seed);
void pool_destroy(polykv_pool* pool);

/* Bytes of device storage the packed pool needs (tokens are padded to tiles of 32; per token and
 * KV head: head_dim code bytes + head_dim/16 scale bytes + 3*head_dim/8 value-code bytes, the
 * byte counts behind section "Compression Scheme", compression ratio; + 2 bytes with value scales).
 * 0 if pool is NULL. */
size_t pool_bytes(const polykv_pool* pool);

/* Attach caller-owned device storage (256-byte aligned, >= pool_bytes()).  Re-binding is allowed
 * and marks the pool as not yet encoded. */
int pool_bind(polykv_pool* pool, void* dev_storage, size_t bytes);

/* Compress a dense fp16 cache into the bound storage (section "Compression Scheme"):
 *   keys    per 32-element block: s = fp16(max|k| / 127), code = clip(rint(k / s), -128, 127),
 *           ties to even, codes formed with the stored (rounded) s; an all-zero block gets s = 0;
 *   values  v_rot = H_d v / sqrt(d) (natural-order Walsh-Hadamard), code = number of Lloyd-Max
 *           thresholds strictly below v_rot, 3 bits.
 * K_dev, V_dev: fp16 [layers, kv_heads, tokens, head_dim], read-only.  May be called again; it
 * overwrites the pool (the pool is otherwise write-once / read-many). */
int pool_encode(polykv_pool* pool, const void* K_dev, const void* V_dev, void* stream);
/* The same for K_dev, V_dev of type in_dtype, POLYKV_F16 or POLYKV_BF16.  A bfloat16 key block whose
 * max|k| / 127 exceeds the fp16 maximum stores the scale 65504 and saturates. */
int pool_encode_dtype(polykv_pool* pool, const void* K_dev, const void* V_dev, int in_dtype, void* stream);

/* Incremental fill (an extension: the paper's pool is written once, section "PolyKV Architecture"):
 * compress `count` further tokens, K_dev, V_dev fp16 [layers, kv_heads, count, head_dim], as pool tokens
 * [pool_length(), pool_length() + count), with the same arithmetic as pool_encode -- the pool then holds
 * exactly what one pool_encode of the concatenated tensors would have produced.  Starts from an empty
 * pool after pool_bind; pool_encode fills the pool to its capacity (pool_create's `tokens`) in one go.
 * POLYKV_ESHAPE if the tokens do not fit.  Calls that fill and calls that read must be ordered by the
 * caller (same stream, or events). */
int pool_append(polykv_pool* pool, const void* K_dev, const void* V_dev, int count, void* stream);
int pool_append_dtype(polykv_pool* pool, const void* K_dev, const void* V_dev, int count, int in_dtype, void* stream);

/* Tokens encoded so far (0 .. tokens).  pool_decode, pool_export and pool_attend work on these;
 * their dense tensors have pool_length() tokens per (layer, KV head). */
int pool_length(const polykv_pool* pool);

/* Decompress the whole pool to dense tensors (the paper's get_kv_for_layer, section
 * "DynamicCache Injection", for all layers): K = code * s, V = H_d c[code] / sqrt(d).
 * out_dtype: POLYKV_F16, POLYKV_F32 or POLYKV_BF16 (fp32 result rounded once, to nearest even); K_out_dev, V_out_dev: [layers, kv_heads, pool_length(), head_dim].
 * Either output may be NULL to skip it. */
int pool_decode(const polykv_pool* pool, void* K_out_dev, void* V_out_dev, int out_dtype, void* stream);

/* The same for layers [layer_begin, layer_end) only (one layer = the paper's get_kv_for_layer(l));
 * K_out_dev, V_out_dev: [layer_end - layer_begin, kv_heads, pool_length(), head_dim]. */
int pool_decode_layers(const polykv_pool* pool, void* K_out_dev, void* V_out_dev, int out_dtype, int layer_begin,
                       int layer_end, void* stream);

/* Copy the pool out in the canonical format used to compare implementations:
 *   k_codes_dev  int8   [layers, kv_heads, pool_length(), head_dim]
 *   k_scales_dev fp16   [layers, kv_heads, pool_length(), head_dim/32]  ([layers] for POLYKV_KEYS_Q8_TENSOR)
 *   v_packed_dev uint8  [layers, kv_heads, pool_length(), 3*head_dim/8], little-endian bit stream:
 *                code j of a vector occupies stream bits 3j..3j+2, stream bit i is bit (i mod 8)
 *                of byte floor(i/8).
 *                A POLYKV_VALUES_INT8 pool writes int8 [layers, kv_heads, pool_length(), head_dim] here,
 *                the value codes themselves; the 2- and 4-bit codecs the same stream with 2 / 4 bits per code
 *                (head_dim/4 and head_dim/2 bytes per vector).
 * (The in-HBM layout is tiled for the attention kernel and is not part of the ABI.)  Any of the
 * three may be NULL. */
int pool_export(const polykv_pool* pool, void* k_codes_dev, void* k_scales_dev, void* v_packed_dev,
                void* stream);

/* The per-vector value scales of a pool whose value codec stores them (the _SCALED codecs and POLYKV_VALUES_INT8):
 * v_scales_dev fp16 [layers, kv_heads, pool_length()].  POLYKV_ESTATE for the other codecs. */
int pool_export_value_scales(const polykv_pool* pool, void* v_scales_dev, void* stream);

/* Decode attention of N agents directly over the packed pool (replaces the paper's per-agent
 * decompress-and-inject read path of section "DynamicCache Injection"; the result equals softmax
 * attention over pool_decode()'s tensors).  Every query row attends all pool tokens, then, if
 * tails are given, the agent's own uncompressed continuation (section "Introduction": each agent
 * generates independently after the shared prefix).  No mask, no positional transform: Q and K
 * are taken as already position-encoded. */
typedef struct {
    int agents;       /* N >= 1                                                             */
    int q_per_agent;  /* decode queries per agent per head (1 = plain decode)               */
    int q_heads;      /* multiple of kv_heads; q head h reads kv head h / (q_heads/kv_heads) */
    int layer_begin;  /* attend layers [layer_begin, layer_end)                             */
    int layer_end;
    float scale;      /* softmax scale; 0 means 1/sqrt(head_dim)                            */
    /* Optional private tails: host arrays of `agents` device pointers / lengths (NULL = none).
     * tail_K[a], tail_V[a]: fp16 [layers, kv_heads, tail_capacity, head_dim] (all pool layers),
     * of which the first tail_len[a] tokens are attended by agent a's queries.  The arrays are
     * read during the call only.  agents <= POLYKV_MAX_TAIL_AGENTS when tails are used. */
    const void* const* tail_K;
    const void* const* tail_V;
    const int* tail_len;
    int tail_capacity;
    /* Nonzero: the agent's q_per_agent queries sit at its last q_per_agent tail positions (a multi-token
     * decode step): query i attends the pool and the first tail_len[a] - (q_per_agent - 1 - i) tail tokens
     * (none if that is <= 0) -- ordinary causal attention among the new tokens.  Zero: every query attends
     * the whole tail. */
    int tail_causal;
    int kernel;       /* POLYKV_KERNEL_*                                                    */
    int splits;       /* token-range splits per KV head; 0 = choose automatically           */
    void* workspace_dev;     /* scratch for split partials, 256-byte aligned                */
    size_t workspace_bytes;  /* >= pool_attend_workspace()                                  */
    int io_dtype;     /* type of Q and of the tails: POLYKV_F16 (0) or POLYKV_BF16.  bfloat16 queries are
                         converted to fp16 operands in the matrix-core kernel: |q| must stay below 65504 */
    int key_precision; /* POLYKV_KEY_PRECISION_EXACT (0, the default): scores over K = code * s exactly.
                          POLYKV_KEY_PRECISION_FP16: scores over fp16(code * s), the dequantized key rounded once to
                          the 16-bit type of the dense cache -- what the paper's read path attends over after its cast
                          to the model dtype (section "DynamicCache Injection"); saves a third of the score products.
                          Honoured by the matrix-core kernel for pools with q8_0 block keys and the paper's value
                          codec at head_dim 64 / 128; every other case is computed with exact keys. */
} polykv_attend_params;

/* Scratch bytes pool_attend needs for these parameters (workspace fields are ignored). */
size_t pool_attend_workspace(const polykv_pool* pool, const polykv_attend_params* params);

/* Q_dev: fp16 (or bfloat16, see io_dtype) [layer_end-layer_begin, agents, q_per_agent, q_heads, head_dim];
 * out_dev: fp32, same shape.  Reads the pool only; concurrent calls on different streams are
 * safe if they use different workspaces.  POLYKV_ESHAPE for shapes beyond the launch limits: more than 2^20 query
 * rows (agents * q_per_agent * q_heads / kv_heads) per KV head; more than 262,140 with POLYKV_KERNEL_VECTOR; with
 * tails, q_per_agent * q_heads / kv_heads above 262,140.  POLYKV_EINVAL for a negative or non-finite scale. */
int pool_attend(const polykv_pool* pool, const void* Q_dev, void* out_dev,
                const polykv_attend_params* params, void* stream);

/* pool_attend for callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: the same operation, kernels and results, but the split partials live
 * in a buffer of POLYKV_STATIC_WORKSPACE_BYTES that is part of the library's code object (every GPU the library
 * runs on holds one until the process ends); params->workspace_dev / workspace_bytes are ignored.  The call
 * allocates nothing on the host or the device.  POLYKV_ENOMEM, with the sizes in polykv_last_error(), if the
 * call needs more scratch than that (pool_attend_workspace() says how much).  All calls on one GPU share that
 * GPU's buffer: two calls that may run at the same time on one GPU (different streams) race -- order them, or
 * use pool_attend with workspaces of the caller's.  Nothing in the buffer has to be cleared between calls:
 * every call writes all the partials it later reads. */
#define POLYKV_STATIC_WORKSPACE_BYTES (32u << 20)
int pool_attend_static(const polykv_pool* pool, const void* Q_dev, void* out_dev,
                       const polykv_attend_params* params, void* stream);

/* The value codebook the library uses: 8 ascending centroids and the 7 decision thresholds
 * (midpoints), as fp32 (section "TurboQuant", Lloyd-Max quantization).  Host call. */
void polykv_codebook(float* centroids8, float* thresholds7);
/* The same for bits = 2, 3 or 4: 2^bits ascending centroids and 2^bits - 1 thresholds.  POLYKV_EINVAL otherwise. */
int polykv_codebook_bits(int bits, float* centroids, float* thresholds);

/* Measurement hook (for benchmarks and profilers; not an operation of the method).  Arms the calling
 * thread: the NEXT pool_encode, pool_decode or pool_attend call of this thread that launches has the HIP runtime
 * record `start_event` when its main kernel (the encode kernel, the decode kernel, the pool attention
 * kernel -- not the small tail / merge kernels) begins to execute and `stop_event` when it has finished,
 * on the stream the kernel is launched on; the hook then disarms itself.  Both are hipEvent_t handles
 * created (with timing enabled) and owned by the caller; either may be NULL.  hipEventElapsedTime(start,
 * stop), after the stream has been synchronized, is then the kernel's own duration, without the launch
 * gaps that events recorded around the call include.  Host pointers only; never fails (POLYKV_OK). */
int polykv_time_next_kernel(void* start_event, void* stop_event);

/* Description of the last error on this thread ("" if none). */
const char* polykv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* POLYKV_H */
