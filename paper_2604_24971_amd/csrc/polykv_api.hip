// C ABI of libpolykv: argument validation, planning, and dispatch to the kernel launchers.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "polykv_internal.hpp"
#include "polykv_layout.hpp"

namespace polykv {

static thread_local char g_err[256] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

static thread_local KernelEvents g_kernel_events;

KernelEvents take_kernel_events() {
    const KernelEvents ev = g_kernel_events;
    g_kernel_events = KernelEvents{};
    return ev;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Bytes of one tile record for the given head_dim and codecs.
template <int D> static int tile_bytes_of(int vc, int kc) {
    const int t[2][kNumValueCodecs] = {
        {Layout<D, 0, 0>::tile_bytes, Layout<D, 1, 0>::tile_bytes, Layout<D, 2, 0>::tile_bytes, Layout<D, 3, 0>::tile_bytes,
         Layout<D, 4, 0>::tile_bytes, Layout<D, 5, 0>::tile_bytes, Layout<D, 6, 0>::tile_bytes},
        {Layout<D, 0, 1>::tile_bytes, Layout<D, 1, 1>::tile_bytes, Layout<D, 2, 1>::tile_bytes, Layout<D, 3, 1>::tile_bytes,
         Layout<D, 4, 1>::tile_bytes, Layout<D, 5, 1>::tile_bytes, Layout<D, 6, 1>::tile_bytes}};
    return t[kc][vc];
}

// Resolve every choice pool_attend makes from the pool shape and the caller's parameters, so that
// pool_attend_workspace() and pool_attend() agree by construction.
static int make_plan(const polykv_pool* pool, const polykv_attend_params* prm, AttendPlan* plan) {
    if (pool == nullptr || prm == nullptr) {
        set_error("pool_attend: NULL pool or params");
        return POLYKV_EINVAL;
    }
    if (prm->agents < 1 || prm->q_per_agent < 1 || prm->q_heads < 1 || prm->q_heads % pool->kv_heads != 0) {
        set_error("pool_attend: agents=%d q_per_agent=%d q_heads=%d must be >= 1 and q_heads a multiple of kv_heads=%d",
                  prm->agents, prm->q_per_agent, prm->q_heads, pool->kv_heads);
        return POLYKV_ESHAPE;
    }
    if (prm->layer_begin < 0 || prm->layer_end > pool->layers || prm->layer_begin >= prm->layer_end) {
        set_error("pool_attend: layer range [%d,%d) outside [0,%d)", prm->layer_begin, prm->layer_end, pool->layers);
        return POLYKV_ESHAPE;
    }
    if (prm->kernel < POLYKV_KERNEL_AUTO || prm->kernel > POLYKV_KERNEL_MATRIX || prm->splits < 0) {
        set_error("pool_attend: bad kernel selector %d or splits %d", prm->kernel, prm->splits);
        return POLYKV_EINVAL;
    }
    const bool tails = prm->tail_len != nullptr;
    if (tails) {
        if (prm->tail_K == nullptr || prm->tail_V == nullptr) {
            set_error("pool_attend: tail_len given without tail_K/tail_V");
            return POLYKV_EINVAL;
        }
        if (prm->agents > POLYKV_MAX_TAIL_AGENTS) {
            set_error("pool_attend: tails support at most %d agents", POLYKV_MAX_TAIL_AGENTS);
            return POLYKV_ESHAPE;
        }
        for (int a = 0; a < prm->agents; ++a) {
            if (prm->tail_len[a] < 0 || prm->tail_len[a] > prm->tail_capacity) {
                set_error("pool_attend: tail_len[%d]=%d outside [0, tail_capacity=%d]", a, prm->tail_len[a], prm->tail_capacity);
                return POLYKV_ESHAPE;
            }
            if (prm->tail_len[a] > 0 && (prm->tail_K[a] == nullptr || prm->tail_V[a] == nullptr)) {
                set_error("pool_attend: agent %d has tail_len > 0 but a NULL tail pointer", a);
                return POLYKV_EINVAL;
            }
        }
    }
    AttendPlan& p = *plan;
    memset(&p, 0, sizeof(p));
    p.D = pool->head_dim;
    p.vcodec = pool->value_codec;
    p.kcodec = pool->key_codec;
    p.kmax = pool->key_codec == POLYKV_KEYS_Q8_TENSOR
                 ? reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(pool->storage) + pool->kmax_off)
                 : nullptr;
    p.T = pool->length;
    p.tiles = tiles_of(pool->length);
    p.tiles_cap = pool->tiles;
    p.H = pool->kv_heads;
    p.layer_begin = prm->layer_begin;
    p.layers = prm->layer_end - prm->layer_begin;
    p.A = prm->agents;
    p.nq = prm->q_per_agent;
    p.q_heads = prm->q_heads;
    p.G = prm->q_heads / pool->kv_heads;
    const long rows = (long)p.A * p.nq * p.G;
    if (rows > (1 << 20)) {
        set_error("pool_attend: %ld query rows per KV head is more than supported", rows);
        return POLYKV_ESHAPE;
    }
    p.R = (int)rows;
    if (!(prm->scale >= 0.0f) || !(prm->scale <= 3.0e38f)) {
        set_error("pool_attend: the softmax scale must be finite and >= 0 (0 = 1/sqrt(head_dim))");
        return POLYKV_EINVAL;
    }
    const float scale = prm->scale != 0.0f ? prm->scale : 1.0f / sqrtf((float)p.D);
    p.qscale = scale * 1.4426950408889634f;
    p.has_tails = tails ? 1 : 0;
    p.tail_capacity = tails ? prm->tail_capacity : 0;
    p.tail_causal = (tails && prm->tail_causal != 0) ? 1 : 0;
    if (prm->io_dtype != POLYKV_F16 && prm->io_dtype != POLYKV_BF16) {
        set_error("pool_attend: io_dtype %d is neither POLYKV_F16 nor POLYKV_BF16", prm->io_dtype);
        return POLYKV_EINVAL;
    }
    p.io_bf16 = prm->io_dtype == POLYKV_BF16 ? 1 : 0;
    if (prm->key_precision != POLYKV_KEY_PRECISION_EXACT && prm->key_precision != POLYKV_KEY_PRECISION_FP16) {
        set_error("pool_attend: key_precision %d is not a POLYKV_KEY_PRECISION_* value", prm->key_precision);
        return POLYKV_EINVAL;
    }
    p.signs = pool->signs;

    const bool mat_ok = matrix_kernel_supports(p.D, p.R, p.vcodec);
    if (prm->kernel == POLYKV_KERNEL_MATRIX && !mat_ok) {
        set_error("pool_attend: the matrix-core kernel does not support head_dim=%d rows=%d with this value codec", p.D, p.R);
        return POLYKV_ESHAPE;
    }
    p.kernel = prm->kernel == POLYKV_KERNEL_AUTO ? (mat_ok ? POLYKV_KERNEL_MATRIX : POLYKV_KERNEL_VECTOR) : prm->kernel;
    // Launch limits: the vector kernel and the tail kernel put their 4-row blocks on grid.z (at most 65,535).
    if (p.kernel == POLYKV_KERNEL_VECTOR && (p.R + 3) / 4 > 65535) {
        set_error("pool_attend: the vector kernel supports at most 262,140 query rows per KV head (got %d)", p.R);
        return POLYKV_ESHAPE;
    }
    if (tails && ((long)p.nq * p.G + 3) / 4 > 65535) {
        set_error("pool_attend: with tails, q_per_agent * (q_heads / kv_heads) = %ld exceeds 262,140", (long)p.nq * p.G);
        return POLYKV_ESHAPE;
    }
    p.key_fp16 = (prm->key_precision == POLYKV_KEY_PRECISION_FP16 && p.kernel == POLYKV_KERNEL_MATRIX &&
                  p.kcodec == POLYKV_KEYS_Q8_BLOCK32 && p.vcodec == POLYKV_VALUES_TQ3 && p.D != 256)
                     ? 1
                     : 0;

    // Token-range splits per KV head.  Work items are waves; aim at ~2 waves per SIMD of the 256 CUs.
    // The count is derived from the pool's capacity, not from its current fill, so that the workspace
    // size of a call does not change while the pool grows (splits beyond the filled part are empty).
    const int units = p.layers * p.H;
    const int cap_tiles = pool->tiles;
    int nsplit;
    if (p.kernel == POLYKV_KERNEL_VECTOR) {
        const int nchunks = (cap_tiles + 1) / 2;
        const long groups = (long)units * ((p.R + 3) / 4);
        long want = prm->splits > 0 ? prm->splits : (2048 + groups - 1) / groups;
        if (want > nchunks) want = nchunks;
        if (want < 1) want = 1;
        nsplit = (int)((want + 3) / 4 * 4);
    } else {
        // One workgroup (4 waves, one per SIMD) per split: fill the 256 CUs once, but keep at least two
        // tiles per wave -- below that the per-workgroup prologue, epilogue and the partials written for
        // the merge kernel cost more than the idle CUs (measured on one-layer calls of the Llama shape:
        // 16 splits of 8 tiles 16.8 us, 32 splits of 4 tiles 19.3 us).
        // Rows per workgroup: 64 where the kernel has such a form, but 32 when 64-row blocks, split as far as
        // the two-tiles-per-wave rule allows, would leave CUs without a workgroup (one-layer calls: 8 KV heads x
        // 16 splits = 128 workgroups of 64 rows, or 256 of 32 rows that each do half the matrix work).
        auto splits_for = [&](int block_rows, long* n_groups) {
            const long groups = (long)units * ((p.R + block_rows - 1) / block_rows);
            long want = (256 + groups - 1) / groups;
            if (want > cap_tiles / 8) want = cap_tiles / 8;
            if (prm->splits > 0) want = prm->splits;
            if (want > (cap_tiles + 3) / 4) want = (cap_tiles + 3) / 4;
            if (want < 1) want = 1;
            *n_groups = groups;
            return want;
        };
        int block_rows = matrix_kernel_block_rows(p.D, p.vcodec);
        long groups = 0;
        long want = splits_for(block_rows, &groups);
        if (block_rows == 64 && p.R > 32 && groups * want < 256) {
            long g32 = 0;
            const long w32 = splits_for(32, &g32);
            if (g32 * w32 > groups * want) block_rows = 32, want = w32;
        }
        p.block_rows = block_rows;
        nsplit = (int)want;
    }
    p.nsplit = nsplit;

    size_t off = 0;
    p.off_ml = off;
    off = align_up(off + (size_t)units * nsplit * p.R * 2 * sizeof(float), 256);
    p.off_o = off;
    off = align_up(off + (size_t)units * nsplit * p.R * p.D * sizeof(float), 256);
    p.off_tail_ml = off;
    if (tails) off = align_up(off + (size_t)units * p.R * 2 * sizeof(float), 256);
    p.off_tail_o = off;
    if (tails) off = align_up(off + (size_t)units * p.R * p.D * sizeof(float), 256);
    p.total = off;
    return POLYKV_OK;
}

}  // namespace polykv

using namespace polykv;

extern "C" {

int pool_create(int layers, int kv_heads, int head_dim, int tokens, polykv_pool** out) {
    return pool_create_codec(layers, kv_heads, head_dim, tokens, POLYKV_VALUES_TQ3, out);
}

int pool_create_codec(int layers, int kv_heads, int head_dim, int tokens, int value_codec, polykv_pool** out) {
    return pool_create_codecs(layers, kv_heads, head_dim, tokens, POLYKV_KEYS_Q8_BLOCK32, value_codec, out);
}

int pool_create_codecs(int layers, int kv_heads, int head_dim, int tokens, int key_codec, int value_codec,
                       polykv_pool** out) {
    if (out == nullptr) {
        set_error("pool_create: out is NULL");
        return POLYKV_EINVAL;
    }
    *out = nullptr;
    if (value_codec < POLYKV_VALUES_TQ3 || value_codec > POLYKV_VALUES_TQ4_SCALED) {
        set_error("pool_create: unknown value codec %d", value_codec);
        return POLYKV_EINVAL;
    }
    if (key_codec != POLYKV_KEYS_Q8_BLOCK32 && key_codec != POLYKV_KEYS_Q8_TENSOR) {
        set_error("pool_create: unknown key codec %d", key_codec);
        return POLYKV_EINVAL;
    }
    if (head_dim != 64 && head_dim != 128 && head_dim != 256) {
        set_error("pool_create: head_dim=%d not supported (64, 128 or 256)", head_dim);
        return POLYKV_ESHAPE;
    }
    if (layers < 1 || kv_heads < 1 || tokens < 1 || (long)layers * kv_heads > 65535) {
        set_error("pool_create: layers=%d kv_heads=%d tokens=%d must be >= 1 and layers*kv_heads <= 65535",
                  layers, kv_heads, tokens);
        return POLYKV_ESHAPE;
    }
    const int tile_bytes = head_dim == 128  ? tile_bytes_of<128>(value_codec, key_codec)
                           : head_dim == 64 ? tile_bytes_of<64>(value_codec, key_codec)
                                            : tile_bytes_of<256>(value_codec, key_codec);
    // the kernels address a tile within its KV head's records with 32-bit byte offsets
    if (((long long)tokens + kTile - 1) / kTile * tile_bytes > 0xFFFFFFFFll) {
        set_error("pool_create: tokens=%d: the records of one KV head would exceed 4 GiB", tokens);
        return POLYKV_ESHAPE;
    }
    polykv_pool* p = new (std::nothrow) polykv_pool();
    if (p == nullptr) {
        set_error("pool_create: out of host memory");
        return POLYKV_ENOMEM;
    }
    p->layers = layers;
    p->kv_heads = kv_heads;
    p->head_dim = head_dim;
    p->tokens = tokens;
    p->tiles = tiles_of(tokens);
    p->value_codec = value_codec;
    p->key_codec = key_codec;
    p->tile_bytes = tile_bytes;
    p->bytes = (size_t)layers * kv_heads * p->tiles * p->tile_bytes;
    p->kmax_off = 0;
    if (key_codec == POLYKV_KEYS_Q8_TENSOR) {  // the layers' max|k| behind the records, 256-byte aligned
        p->kmax_off = align_up(p->bytes, 256);
        p->bytes = p->kmax_off + align_up((size_t)layers * sizeof(uint32_t), 256);
    }
    p->storage = nullptr;
    p->length = 0;
    memset(&p->signs, 0, sizeof(p->signs));
    *out = p;
    return POLYKV_OK;
}

int pool_set_sign_seed(polykv_pool* pool, uint64_t seed) {
    if (pool == nullptr) {
        set_error("pool_set_sign_seed: pool is NULL");
        return POLYKV_EINVAL;
    }
    if (pool->length != 0) {
        set_error("pool_set_sign_seed: the pool already holds %d tokens", pool->length);
        return POLYKV_ESTATE;
    }
    if (seed != 0 && pool->value_codec == POLYKV_VALUES_INT8) {
        set_error("pool_set_sign_seed: int8 values are not rotated");
        return POLYKV_ESTATE;
    }
    memset(&pool->signs, 0, sizeof(pool->signs));
    if (seed == 0) return POLYKV_OK;
    for (int i = 0; i < pool->head_dim; ++i) {
        // output i of SplitMix64 started at `seed`; the coordinate is negated iff it is odd
        uint64_t z = seed + (uint64_t)(i + 1) * 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        if (z & 1) pool->signs.w[i >> 5] |= 1u << (i & 31);
    }
    for (int k = 0; k < 8; ++k) pool->signs.on |= pool->signs.w[k] != 0;
    return POLYKV_OK;
}

void pool_destroy(polykv_pool* pool) { delete pool; }

size_t pool_bytes(const polykv_pool* pool) { return pool ? pool->bytes : 0; }

int pool_bind(polykv_pool* pool, void* dev_storage, size_t bytes) {
    if (pool == nullptr || dev_storage == nullptr) {
        set_error("pool_bind: NULL pool or storage");
        return POLYKV_EINVAL;
    }
    if (((uintptr_t)dev_storage & 255) != 0) {
        set_error("pool_bind: storage must be 256-byte aligned");
        return POLYKV_EINVAL;
    }
    if (bytes < pool->bytes) {
        set_error("pool_bind: %zu bytes given, %zu needed", bytes, pool->bytes);
        return POLYKV_ENOMEM;
    }
    pool->storage = dev_storage;
    pool->length = 0;
    return POLYKV_OK;
}

static int check_readable(const polykv_pool* pool, const char* who) {
    if (pool == nullptr) {
        set_error("%s: pool is NULL", who);
        return POLYKV_EINVAL;
    }
    if (pool->storage == nullptr) {
        set_error("%s: no storage bound", who);
        return POLYKV_ESTATE;
    }
    if (pool->length == 0) {
        set_error("%s: pool has not been encoded", who);
        return POLYKV_ESTATE;
    }
    return POLYKV_OK;
}

static int hip_result(hipError_t e, const char* who) {
    if (e == hipSuccess) return POLYKV_OK;
    set_error("%s: HIP error %d (%s)", who, (int)e, hipGetErrorString(e));
    return POLYKV_EHIP;
}

static int encode_range(polykv_pool* pool, const void* K_dev, const void* V_dev, int in_dtype, int begin, int count,
                        void* stream, const char* who) {
    if (pool == nullptr || K_dev == nullptr || V_dev == nullptr) {
        set_error("%s: NULL argument", who);
        return POLYKV_EINVAL;
    }
    if (in_dtype != POLYKV_F16 && in_dtype != POLYKV_BF16) {
        set_error("%s: in_dtype %d is neither POLYKV_F16 nor POLYKV_BF16", who, in_dtype);
        return POLYKV_EINVAL;
    }
    if (pool->storage == nullptr) {
        set_error("%s: no storage bound", who);
        return POLYKV_ESTATE;
    }
    if ((((uintptr_t)K_dev | (uintptr_t)V_dev) & 15) != 0) {
        set_error("%s: K and V must be 16-byte aligned", who);
        return POLYKV_EINVAL;
    }
    if (count < 1 || count > pool->tokens - begin) {
        set_error("%s: %d tokens do not fit: %d of the pool's %d are in use", who, count, begin, pool->tokens);
        return POLYKV_ESHAPE;
    }
    const int rc = hip_result(launch_encode(pool, K_dev, V_dev, in_dtype, begin, count, (hipStream_t)stream), who);
    if (rc == POLYKV_OK) pool->length = begin + count;
    return rc;
}

int pool_encode(polykv_pool* pool, const void* K_dev, const void* V_dev, void* stream) {
    return encode_range(pool, K_dev, V_dev, POLYKV_F16, 0, pool ? pool->tokens : 0, stream, "pool_encode");
}

int pool_encode_dtype(polykv_pool* pool, const void* K_dev, const void* V_dev, int in_dtype, void* stream) {
    return encode_range(pool, K_dev, V_dev, in_dtype, 0, pool ? pool->tokens : 0, stream, "pool_encode");
}

int pool_append(polykv_pool* pool, const void* K_dev, const void* V_dev, int count, void* stream) {
    return pool_append_dtype(pool, K_dev, V_dev, count, POLYKV_F16, stream);
}

int pool_append_dtype(polykv_pool* pool, const void* K_dev, const void* V_dev, int count, int in_dtype, void* stream) {
    if (pool != nullptr && pool->key_codec == POLYKV_KEYS_Q8_TENSOR) {
        set_error("pool_append: a pool with one key scale per layer tensor is filled by one pool_encode");
        return POLYKV_ESTATE;
    }
    return encode_range(pool, K_dev, V_dev, in_dtype, pool ? pool->length : 0, count, stream, "pool_append");
}

int pool_length(const polykv_pool* pool) { return pool ? pool->length : 0; }

int pool_decode_layers(const polykv_pool* pool, void* K_out_dev, void* V_out_dev, int out_dtype, int layer_begin,
                       int layer_end, void* stream) {
    int rc = check_readable(pool, "pool_decode");
    if (rc != POLYKV_OK) return rc;
    if (out_dtype != POLYKV_F16 && out_dtype != POLYKV_F32 && out_dtype != POLYKV_BF16) {
        set_error("pool_decode: out_dtype %d is not one of POLYKV_F16, POLYKV_F32, POLYKV_BF16", out_dtype);
        return POLYKV_EINVAL;
    }
    if (layer_begin < 0 || layer_end > pool->layers || layer_begin >= layer_end) {
        set_error("pool_decode: layer range [%d,%d) outside [0,%d)", layer_begin, layer_end, pool->layers);
        return POLYKV_ESHAPE;
    }
    if ((((uintptr_t)K_out_dev | (uintptr_t)V_out_dev) & 15) != 0) {
        set_error("pool_decode: outputs must be 16-byte aligned");
        return POLYKV_EINVAL;
    }
    if (K_out_dev == nullptr && V_out_dev == nullptr) return POLYKV_OK;
    return hip_result(launch_decode(pool, K_out_dev, V_out_dev, out_dtype, layer_begin, layer_end, (hipStream_t)stream),
                      "pool_decode");
}

int pool_decode(const polykv_pool* pool, void* K_out_dev, void* V_out_dev, int out_dtype, void* stream) {
    return pool_decode_layers(pool, K_out_dev, V_out_dev, out_dtype, 0, pool ? pool->layers : 0, stream);
}

int pool_export(const polykv_pool* pool, void* k_codes_dev, void* k_scales_dev, void* v_packed_dev, void* stream) {
    int rc = check_readable(pool, "pool_export");
    if (rc != POLYKV_OK) return rc;
    if (k_codes_dev == nullptr && k_scales_dev == nullptr && v_packed_dev == nullptr) return POLYKV_OK;
    return hip_result(launch_export(pool, k_codes_dev, k_scales_dev, v_packed_dev, nullptr, (hipStream_t)stream),
                      "pool_export");
}

int pool_export_value_scales(const polykv_pool* pool, void* v_scales_dev, void* stream) {
    int rc = check_readable(pool, "pool_export_value_scales");
    if (rc != POLYKV_OK) return rc;
    if (!vc_has_scale(pool->value_codec)) {
        set_error("pool_export_value_scales: the pool's value codec stores no scales");
        return POLYKV_ESTATE;
    }
    if (v_scales_dev == nullptr) {
        set_error("pool_export_value_scales: NULL output");
        return POLYKV_EINVAL;
    }
    return hip_result(launch_export(pool, nullptr, nullptr, nullptr, v_scales_dev, (hipStream_t)stream),
                      "pool_export_value_scales");
}

size_t pool_attend_workspace(const polykv_pool* pool, const polykv_attend_params* params) {
    AttendPlan plan;
    if (make_plan(pool, params, &plan) != POLYKV_OK) return 0;
    return plan.total;
}

// pool_attend with the workspace already resolved: `workspace` holds at least plan.total bytes.
static int attend_with_workspace(const polykv_pool* pool, const AttendPlan& plan, const void* Q_dev, void* out_dev,
                                 const polykv_attend_params* params, void* workspace, void* stream);

int pool_attend(const polykv_pool* pool, const void* Q_dev, void* out_dev, const polykv_attend_params* params,
                void* stream) {
    int rc = check_readable(pool, "pool_attend");
    if (rc != POLYKV_OK) return rc;
    AttendPlan plan;
    rc = make_plan(pool, params, &plan);
    if (rc != POLYKV_OK) return rc;
    if (params->workspace_dev == nullptr || ((uintptr_t)params->workspace_dev & 255) != 0) {
        set_error("pool_attend: workspace must be a 256-byte aligned device pointer");
        return POLYKV_EINVAL;
    }
    if (params->workspace_bytes < plan.total) {
        set_error("pool_attend: workspace has %zu bytes, %zu needed", params->workspace_bytes, plan.total);
        return POLYKV_ENOMEM;
    }
    return attend_with_workspace(pool, plan, Q_dev, out_dev, params, params->workspace_dev, stream);
}

// ---- pool_attend_static: the split partials live in an array that is part of the library's code object.
// Each GPU holds its own copy at its own address; the address is looked up once per device, with that device
// current, and only that pointer -- never the array's name -- is handed to kernels.
static __device__ __align__(256) unsigned char scratch[POLYKV_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

// Device address of `scratch` on the current device (nullptr and an error message on failure).
static void* static_scratch_for_current_device() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        set_error("pool_attend_static: cannot identify the current device (HIP error %d, device %d)", (int)e, dev);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            set_error("pool_attend_static: hipGetSymbolAddress failed on device %d: HIP error %d (%s)", dev, (int)e,
                      hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

int pool_attend_static(const polykv_pool* pool, const void* Q_dev, void* out_dev, const polykv_attend_params* params,
                       void* stream) {
    int rc = check_readable(pool, "pool_attend_static");
    if (rc != POLYKV_OK) return rc;
    AttendPlan plan;
    rc = make_plan(pool, params, &plan);
    if (rc != POLYKV_OK) return rc;
    if (plan.total > (size_t)POLYKV_STATIC_WORKSPACE_BYTES) {
        set_error("pool_attend_static: this call needs %zu bytes of scratch, the built-in buffer holds %zu; use "
                  "pool_attend with a workspace of the caller's",
                  plan.total, (size_t)POLYKV_STATIC_WORKSPACE_BYTES);
        return POLYKV_ENOMEM;
    }
    void* ws = static_scratch_for_current_device();
    if (ws == nullptr) return POLYKV_EHIP;
    return attend_with_workspace(pool, plan, Q_dev, out_dev, params, ws, stream);
}

static int attend_with_workspace(const polykv_pool* pool, const AttendPlan& plan, const void* Q_dev, void* out_dev,
                                 const polykv_attend_params* params, void* workspace, void* stream) {
    if (Q_dev == nullptr || out_dev == nullptr) {
        set_error("pool_attend: NULL Q or out");
        return POLYKV_EINVAL;
    }
    if (((uintptr_t)Q_dev & 15) != 0 || ((uintptr_t)out_dev & 15) != 0) {
        set_error("pool_attend: Q and out must be 16-byte aligned");
        return POLYKV_EINVAL;
    }
    TailPtrs tails;
    if (plan.has_tails) {
        memset(&tails, 0, sizeof(tails));
        for (int a = 0; a < plan.A; ++a) {
            tails.K[a] = params->tail_K[a];
            tails.V[a] = params->tail_V[a];
            tails.len[a] = params->tail_len[a];
            if (tails.len[a] > 0 && ((((uintptr_t)tails.K[a]) | ((uintptr_t)tails.V[a])) & 15) != 0) {
                set_error("pool_attend: tail pointers of agent %d must be 16-byte aligned", a);
                return POLYKV_EINVAL;
            }
        }
    }
    return hip_result(launch_attend(pool, plan, Q_dev, out_dev, plan.has_tails ? &tails : nullptr, workspace,
                                    (hipStream_t)stream),
                      "pool_attend");
}

void polykv_codebook(float* centroids8, float* thresholds7) {
    const float c[4] = {POLYKV_C0, POLYKV_C1, POLYKV_C2, POLYKV_C3};
    const float t[3] = {POLYKV_T1, POLYKV_T2, POLYKV_T3};
    if (centroids8 != nullptr)
        for (int i = 0; i < 4; ++i) {
            centroids8[4 + i] = c[i];
            centroids8[3 - i] = -c[i];
        }
    if (thresholds7 != nullptr) {
        thresholds7[3] = 0.0f;
        for (int i = 0; i < 3; ++i) {
            thresholds7[4 + i] = t[i];
            thresholds7[2 - i] = -t[i];
        }
    }
}

int polykv_codebook_bits(int bits, float* centroids, float* thresholds) {
    if (bits < 2 || bits > 4) {
        set_error("polykv_codebook_bits: bits=%d (2, 3 or 4)", bits);
        return POLYKV_EINVAL;
    }
    const int half = 1 << (bits - 1);
    if (centroids != nullptr)
        for (int i = 0; i < half; ++i) {
            centroids[half + i] = centroid_mag(bits, i);
            centroids[half - 1 - i] = -centroid_mag(bits, i);
        }
    if (thresholds != nullptr) {
        thresholds[half - 1] = 0.0f;
        for (int i = 0; i < half - 1; ++i) {
            thresholds[half + i] = threshold_mag(bits, i);
            thresholds[half - 2 - i] = -threshold_mag(bits, i);
        }
    }
    return POLYKV_OK;
}

int polykv_time_next_kernel(void* start_event, void* stop_event) {
    polykv::g_kernel_events.start = reinterpret_cast<hipEvent_t>(start_event);
    polykv::g_kernel_events.stop = reinterpret_cast<hipEvent_t>(stop_event);
    return POLYKV_OK;
}

const char* polykv_last_error(void) { return g_err; }

}  // extern "C"
