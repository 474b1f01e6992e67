// C ABI of the library: argument validation and kernel dispatch.  See include/vecinfer.h.
#include "../../include/vecinfer.h"

#include "common.h"

#include <atomic>
#include <mutex>

using namespace vecinfer;

// Split partials of vecinfer_decode_attention_static: one fixed array per GPU (every device the
// library's code object is loaded on holds its own copy, at its own address, until the process
// ends).  In host code the name is only a handle for hipGetSymbolAddress; the address that call
// returns is what the kernels get.
static __device__ __align__(256) unsigned char scratch[VECINFER_STATIC_SCRATCH_BYTES];

namespace {

bool cfg_ok(const vecinfer_cfg *c)
{
    if (!c) return false;
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->num_q_heads < 1 || c->num_kv_heads < 1 || c->num_q_heads % c->num_kv_heads) return false;
    const int G = c->num_q_heads / c->num_kv_heads;
    if (G > 8) return false;
    auto sub_ok = [](int d) { return d == 2 || d == 4 || d == 8; };
    if (!sub_ok(c->k_sub_dim) || !sub_ok(c->v_sub_dim)) return false;
    // 10- and 12-bit codes (shared codebook, packed rows): d = 4 or 8 on that side and rows of whole
    // 32-bit words (all but d = 8 with 10 bits at D = 64)
    auto bits_ok = [&](int bits, int d) {
        return bits == 8 || ((bits == 10 || bits == 12) && (d == 4 || d == 8) && (c->head_dim / d * bits) % 32 == 0);
    };
    if (!bits_ok(c->k_bits, c->k_sub_dim) || !bits_ok(c->v_bits, c->v_sub_dim)) return false;
    // tiled value codes: one byte per code, and at least the 16 sub-spaces the block order is made of
    return c->v_tiled == 0 || (c->v_tiled == 1 && c->v_bits == 8 && c->head_dim / c->v_sub_dim >= 16);
}

bool wide(const vecinfer_cfg *c) { return c->k_bits != 8 || c->v_bits != 8; }

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

} // namespace

namespace vecinfer {

int num_cus()
{
    // queried once per process (function-local static: initialised thread-safely); the library is
    // built for one chip, so the first device's count serves every device
    static const int cached = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;                     // MI355X; used only to size the grid
        return n;
    }();
    return cached;
}

} // namespace vecinfer

namespace {

// Splits so that B * H_kv * S fills the compute units once, each split keeping enough
// tokens to amortise staging the codebooks in LDS.
int32_t auto_splits(const vecinfer_cfg *c, int32_t B, int64_t N)
{
    const int64_t groups = (int64_t)B * c->num_kv_heads;
    int64_t s = (num_cus() + groups - 1) / groups;
    const int64_t min_tokens = 1024;
    const int64_t cap = (N + min_tokens - 1) / min_tokens;
    if (s > cap) s = cap;
    if (s > VECINFER_MAX_SPLITS) s = VECINFER_MAX_SPLITS;
    if (s < 1) s = 1;
    return (int32_t)s;
}

// Device address of `scratch` on the current device, resolved once per device.
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

int static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VECINFER_ELAUNCH;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return VECINFER_ELAUNCH;
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *ptr = p;
    return VECINFER_OK;
}

struct WorkspaceLayout {
    size_t off_o, off_m, off_l, off_nsc, off_nv, total;
};

WorkspaceLayout ws_layout(const vecinfer_cfg *c, int32_t B, int32_t S)
{
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    const size_t rows = (size_t)B * c->num_q_heads * S;     // = B * Hkv * S * G
    WorkspaceLayout w;
    size_t off = 0;
    w.off_o = off;
    off += up(sizeof(float) * rows * c->head_dim);
    w.off_m = off;
    off += up(sizeof(float) * rows);
    w.off_l = off;
    off += up(sizeof(float) * rows);
    // fused append: score shares [B, Hkv, Mk, G] and dequantized value [B, Hkv, D] of the new token
    w.off_nsc = off;
    off += up(sizeof(float) * (size_t)B * c->num_q_heads * (c->head_dim / c->k_sub_dim));
    w.off_nv = off;
    off += up(sizeof(float) * (size_t)B * c->num_kv_heads * c->head_dim);
    w.total = off;
    return w;
}

// Validates one encode request and fills the kernel arguments; VECINFER_OK or an error code.
int encode_args(const vecinfer_cfg *cfg, const void *x, const float *lambda, bool keys, const void *cb,
                uint8_t *idx, int32_t B, int64_t T, int64_t pos0, int64_t n_cap, EncodeParams &p)
{
    if (!cfg || !x || !cb || !idx || (keys && !lambda)) return VECINFER_EINVAL;
    if (!cfg_ok(cfg)) return VECINFER_EUNSUPPORTED;
    if (B < 1 || T < 1 || pos0 < 0 || n_cap < 1 || pos0 + T > n_cap) return VECINFER_EINVAL;
    if (!keys && cfg->v_tiled && n_cap % 64 != 0) return VECINFER_EINVAL;       // whole 64-token blocks
    if ((int64_t)B * cfg->num_kv_heads > 65535) return VECINFER_EUNSUPPORTED;
    if ((T + 63) / 64 > 0x7fffffffLL) return VECINFER_EUNSUPPORTED;
    if (!aligned(x, 16) || !aligned(cb, 16) || !aligned(idx, 16) || (keys && !aligned(lambda, 16)))
        return VECINFER_EINVAL;
    p.x = static_cast<const __half *>(x);
    p.lam = keys ? lambda : nullptr;
    p.cb = static_cast<const __half *>(cb);
    p.idx = idx;
    p.B = B;
    p.Hkv = cfg->num_kv_heads;
    p.D = cfg->head_dim;
    p.d = keys ? cfg->k_sub_dim : cfg->v_sub_dim;
    p.M = p.D / p.d;
    p.bits = keys ? cfg->k_bits : cfg->v_bits;
    p.tiled = keys ? 0 : cfg->v_tiled;
    p.T = T;
    p.pos0 = pos0;
    p.n_cap = n_cap;
    p.seq_lens = nullptr;
    p.len_max = 0;
    p.km_sums = nullptr;
    p.km_counts = nullptr;
    p.km_state = nullptr;
    p.km_iter = 0;
    return VECINFER_OK;
}

int launch_status(int rc) { return rc == 0 ? VECINFER_OK : (rc == -2 ? VECINFER_EUNSUPPORTED : VECINFER_ELAUNCH); }

int encode_common(const vecinfer_cfg *cfg, const void *x, const float *lambda, bool keys,
                  const void *cb, uint8_t *idx, int32_t B, int64_t T, int64_t pos0, int64_t n_cap,
                  void *stream)
{
    EncodeParams p;
    const int rc = encode_args(cfg, x, lambda, keys, cb, idx, B, T, pos0, n_cap, p);
    if (rc != VECINFER_OK) return rc;
    return launch_status(launch_encode(p, static_cast<hipStream_t>(stream)));
}

static_assert(VECINFER_MAX_RESIDUAL == kMaxResidual, "header and kernels agree on the window size");

// Shared body of the decode entry points; k_res == nullptr means no residual window,
// k_new == nullptr no fused append (the two are never given together).
int decode_common(const vecinfer_cfg *cfg, const void *q_f16, const float *lambda, const void *cb_k_f16,
                  const void *cb_v_f16, const uint8_t *k_idx, const uint8_t *v_idx, const int32_t *seq_lens,
                  int32_t B, int64_t N, int64_t n_cap, const void *k_res, const void *v_res,
                  const int32_t *res_lens, int32_t R, int64_t r_cap, const void *k_new, const void *v_new,
                  int32_t num_splits, int32_t variant, void *workspace, size_t workspace_bytes, void *out_f16,
                  float *lse, void *stream)
{
    if (!cfg || !q_f16 || !lambda || !cb_k_f16 || !cb_v_f16 || !out_f16) return VECINFER_EINVAL;
    if (!cfg_ok(cfg)) return VECINFER_EUNSUPPORTED;
    const bool window = k_res != nullptr;
    const bool append = k_new != nullptr;
    if (append && (!v_new || !aligned(k_new, 16) || !aligned(v_new, 16))) return VECINFER_EINVAL;
    if (B < 1 || N < (window ? 0 : 1) || n_cap < N) return VECINFER_EINVAL;
    if (cfg->v_tiled && n_cap % 64 != 0) return VECINFER_EINVAL;                  // whole 64-token blocks
    if (N > 0 && (!k_idx || !v_idx)) return VECINFER_EINVAL;
    if (window) {
        if (!v_res || R < 0 || R > r_cap || N + R < 1) return VECINFER_EINVAL;
        if (R > VECINFER_MAX_RESIDUAL) return VECINFER_EUNSUPPORTED;
        if (!aligned(k_res, 16) || !aligned(v_res, 16)) return VECINFER_EINVAL;
    }
    if (num_splits < 0 || num_splits > VECINFER_MAX_SPLITS) return VECINFER_EINVAL;
    if (variant != VECINFER_VARIANT_AUTO && variant != VECINFER_VARIANT_LUT && variant != VECINFER_VARIANT_MFMA &&
        variant != VECINFER_VARIANT_ROLES)
        return VECINFER_EINVAL;
    if (B > 65535 || cfg->num_kv_heads > 65535) return VECINFER_EUNSUPPORTED;      // grid dimensions
    if (!aligned(q_f16, 16) || !aligned(lambda, 16) || !aligned(cb_k_f16, 16) || !aligned(cb_v_f16, 16) ||
        !aligned(k_idx, 16) || !aligned(v_idx, 16) || !aligned(out_f16, 16))
        return VECINFER_EINVAL;
    const int32_t S = N == 0 ? 1 : (num_splits ? num_splits : auto_splits(cfg, B, N));
    const WorkspaceLayout w = ws_layout(cfg, B, S);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < w.total) return VECINFER_EWORKSPACE;

    DecodeParams p;
    p.q = static_cast<const __half *>(q_f16);
    p.lam = lambda;
    p.cb_k = static_cast<const __half *>(cb_k_f16);
    p.cb_v = static_cast<const __half *>(cb_v_f16);
    p.k_idx = k_idx;
    p.v_idx = v_idx;
    p.seq_lens = seq_lens;
    p.B = B;
    p.Hq = cfg->num_q_heads;
    p.Hkv = cfg->num_kv_heads;
    p.G = p.Hq / p.Hkv;
    p.D = cfg->head_dim;
    p.dk = cfg->k_sub_dim;
    p.dv = cfg->v_sub_dim;
    p.Mk = p.D / p.dk;
    p.Mv = p.D / p.dv;
    p.bk = cfg->k_bits;
    p.bv = cfg->v_bits;
    p.v_tiled = cfg->v_tiled;
    p.N = N;
    p.n_cap = n_cap;
    p.S = S;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    p.part_o = reinterpret_cast<float *>(ws + w.off_o);
    p.part_m = reinterpret_cast<float *>(ws + w.off_m);
    p.part_l = reinterpret_cast<float *>(ws + w.off_l);
    p.out = static_cast<__half *>(out_f16);
    p.lse = lse;
    p.k_res = static_cast<const __half *>(k_res);
    p.v_res = static_cast<const __half *>(v_res);
    p.res_lens = window ? res_lens : nullptr;
    p.R = window ? R : 0;
    p.r_cap = window ? r_cap : 0;
    p.k_new = p.v_new = nullptr;
    p.k_idx_w = p.v_idx_w = nullptr;
    p.new_sc = reinterpret_cast<float *>(ws + w.off_nsc);
    p.new_v = reinterpret_cast<float *>(ws + w.off_nv);

    const bool mfma_ok = decode_mfma_supports(p);
    if (variant == VECINFER_VARIANT_MFMA && !mfma_ok) return VECINFER_EUNSUPPORTED;
    const bool use_roles = variant == VECINFER_VARIANT_ROLES;
    if (use_roles && !(mfma_ok && decode_roles_supports(p))) return VECINFER_EUNSUPPORTED;
    const bool use_mfma = use_roles || (variant == VECINFER_VARIANT_MFMA) || (variant == VECINFER_VARIANT_AUTO && mfma_ok);
    // the lookup-table kernel reads one byte per code, from rows
    if (!use_mfma && (wide(cfg) || cfg->v_tiled)) return VECINFER_EUNSUPPORTED;
    int rc = 0;
    if (append && use_mfma) {           // the attention launch encodes the new token itself
        p.k_new = static_cast<const __half *>(k_new);
        p.v_new = static_cast<const __half *>(v_new);
        p.k_idx_w = const_cast<uint8_t *>(k_idx);
        p.v_idx_w = const_cast<uint8_t *>(v_idx);
    } else if (append) {                // separate append launch in front of the plain attention
        EncodeParams pk, pv;
        rc = encode_args(cfg, k_new, lambda, true, cb_k_f16, const_cast<uint8_t *>(k_idx), B, 1, N - 1, n_cap, pk);
        if (rc != VECINFER_OK) return rc;
        rc = encode_args(cfg, v_new, nullptr, false, cb_v_f16, const_cast<uint8_t *>(v_idx), B, 1, N - 1, n_cap, pv);
        if (rc != VECINFER_OK) return rc;
        pk.seq_lens = pv.seq_lens = seq_lens;
        pk.len_max = pv.len_max = N;
        rc = launch_append(pk, pv, static_cast<hipStream_t>(stream));
        if (rc != 0) return launch_status(rc);
    }
    if (N > 0)
        rc = use_roles  ? launch_decode_roles(p, static_cast<hipStream_t>(stream))
             : use_mfma ? launch_decode_mfma(p, static_cast<hipStream_t>(stream))
                        : launch_decode_lut(p, static_cast<hipStream_t>(stream));
    else
        p.S = 0;                        // nothing but the window: the merge kernel sees no split partial
    // log-sum-exp merge of the splits and of the window (single split, no window: done in-kernel)
    if (rc == 0 && (p.S != 1 || window)) rc = launch_merge(p, static_cast<hipStream_t>(stream));
    return launch_status(rc);
}

} // namespace

extern "C" {

int vecinfer_encode_keys(const vecinfer_cfg *cfg, const void *k_f16, const float *lambda,
                         const void *cb_k_f16, uint8_t *k_idx, int32_t B, int64_t T, int64_t pos0,
                         int64_t n_cap, void *stream)
{
    return encode_common(cfg, k_f16, lambda, true, cb_k_f16, k_idx, B, T, pos0, n_cap, stream);
}

int vecinfer_encode_values(const vecinfer_cfg *cfg, const void *v_f16, const void *cb_v_f16,
                           uint8_t *v_idx, int32_t B, int64_t T, int64_t pos0, int64_t n_cap,
                           void *stream)
{
    return encode_common(cfg, v_f16, nullptr, false, cb_v_f16, v_idx, B, T, pos0, n_cap, stream);
}

int vecinfer_append_kv(const vecinfer_cfg *cfg, const void *k_f16, const void *v_f16, const float *lambda,
                       const void *cb_k_f16, const void *cb_v_f16, uint8_t *k_idx, uint8_t *v_idx, int32_t B,
                       int64_t T, int64_t pos0, int64_t n_cap, void *stream)
{
    EncodeParams pk, pv;
    int rc = encode_args(cfg, k_f16, lambda, true, cb_k_f16, k_idx, B, T, pos0, n_cap, pk);
    if (rc != VECINFER_OK) return rc;
    rc = encode_args(cfg, v_f16, nullptr, false, cb_v_f16, v_idx, B, T, pos0, n_cap, pv);
    if (rc != VECINFER_OK) return rc;
    if (T > append_max_tokens()) return VECINFER_EINVAL;
    return launch_status(launch_append(pk, pv, static_cast<hipStream_t>(stream)));
}

int vecinfer_calibrate_lambda(const vecinfer_cfg *cfg, const void *k_f16, float *lambda, int32_t B, int64_t T,
                              void *stream)
{
    if (!cfg || !k_f16 || !lambda) return VECINFER_EINVAL;
    if (!cfg_ok(cfg)) return VECINFER_EUNSUPPORTED;
    if (B < 1 || T < 1) return VECINFER_EINVAL;
    if (B > 65535 || cfg->num_kv_heads > 65535 || (T + 255) / 256 > 0x7fffffffLL) return VECINFER_EUNSUPPORTED;
    if (!aligned(k_f16, 16) || !aligned(lambda, 16)) return VECINFER_EINVAL;
    return launch_status(launch_calibrate_lambda(static_cast<const __half *>(k_f16), lambda, B, cfg->num_kv_heads,
                                                 cfg->head_dim, T, VECINFER_LAMBDA_FLOOR,
                                                 static_cast<hipStream_t>(stream)));
}

size_t vecinfer_kmeans_workspace_bytes(const vecinfer_cfg *cfg, int32_t keys)
{
    if (!cfg_ok(cfg)) return 0;
    const size_t d = keys ? cfg->k_sub_dim : cfg->v_sub_dim;
    const size_t cen = vecinfer_codebook_elems(cfg, keys) / d;     // centroids of the whole tensor
    // fp32 sums, int32 counts, the training state (error accumulators, stopping flag)
    return (cen * d * sizeof(float) + 255) / 256 * 256 + (cen * sizeof(int32_t) + 255) / 256 * 256 +
           (kmeans_state_bytes() + 255) / 256 * 256;
}

namespace {

// Shared body of vecinfer_kmeans_step (one iteration, cb_in -> cb_out) and vecinfer_kmeans_train
// (up to max_iters iterations in place, every one enqueued; iterations after the stop do nothing).
int kmeans_common(const vecinfer_cfg *cfg, const void *x_f16, const float *lambda, const void *cb_in_f16,
                  void *cb_out_f16, uint8_t *codes, int32_t *counts, int32_t B, int64_t T, int32_t max_iters,
                  float tol, int32_t *iters_run, double *errors, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!cfg || !cb_out_f16 || !aligned(cb_out_f16, 16)) return VECINFER_EINVAL;
    vecinfer_cfg rows_cfg = *cfg;
    rows_cfg.v_tiled = 0;                  // the assignment output is always rows
    cfg = &rows_cfg;
    EncodeParams p;
    const bool keys = lambda != nullptr;
    const bool in_place = cb_in_f16 == cb_out_f16;
    const int rc = encode_args(cfg, x_f16, lambda, keys, cb_in_f16, codes, B, T, 0, T, p);
    if (rc != VECINFER_OK) return rc;
    const size_t need = vecinfer_kmeans_workspace_bytes(cfg, keys ? 1 : 0);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < need) return VECINFER_EWORKSPACE;
    const size_t cen = vecinfer_codebook_elems(cfg, keys ? 1 : 0) / p.d;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    p.km_sums = reinterpret_cast<float *>(ws);
    p.km_counts = reinterpret_cast<int32_t *>(ws + (cen * p.d * sizeof(float) + 255) / 256 * 256);
    void *state = ws + (cen * p.d * sizeof(float) + 255) / 256 * 256 + (cen * sizeof(int32_t) + 255) / 256 * 256;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int lr = 0;
    if (!in_place)       // the update works in place on cb_out: start it from cb_in
        lr = hipMemcpyAsync(cb_out_f16, cb_in_f16, cen * p.d * sizeof(__half), hipMemcpyDeviceToDevice, st) == hipSuccess
                 ? 0 : -4;
    p.cb = static_cast<const __half *>(cb_out_f16);
    for (int it = 0; it < max_iters && lr == 0; ++it) {
        lr = launch_kmeans_begin(p.km_sums, p.km_counts, cen * p.d, cen, it, state, st);
        if (lr == 0) {
            if (p.bits == 8) {
                lr = launch_kmeans_assign(p, it, state, st);
            } else {           // 10- / 12-bit codes: the tiled wide cache-fill kernel with its accumulation epilogue
                p.km_state = state;
                p.km_iter = it;
                lr = launch_encode(p, st);
            }
        }
        if (lr == 0)
            lr = launch_kmeans_end(p.km_sums, p.km_counts, static_cast<__half *>(cb_out_f16), counts, cen, p.d, it, tol,
                                   state, iters_run, errors, st);
    }
    return launch_status(lr);
}

} // namespace

int vecinfer_kmeans_step(const vecinfer_cfg *cfg, const void *x_f16, const float *lambda, const void *cb_in_f16,
                         void *cb_out_f16, uint8_t *codes, int32_t *counts, int32_t B, int64_t T, void *workspace,
                         size_t workspace_bytes, void *stream)
{
    return kmeans_common(cfg, x_f16, lambda, cb_in_f16, cb_out_f16, codes, counts, B, T, 1, -1.0f, nullptr, nullptr,
                         workspace, workspace_bytes, stream);
}

int vecinfer_kmeans_train(const vecinfer_cfg *cfg, const void *x_f16, const float *lambda, void *cb_f16, uint8_t *codes,
                          int32_t *counts, int32_t B, int64_t T, int32_t max_iters, float tol, int32_t *iters_run,
                          double *errors, void *workspace, size_t workspace_bytes, void *stream)
{
    if (max_iters < 1 || max_iters > VECINFER_KMEANS_MAX_ITERS || !(tol == tol)) return VECINFER_EINVAL;
    if (errors && !aligned(errors, 8)) return VECINFER_EINVAL;
    if (iters_run && !aligned(iters_run, 4)) return VECINFER_EINVAL;
    return kmeans_common(cfg, x_f16, lambda, cb_f16, cb_f16, codes, counts, B, T, max_iters, tol, iters_run, errors,
                         workspace, workspace_bytes, stream);
}

int32_t vecinfer_decode_auto_splits(const vecinfer_cfg *cfg, int32_t B, int64_t N)
{
    if (!cfg || B < 1 || N < 1) return VECINFER_EINVAL;
    if (!cfg_ok(cfg)) return VECINFER_EUNSUPPORTED;
    return auto_splits(cfg, B, N);
}

size_t vecinfer_decode_workspace_bytes(const vecinfer_cfg *cfg, int32_t B, int64_t N, int32_t num_splits)
{
    if (!cfg_ok(cfg) || B < 1 || N < 0 || num_splits < 0 || num_splits > VECINFER_MAX_SPLITS) return 0;
    const int32_t S = N == 0 ? 1 : (num_splits ? num_splits : auto_splits(cfg, B, N));
    return ws_layout(cfg, B, S).total;
}

int vecinfer_decode_attention(const vecinfer_cfg *cfg, const void *q_f16, const float *lambda,
                              const void *cb_k_f16, const void *cb_v_f16, const uint8_t *k_idx,
                              const uint8_t *v_idx, const int32_t *seq_lens, int32_t B, int64_t N,
                              int64_t n_cap, int32_t num_splits, int32_t variant, void *workspace,
                              size_t workspace_bytes, void *out_f16, float *lse, void *stream)
{
    return decode_common(cfg, q_f16, lambda, cb_k_f16, cb_v_f16, k_idx, v_idx, seq_lens, B, N, n_cap, nullptr,
                         nullptr, nullptr, 0, 0, nullptr, nullptr, num_splits, variant, workspace,
                         workspace_bytes, out_f16, lse, stream);
}

int vecinfer_decode_attention_static(const vecinfer_cfg *cfg, const void *q_f16, const float *lambda,
                                     const void *cb_k_f16, const void *cb_v_f16, const uint8_t *k_idx,
                                     const uint8_t *v_idx, const int32_t *seq_lens, int32_t B, int64_t N,
                                     int64_t n_cap, int32_t num_splits, int32_t variant, void *out_f16, float *lse,
                                     void *stream)
{
    // the size check comes first: a request that does not fit is refused before anything else happens
    if (!cfg) return VECINFER_EINVAL;
    if (!cfg_ok(cfg)) return VECINFER_EUNSUPPORTED;
    if (B < 1 || N < 1 || num_splits < 0 || num_splits > VECINFER_MAX_SPLITS) return VECINFER_EINVAL;
    const int32_t S = num_splits ? num_splits : auto_splits(cfg, B, N);
    if (ws_layout(cfg, B, S).total > (size_t)VECINFER_STATIC_SCRATCH_BYTES) return VECINFER_EWORKSPACE;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != VECINFER_OK) return rc;
    return decode_common(cfg, q_f16, lambda, cb_k_f16, cb_v_f16, k_idx, v_idx, seq_lens, B, N, n_cap, nullptr,
                         nullptr, nullptr, 0, 0, nullptr, nullptr, num_splits, variant, ws,
                         VECINFER_STATIC_SCRATCH_BYTES, out_f16, lse, stream);
}

int vecinfer_decode_step(const vecinfer_cfg *cfg, const void *q_f16, const void *k_new_f16,
                         const void *v_new_f16, const float *lambda, const void *cb_k_f16,
                         const void *cb_v_f16, uint8_t *k_idx, uint8_t *v_idx, const int32_t *seq_lens,
                         int32_t B, int64_t N, int64_t n_cap, int32_t num_splits, int32_t variant,
                         void *workspace, size_t workspace_bytes, void *out_f16, float *lse, void *stream)
{
    if (!k_new_f16 || !v_new_f16 || !k_idx || !v_idx) return VECINFER_EINVAL;
    return decode_common(cfg, q_f16, lambda, cb_k_f16, cb_v_f16, k_idx, v_idx, seq_lens, B, N, n_cap, nullptr,
                         nullptr, nullptr, 0, 0, k_new_f16, v_new_f16, num_splits, variant, workspace,
                         workspace_bytes, out_f16, lse, stream);
}

int vecinfer_decode_attention_residual(const vecinfer_cfg *cfg, const void *q_f16, const float *lambda,
                                       const void *cb_k_f16, const void *cb_v_f16, const uint8_t *k_idx,
                                       const uint8_t *v_idx, const int32_t *seq_lens, int32_t B, int64_t N,
                                       int64_t n_cap, const void *k_res_f16, const void *v_res_f16,
                                       const int32_t *res_lens, int32_t R, int64_t r_cap, int32_t num_splits,
                                       int32_t variant, void *workspace, size_t workspace_bytes, void *out_f16,
                                       float *lse, void *stream)
{
    if (!k_res_f16 || !v_res_f16) return VECINFER_EINVAL;
    return decode_common(cfg, q_f16, lambda, cb_k_f16, cb_v_f16, k_idx, v_idx, seq_lens, B, N, n_cap, k_res_f16,
                         v_res_f16, res_lens, R, r_cap, nullptr, nullptr, num_splits, variant, workspace,
                         workspace_bytes, out_f16, lse, stream);
}

int vecinfer_export_value_codes(const vecinfer_cfg *cfg, const uint8_t *v_idx_tiled, uint8_t *v_idx_rows, int32_t B,
                                int64_t N, int64_t n_cap, void *stream)
{
    if (!cfg || !v_idx_tiled || !v_idx_rows || v_idx_tiled == v_idx_rows) return VECINFER_EINVAL;
    if (!cfg_ok(cfg) || cfg->v_bits != 8) return VECINFER_EUNSUPPORTED;
    if (B < 1 || N < 1 || n_cap < N || n_cap % 64 != 0) return VECINFER_EINVAL;
    if ((int64_t)B * cfg->num_kv_heads > 65535) return VECINFER_EUNSUPPORTED;
    return launch_status(launch_export_value_codes(v_idx_tiled, v_idx_rows, B * cfg->num_kv_heads,
                                                   cfg->head_dim / cfg->v_sub_dim, N, n_cap,
                                                   static_cast<hipStream_t>(stream)));
}

int vecinfer_read_probe(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink || bytes < 16) return VECINFER_EINVAL;
    if (!aligned(src, 16) || !aligned(sink, 4)) return VECINFER_EINVAL;
    return launch_status(launch_read_probe(src, bytes, sink, num_cus(), static_cast<hipStream_t>(stream)));
}

size_t vecinfer_index_row_bytes(const vecinfer_cfg *cfg, int32_t keys)
{
    if (!cfg_ok(cfg)) return 0;
    const size_t d = keys ? cfg->k_sub_dim : cfg->v_sub_dim, bits = keys ? cfg->k_bits : cfg->v_bits;
    return (size_t)cfg->head_dim / d * bits / 8;
}

size_t vecinfer_codebook_elems(const vecinfer_cfg *cfg, int32_t keys)
{
    if (!cfg_ok(cfg)) return 0;
    const size_t d = keys ? cfg->k_sub_dim : cfg->v_sub_dim, bits = keys ? cfg->k_bits : cfg->v_bits;
    const size_t per_head = bits == 8 ? (size_t)cfg->head_dim * kCentroids : ((size_t)1 << bits) * d;
    return per_head * cfg->num_kv_heads;
}

const char *vecinfer_strerror(int code)
{
    switch (code) {
    case VECINFER_OK: return "ok";
    case VECINFER_EINVAL: return "invalid argument";
    case VECINFER_EUNSUPPORTED: return "unsupported configuration";
    case VECINFER_EWORKSPACE: return "workspace missing, misaligned or too small";
    case VECINFER_ELAUNCH: return "HIP launch or device query failed";
    default: return "unknown error code";
    }
}

int vecinfer_version(void) { return VECINFER_VERSION; }

} // extern "C"
