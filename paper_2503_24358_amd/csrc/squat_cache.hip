// squat_cache_*: the residual-buffer bookkeeping of Algorithm 1 (prefill split,
// decoding-phase flush) and of the value path it borrows from KIVI (appendix
// "Details of Our Main Algorithm"), on top of the stateless calls.
//
// Keys: the most recent tokens stay in full precision in a residual buffer of R
// slots; a prompt of l tokens is split into l - (l mod R) quantized tokens and
// l mod R residual tokens; every decoded token is appended to the buffer and,
// when it holds R tokens, all R are quantized with the update matrix and the
// buffer is emptied.  Values: per-token round-to-nearest, the most recent R
// tokens in full precision (a ring): when token R + 1 arrives the oldest one is
// quantized.  Logits: squat_key_scores over the quantized tokens plus plain dot
// products over the residual ones.
//
// key_per_channel selects the grouping Algorithm 1 prints for the keys: every
// flush of R = 32 tokens is one token group quantized per channel
// (squat_quantize_keys_per_channel / squat_key_scores_per_channel); otherwise
// keys are grouped per token (squat_quantize_keys / squat_key_scores).
//
// The object itself is host memory (counters and pointers); every device byte
// lives in one arena the caller provides.  Calls enqueue work on the given
// stream and update the counters at enqueue time: one stream, one host thread
// per cache.
#include <new>

#include "squat_internal.h"

using namespace squat;

struct squat_cache {
    squat_cache_config cfg;
    squat_cache_buffers buf;
    const float* update;
    int64_t n_tokens;          // tokens seen (per sequence; all sequences advance together)
    int64_t n_kq;              // keys in the quantized store
    int n_kres;                // keys in the residual buffer
    int64_t n_vq;              // values in the quantized store
    int v_head;                // ring slot of the oldest full-precision value
    int n_vres;                // full-precision values in the ring
};

namespace {

size_t align_up(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

bool config_ok(const squat_cache_config* c) {
    if (!c) return false;
    if (c->d != kD || (c->bits != 2 && c->bits != 4)) return false;
    if (c->group != 32 && c->group != 64 && c->group != 128) return false;
    if (c->g != 32 && c->g != 64 && c->g != 128) return false;
    if (!(c->group % c->g == 0 || c->g % c->group == 0)) return false;
    if (c->n_batch < 1 || c->n_kv_heads < 1 || c->q_per_kv < 1 || c->q_per_kv > 8) return false;
    if (c->residual < 1 || c->residual > 1024) return false;
    if (c->max_tokens < c->residual || c->max_tokens % c->residual || c->max_tokens >= (int64_t(1) << 25)) return false;
    if (c->kv_dtype != SQUAT_F32 && c->kv_dtype != SQUAT_F16 && c->kv_dtype != SQUAT_BF16) return false;
    if (c->key_per_channel && (c->residual % kTileTokens)) return false;      // whole token groups per flush
    return true;
}

struct Layout {
    size_t codes, meta, kmeta, res, total;
    size_t off_kc, off_ks, off_kz, off_kr, off_vc, off_vs, off_vz, off_vr;
};

Layout layout(const squat_cache_config& c) {
    Layout l;
    const size_t bh = static_cast<size_t>(c.n_batch) * c.n_kv_heads;
    l.codes = align_up(bh * c.max_tokens * (c.d * c.bits / 8));
    l.meta = align_up(bh * c.max_tokens * (c.d / c.group) * 2);
    // per-channel keys: d scales per group of 32 tokens = 4 per token
    l.kmeta = c.key_per_channel ? align_up(bh * c.max_tokens * (c.d / kTileTokens) * 2) : l.meta;
    l.res = align_up(bh * c.residual * c.d * elem_size(c.kv_dtype));
    size_t o = 0;
    l.off_kc = o; o += l.codes;
    l.off_ks = o; o += l.kmeta;
    l.off_kz = o; o += l.kmeta;
    l.off_kr = o; o += l.res;
    l.off_vc = l.off_vs = l.off_vz = l.off_vr = 0;
    if (c.quantize_values) {
        l.off_vc = o; o += l.codes;
        l.off_vs = o; o += l.meta;
        l.off_vz = o; o += l.meta;
        l.off_vr = o; o += l.res;
    }
    l.total = o;
    return l;
}

// dst[b, h, slot0 + t, :] = src[b, h, t, :] for t < count, in 16-byte pieces
__global__ void __launch_bounds__(256) copy_tokens_kernel(const unsigned char* src, int64_t sb, int64_t sh, int64_t st,
                                                         unsigned char* dst, int slots, int slot0, int count,
                                                         int n_heads, int row_bytes, int64_t total) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int ppr = row_bytes / 16;
    const int piece = static_cast<int>(i % ppr);
    const int64_t r = i / ppr;
    const int t = static_cast<int>(r % count);
    const int64_t bh = r / count;
    const int64_t b = bh / n_heads, h = bh % n_heads;
    const u32x4 v = *reinterpret_cast<const u32x4*>(src + b * sb + h * sh + t * st + piece * 16);
    *reinterpret_cast<u32x4*>(dst + (bh * slots + slot0 + t) * row_bytes + piece * 16) = v;
}

// 8 consecutive elements (16-byte aligned) as floats
template <int DT>
__device__ __forceinline__ void load8(const unsigned char* p, float* out) {
    if constexpr (DT == SQUAT_F32) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(p);
        const f32x4 b = *reinterpret_cast<const f32x4*>(p + 16);
        out[0] = a[0]; out[1] = a[1]; out[2] = a[2]; out[3] = a[3];
        out[4] = b[0]; out[5] = b[1]; out[6] = b[2]; out[7] = b[3];
    } else {
        const u32x4 v = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if constexpr (DT == SQUAT_BF16) {
                out[2 * w] = as_f32(v[w] << 16);
                out[2 * w + 1] = as_f32(v[w] & 0xFFFF0000u);
            } else {
                out[2 * w] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(v[w] & 0xFFFFu)));
                out[2 * w + 1] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(v[w] >> 16)));
            }
        }
    }
}

// scores[b, hq, t0 + t] = out_scale * q[b, hq, :] . res[b, hq / qpk, t, :]   for t < count.  Eight lanes per
// (batch, KV head, token): each loads its 16 channels of the key once and meets the same channels of the
// KV head's query heads one after the other (the buffer is read once, not once per query head); a dot
// product is summed by three lane exchanges inside the group.  total = batch x KV heads x count.
template <int QDT, int KDT>
__global__ void __launch_bounds__(256) residual_scores_kernel(const unsigned char* q, int64_t qsb, int64_t qsh,
                                                             const unsigned char* res, int slots, int count,
                                                             int n_kv_heads, int qpk, float out_scale, float* scores,
                                                             int64_t ssb, int64_t ssh, int64_t t0, int64_t total) {
    constexpr int QES = QDT == SQUAT_F32 ? 4 : 2, KES = KDT == SQUAT_F32 ? 4 : 2;
    const int64_t gi = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int part = static_cast<int>(gi & 7);
    int64_t i = gi >> 3;
    const bool live = i < total;
    if (!live) i = total - 1;                      // keep the whole wavefront in the shuffles below
    const int t = static_cast<int>(i % count);
    const int64_t r = i / count;
    const int kvh = static_cast<int>(r % n_kv_heads);
    const int64_t b = r / n_kv_heads;
    const unsigned char* krow =
        res + ((b * n_kv_heads + kvh) * slots + t) * static_cast<int64_t>(kD) * KES + part * 16 * KES;
    float ka[16];
    load8<KDT>(krow, ka);
    load8<KDT>(krow + 8 * KES, ka + 8);
    for (int h = 0; h < qpk; ++h) {
        const int hq = kvh * qpk + h;
        const unsigned char* qrow = q + (b * qsb + hq * qsh) * QES + part * 16 * QES;
        float qa[16];
        load8<QDT>(qrow, qa);
        load8<QDT>(qrow + 8 * QES, qa + 8);
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc = fmaf(qa[e], ka[e], acc);
        acc += __shfl_xor(acc, 1, 64);
        acc += __shfl_xor(acc, 2, 64);
        acc += __shfl_xor(acc, 4, 64);
        if (live && part == 0) scores[b * ssb + hq * ssh + t0 + t] = out_scale * acc;
    }
}

// The same for keys stored before the rotary embedding: the buffered key of cache token t is rotated to position
// pos0 + t first (pairs of channels (c, c + 64), angle position * inv_freq[c]; the partner channels sit in the
// lane four to the side).  The angles depend on the token only, so a thread keeps its 16 (cos, sin) pairs and
// goes over kRopeRes (batch, KV head) pairs with them.  total = ceil(batch x KV heads / kRopeRes) x count.
constexpr int kRopeRes = 8;

template <int QDT, int KDT>
__global__ void __launch_bounds__(256) residual_scores_rope_kernel(const unsigned char* q, int64_t qsb, int64_t qsh,
                                                                  const unsigned char* res, int slots, int count,
                                                                  int64_t n_bh, int n_kv_heads, int qpk,
                                                                  const float* inv_freq, int64_t pos_first,
                                                                  float out_scale, float* scores, int64_t ssb,
                                                                  int64_t ssh, int64_t t0, int64_t total) {
    constexpr int QES = QDT == SQUAT_F32 ? 4 : 2, KES = KDT == SQUAT_F32 ? 4 : 2;
    const int64_t gi = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int part = static_cast<int>(gi & 7);
    int64_t i = gi >> 3;
    const bool live = i < total;
    if (!live) i = total - 1;                      // keep the whole wavefront in the shuffles below
    const int t = static_cast<int>(i % count);
    const int64_t rg = i / count;
    float cs[16], sn[16];
#pragma unroll
    for (int e = 0; e < 16; ++e)
        turn_sincos(static_cast<double>(pos_first + t), inv_freq[16 * (part & 3) + e], cs[e], sn[e]);
    const float sgn = part < 4 ? -1.0f : 1.0f;     // x'_c = x_c cos - x_{c+64} sin,  x'_{c+64} = x_{c+64} cos + x_c sin
    for (int j = 0; j < kRopeRes; ++j) {
        const int64_t r = rg * kRopeRes + j;
        if (r >= n_bh) break;                      // the same for the eight lanes of a group
        const int kvh = static_cast<int>(r % n_kv_heads);
        const int64_t b = r / n_kv_heads;
        const unsigned char* krow = res + (r * slots + t) * static_cast<int64_t>(kD) * KES + part * 16 * KES;
        float ka[16];
        load8<KDT>(krow, ka);
        load8<KDT>(krow + 8 * KES, ka + 8);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float other = __shfl_xor(ka[e], 4, 64);
            ka[e] = fmaf(sgn * other, sn[e], ka[e] * cs[e]);
        }
        for (int h = 0; h < qpk; ++h) {
            const int hq = kvh * qpk + h;
            const unsigned char* qrow = q + (b * qsb + hq * qsh) * QES + part * 16 * QES;
            float qa[16];
            load8<QDT>(qrow, qa);
            load8<QDT>(qrow + 8 * QES, qa + 8);
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc = fmaf(qa[e], ka[e], acc);
            acc += __shfl_xor(acc, 1, 64);
            acc += __shfl_xor(acc, 2, 64);
            acc += __shfl_xor(acc, 4, 64);
            if (live && part == 0) scores[b * ssb + hq * ssh + t0 + t] = out_scale * acc;
        }
    }
}

template <int QDT>
int launch_residual_rope(squat_dtype kdt, dim3 grid, hipStream_t s, const unsigned char* q, int64_t qsb, int64_t qsh,
                         const unsigned char* res, int slots, int count, int64_t n_bh, int n_kv_heads, int qpk,
                         const float* inv_freq, int64_t pos_first, float out_scale, float* scores, int64_t ssb,
                         int64_t ssh, int64_t t0, int64_t total) {
    switch (kdt) {
        case SQUAT_F32: hipLaunchKernelGGL((residual_scores_rope_kernel<QDT, SQUAT_F32>), grid, dim3(256), 0, s, q, qsb, qsh, res, slots, count, n_bh, n_kv_heads, qpk, inv_freq, pos_first, out_scale, scores, ssb, ssh, t0, total); break;
        case SQUAT_F16: hipLaunchKernelGGL((residual_scores_rope_kernel<QDT, SQUAT_F16>), grid, dim3(256), 0, s, q, qsb, qsh, res, slots, count, n_bh, n_kv_heads, qpk, inv_freq, pos_first, out_scale, scores, ssb, ssh, t0, total); break;
        case SQUAT_BF16: hipLaunchKernelGGL((residual_scores_rope_kernel<QDT, SQUAT_BF16>), grid, dim3(256), 0, s, q, qsb, qsh, res, slots, count, n_bh, n_kv_heads, qpk, inv_freq, pos_first, out_scale, scores, ssb, ssh, t0, total); break;
    }
    return check_launch();
}

template <int QDT>
int launch_residual(squat_dtype kdt, dim3 grid, hipStream_t s, const unsigned char* q, int64_t qsb, int64_t qsh,
                    const unsigned char* res, int slots, int count, int n_kv_heads, int qpk, float out_scale,
                    float* scores, int64_t ssb, int64_t ssh, int64_t t0, int64_t total) {
    switch (kdt) {
        case SQUAT_F32: hipLaunchKernelGGL((residual_scores_kernel<QDT, SQUAT_F32>), grid, dim3(256), 0, s, q, qsb, qsh, res, slots, count, n_kv_heads, qpk, out_scale, scores, ssb, ssh, t0, total); break;
        case SQUAT_F16: hipLaunchKernelGGL((residual_scores_kernel<QDT, SQUAT_F16>), grid, dim3(256), 0, s, q, qsb, qsh, res, slots, count, n_kv_heads, qpk, out_scale, scores, ssb, ssh, t0, total); break;
        case SQUAT_BF16: hipLaunchKernelGGL((residual_scores_kernel<QDT, SQUAT_BF16>), grid, dim3(256), 0, s, q, qsb, qsh, res, slots, count, n_kv_heads, qpk, out_scale, scores, ssb, ssh, t0, total); break;
    }
    return check_launch();
}

int copy_tokens(const squat_cache* c, const void* src, int64_t sb, int64_t sh, int64_t st, int64_t first, void* dst,
                int slot0, int count, hipStream_t s) {
    if (count <= 0) return SQUAT_OK;
    const int es = elem_size(c->cfg.kv_dtype);
    const int row_bytes = c->cfg.d * es;
    const int64_t total = c->cfg.n_batch * c->cfg.n_kv_heads * static_cast<int64_t>(count) * (row_bytes / 16);
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFF) return SQUAT_E_BADSHAPE;
    hipLaunchKernelGGL(copy_tokens_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                       static_cast<const unsigned char*>(src) + first * st * es, sb * es, sh * es, st * es,
                       static_cast<unsigned char*>(dst), c->cfg.residual, slot0, count, c->cfg.n_kv_heads, row_bytes,
                       total);
    return check_launch();
}

bool strides_ok(const void* p, int64_t sb, int64_t sh, int64_t st, int d) {
    return p && aligned(p, 16) && st >= d && sb >= 0 && sh >= 0 && !(st % 8) && !(sh % 8) && !(sb % 8);
}

}  // namespace

extern "C" size_t squat_cache_arena_bytes(const squat_cache_config* cfg) {
    return config_ok(cfg) ? layout(*cfg).total : 0;
}

extern "C" int squat_cache_create(const squat_cache_config* cfg, void* arena, size_t arena_bytes, const float* update,
                                  squat_cache** out) {
    if (!out) return SQUAT_E_NULLPTR;
    *out = nullptr;
    if (!config_ok(cfg)) return SQUAT_E_BADSHAPE;
    const Layout l = layout(*cfg);
    if (!arena || arena_bytes < l.total) return SQUAT_E_WORKSPACE;
    if (!aligned(arena, 256) || (update && !aligned(update, 16))) return SQUAT_E_ALIGN;
    squat_cache* c = new (std::nothrow) squat_cache();
    if (!c) return SQUAT_E_WORKSPACE;
    c->cfg = *cfg;
    c->update = update;
    unsigned char* a = static_cast<unsigned char*>(arena);
    c->buf.key_codes = reinterpret_cast<uint32_t*>(a + l.off_kc);
    c->buf.key_scale = reinterpret_cast<uint16_t*>(a + l.off_ks);
    c->buf.key_zero = reinterpret_cast<uint16_t*>(a + l.off_kz);
    c->buf.key_residual = a + l.off_kr;
    c->buf.value_codes = cfg->quantize_values ? reinterpret_cast<uint32_t*>(a + l.off_vc) : nullptr;
    c->buf.value_scale = cfg->quantize_values ? reinterpret_cast<uint16_t*>(a + l.off_vs) : nullptr;
    c->buf.value_zero = cfg->quantize_values ? reinterpret_cast<uint16_t*>(a + l.off_vz) : nullptr;
    c->buf.value_residual = cfg->quantize_values ? a + l.off_vr : nullptr;
    c->n_tokens = c->n_kq = c->n_vq = 0;
    c->n_kres = c->n_vres = c->v_head = 0;
    *out = c;
    return SQUAT_OK;
}

extern "C" void squat_cache_destroy(squat_cache* c) { delete c; }

extern "C" int squat_cache_reset(squat_cache* c) {
    if (!c) return SQUAT_E_NULLPTR;
    c->n_tokens = c->n_kq = c->n_vq = 0;
    c->n_kres = c->n_vres = c->v_head = 0;
    return SQUAT_OK;
}

extern "C" int squat_cache_state(const squat_cache* c, squat_cache_counts* out) {
    if (!c || !out) return SQUAT_E_NULLPTR;
    out->n_tokens = c->n_tokens;
    out->keys_quantized = c->n_kq;
    out->keys_residual = c->n_kres;
    out->values_quantized = c->n_vq;
    out->values_residual = c->n_vres;
    out->value_ring_head = c->v_head;
    return SQUAT_OK;
}

extern "C" int squat_cache_get_buffers(const squat_cache* c, squat_cache_buffers* out) {
    if (!c || !out) return SQUAT_E_NULLPTR;
    *out = c->buf;
    return SQUAT_OK;
}

extern "C" int squat_cache_prefill(squat_cache* c, const void* k, const void* v, int64_t n_tokens,
                                   int64_t stride_batch, int64_t stride_head, int64_t stride_token,
                                   squat_stream stream) {
    if (!c) return SQUAT_E_NULLPTR;
    const squat_cache_config& f = c->cfg;
    if (c->n_tokens != 0 || n_tokens < 0) return SQUAT_E_BADSHAPE;          // prefill fills an empty cache
    if (n_tokens == 0) return SQUAT_OK;
    if (!strides_ok(k, stride_batch, stride_head, stride_token, f.d)) return k ? SQUAT_E_ALIGN : SQUAT_E_NULLPTR;
    if (f.quantize_values && !strides_ok(v, stride_batch, stride_head, stride_token, f.d))
        return v ? SQUAT_E_ALIGN : SQUAT_E_NULLPTR;
    const int R = f.residual;
    const int kres = static_cast<int>(n_tokens % R);
    const int64_t kq = n_tokens - kres;
    const int vres = n_tokens < R ? static_cast<int>(n_tokens) : R;
    const int64_t vq = n_tokens - vres;
    if (kq > f.max_tokens || vq > f.max_tokens) return SQUAT_E_BADSHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = f.key_per_channel
                 ? quantize_keys_pc_into(k, f.kv_dtype, f.n_batch, f.n_kv_heads, kq, f.d, stride_batch, stride_head,
                                         stride_token, c->update, 0, f.bits, kTileTokens, f.g, c->buf.key_codes,
                                         c->buf.key_scale, c->buf.key_zero, f.max_tokens, 0, stream)
                 : quantize_keys_into(k, f.kv_dtype, f.n_batch, f.n_kv_heads, kq, f.d, stride_batch, stride_head,
                                      stride_token, c->update, 0, f.bits, f.group, f.g, c->buf.key_codes,
                                      c->buf.key_scale, c->buf.key_zero, f.max_tokens, 0, stream);
    if (rc) return rc;
    rc = copy_tokens(c, k, stride_batch, stride_head, stride_token, kq, c->buf.key_residual, 0, kres, s);
    if (rc) return rc;
    if (f.quantize_values) {
        // per-token round-to-nearest: no update matrix, one block
        rc = quantize_keys_into(v, f.kv_dtype, f.n_batch, f.n_kv_heads, vq, f.d, stride_batch, stride_head,
                                stride_token, nullptr, 0, f.bits, f.group, f.d, c->buf.value_codes,
                                c->buf.value_scale, c->buf.value_zero, f.max_tokens, 0, stream);
        if (rc) return rc;
        rc = copy_tokens(c, v, stride_batch, stride_head, stride_token, vq, c->buf.value_residual, 0, vres, s);
        if (rc) return rc;
    }
    c->n_tokens = n_tokens;
    c->n_kq = kq;
    c->n_kres = kres;
    c->n_vq = f.quantize_values ? vq : 0;
    c->n_vres = f.quantize_values ? vres : 0;
    c->v_head = 0;
    return SQUAT_OK;
}

extern "C" int squat_cache_append(squat_cache* c, const void* k, const void* v, int64_t stride_batch,
                                  int64_t stride_head, squat_stream stream) {
    if (!c) return SQUAT_E_NULLPTR;
    const squat_cache_config& f = c->cfg;
    if (!strides_ok(k, stride_batch, stride_head, f.d, f.d)) return k ? SQUAT_E_ALIGN : SQUAT_E_NULLPTR;
    if (f.quantize_values && !strides_ok(v, stride_batch, stride_head, f.d, f.d)) return v ? SQUAT_E_ALIGN : SQUAT_E_NULLPTR;
    const int R = f.residual;
    const int es = elem_size(f.kv_dtype);
    const bool flush = c->n_kres + 1 == R;
    if (flush && c->n_kq + R > f.max_tokens) return SQUAT_E_BADSHAPE;           // store full
    const bool v_evict = f.quantize_values && c->n_vres == R;
    if (v_evict && c->n_vq + 1 > f.max_tokens) return SQUAT_E_BADSHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // keys: into the next residual slot; a full buffer is quantized as one group of R tokens and emptied
    int rc = copy_tokens(c, k, stride_batch, stride_head, f.d, 0, c->buf.key_residual, c->n_kres, 1, s);
    if (rc) return rc;
    if (flush) {
        const int64_t rsb = static_cast<int64_t>(f.n_kv_heads) * R * f.d, rsh = static_cast<int64_t>(R) * f.d;
        rc = f.key_per_channel
                 ? quantize_keys_pc_into(c->buf.key_residual, f.kv_dtype, f.n_batch, f.n_kv_heads, R, f.d, rsb, rsh,
                                         f.d, c->update, 0, f.bits, kTileTokens, f.g, c->buf.key_codes,
                                         c->buf.key_scale, c->buf.key_zero, f.max_tokens, c->n_kq, stream)
                 : quantize_keys_into(c->buf.key_residual, f.kv_dtype, f.n_batch, f.n_kv_heads, R, f.d, rsb, rsh, f.d,
                                      c->update, 0, f.bits, f.group, f.g, c->buf.key_codes, c->buf.key_scale,
                                      c->buf.key_zero, f.max_tokens, c->n_kq, stream);
        if (rc) return rc;
    }
    if (f.quantize_values) {
        int slot = (c->v_head + c->n_vres) % R;
        if (v_evict) {
            // the ring is full: its oldest token is quantized, its slot takes the new token
            const unsigned char* oldest = static_cast<const unsigned char*>(c->buf.value_residual) +
                                          static_cast<int64_t>(c->v_head) * f.d * es;
            rc = quantize_keys_into(oldest, f.kv_dtype, f.n_batch, f.n_kv_heads, 1, f.d,
                                    static_cast<int64_t>(f.n_kv_heads) * R * f.d, static_cast<int64_t>(R) * f.d, f.d,
                                    nullptr, 0, f.bits, f.group, f.d, c->buf.value_codes, c->buf.value_scale,
                                    c->buf.value_zero, f.max_tokens, c->n_vq, stream);
            if (rc) return rc;
            slot = c->v_head;
        }
        rc = copy_tokens(c, v, stride_batch, stride_head, f.d, 0, c->buf.value_residual, slot, 1, s);
        if (rc) return rc;
        if (v_evict) {
            c->v_head = (c->v_head + 1) % R;
            c->n_vq += 1;
        } else {
            c->n_vres += 1;
        }
    }
    if (flush) {
        c->n_kq += R;
        c->n_kres = 0;
    } else {
        c->n_kres += 1;
    }
    c->n_tokens += 1;
    return SQUAT_OK;
}

extern "C" int squat_cache_key_scores(const squat_cache* c, const void* q, squat_dtype q_dt, int64_t q_stride_batch,
                                      int64_t q_stride_head, float out_scale, float* scores,
                                      int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream) {
    if (!c) return SQUAT_E_NULLPTR;
    const squat_cache_config& f = c->cfg;
    if (!q || !scores) return SQUAT_E_NULLPTR;
    if (q_dt != SQUAT_F32 && q_dt != SQUAT_F16 && q_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (s_stride_head < c->n_kq + c->n_kres || s_stride_batch < 0 || q_stride_head < f.d || q_stride_batch < 0)
        return SQUAT_E_BADSHAPE;
    if ((q_stride_head % 8) || (q_stride_batch % 8) || !aligned(q, 16) || !aligned(scores, 4)) return SQUAT_E_ALIGN;
    int rc = f.key_per_channel
                 ? key_scores_pc_from(c->buf.key_codes, c->buf.key_scale, c->buf.key_zero, f.n_batch, f.n_kv_heads,
                                      c->n_kq, f.max_tokens, f.d, f.bits, kTileTokens, q, q_dt, f.q_per_kv,
                                      q_stride_batch, q_stride_head, out_scale, scores, s_stride_batch,
                                      s_stride_head, stream)
                 : key_scores_from(c->buf.key_codes, c->buf.key_scale, c->buf.key_zero, f.n_batch, f.n_kv_heads,
                                   c->n_kq, f.max_tokens, f.d, f.bits, f.group, q, q_dt, f.q_per_kv, q_stride_batch,
                                   q_stride_head, out_scale, scores, s_stride_batch, s_stride_head, stream);
    if (rc) return rc;
    if (c->n_kres == 0) return SQUAT_OK;
    const int64_t total = f.n_batch * f.n_kv_heads * static_cast<int64_t>(c->n_kres);
    const int64_t blocks = (total * 8 + 255) / 256;          // eight lanes per buffered key
    if (blocks > 0x7FFFFFFF) return SQUAT_E_BADSHAPE;
    const dim3 grid(static_cast<unsigned>(blocks));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned char* qp = static_cast<const unsigned char*>(q);
    const unsigned char* res = static_cast<const unsigned char*>(c->buf.key_residual);
    switch (q_dt) {
        case SQUAT_F32: return launch_residual<SQUAT_F32>(f.kv_dtype, grid, s, qp, q_stride_batch, q_stride_head, res, f.residual, c->n_kres, f.n_kv_heads, f.q_per_kv, out_scale, scores, s_stride_batch, s_stride_head, c->n_kq, total);
        case SQUAT_F16: return launch_residual<SQUAT_F16>(f.kv_dtype, grid, s, qp, q_stride_batch, q_stride_head, res, f.residual, c->n_kres, f.n_kv_heads, f.q_per_kv, out_scale, scores, s_stride_batch, s_stride_head, c->n_kq, total);
        case SQUAT_BF16: return launch_residual<SQUAT_BF16>(f.kv_dtype, grid, s, qp, q_stride_batch, q_stride_head, res, f.residual, c->n_kres, f.n_kv_heads, f.q_per_kv, out_scale, scores, s_stride_batch, s_stride_head, c->n_kq, total);
    }
    return SQUAT_E_BADDTYPE;
}

extern "C" int squat_cache_key_scores_rope(const squat_cache* c, const void* q, squat_dtype q_dt,
                                           int64_t q_stride_batch, int64_t q_stride_head, const float* inv_freq,
                                           int64_t pos0, float out_scale, float* scores, int64_t s_stride_batch,
                                           int64_t s_stride_head, squat_stream stream) {
    if (!c) return SQUAT_E_NULLPTR;
    const squat_cache_config& f = c->cfg;
    if (!q || !scores || !inv_freq) return SQUAT_E_NULLPTR;
    if (q_dt != SQUAT_F32 && q_dt != SQUAT_F16 && q_dt != SQUAT_BF16) return SQUAT_E_BADDTYPE;
    if (pos0 < 0 || pos0 >= (int64_t(1) << 40)) return SQUAT_E_BADSHAPE;
    if (s_stride_head < c->n_kq + c->n_kres || s_stride_batch < 0 || q_stride_head < f.d || q_stride_batch < 0)
        return SQUAT_E_BADSHAPE;
    if ((q_stride_head % 8) || (q_stride_batch % 8) || !aligned(q, 16) || !aligned(scores, 4) || !aligned(inv_freq, 4))
        return SQUAT_E_ALIGN;
    int rc = f.key_per_channel
                 ? key_scores_pc_rope_from(c->buf.key_codes, c->buf.key_scale, c->buf.key_zero, f.n_batch,
                                           f.n_kv_heads, c->n_kq, f.max_tokens, f.d, f.bits, kTileTokens, inv_freq,
                                           pos0, q, q_dt, f.q_per_kv, q_stride_batch, q_stride_head, out_scale,
                                           scores, s_stride_batch, s_stride_head, stream)
                 : key_scores_rope_from(c->buf.key_codes, c->buf.key_scale, c->buf.key_zero, f.n_batch, f.n_kv_heads,
                                        c->n_kq, f.max_tokens, f.d, f.bits, f.group, inv_freq, pos0, q, q_dt,
                                        f.q_per_kv, q_stride_batch, q_stride_head, out_scale, scores,
                                        s_stride_batch, s_stride_head, stream);
    if (rc) return rc;
    if (c->n_kres == 0) return SQUAT_OK;
    const int64_t n_bh = f.n_batch * f.n_kv_heads;
    const int64_t total = ((n_bh + kRopeRes - 1) / kRopeRes) * static_cast<int64_t>(c->n_kres);
    const int64_t blocks = (total * 8 + 255) / 256;          // eight lanes per (group of pairs, buffered token)
    if (blocks > 0x7FFFFFFF) return SQUAT_E_BADSHAPE;
    const dim3 grid(static_cast<unsigned>(blocks));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned char* qp = static_cast<const unsigned char*>(q);
    const unsigned char* res = static_cast<const unsigned char*>(c->buf.key_residual);
    const int64_t pos_first = pos0 + c->n_kq;                // position of the oldest buffered key
    switch (q_dt) {
        case SQUAT_F32: return launch_residual_rope<SQUAT_F32>(f.kv_dtype, grid, s, qp, q_stride_batch, q_stride_head, res, f.residual, c->n_kres, n_bh, f.n_kv_heads, f.q_per_kv, inv_freq, pos_first, out_scale, scores, s_stride_batch, s_stride_head, c->n_kq, total);
        case SQUAT_F16: return launch_residual_rope<SQUAT_F16>(f.kv_dtype, grid, s, qp, q_stride_batch, q_stride_head, res, f.residual, c->n_kres, n_bh, f.n_kv_heads, f.q_per_kv, inv_freq, pos_first, out_scale, scores, s_stride_batch, s_stride_head, c->n_kq, total);
        case SQUAT_BF16: return launch_residual_rope<SQUAT_BF16>(f.kv_dtype, grid, s, qp, q_stride_batch, q_stride_head, res, f.residual, c->n_kres, n_bh, f.n_kv_heads, f.q_per_kv, inv_freq, pos_first, out_scale, scores, s_stride_batch, s_stride_head, c->n_kq, total);
    }
    return SQUAT_E_BADDTYPE;
}
