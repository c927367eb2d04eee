// C ABI of libloma: argument checking on the host, then dispatch to the kernels.
// Nothing here allocates, frees or synchronises; every error is detected before a launch.
#include <cmath>
#include <cstdint>

#include "loma_internal.h"
#include "loma_rope.h"

namespace {

using loma::Geometry;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool good_ptr(const void* p) { return p != nullptr && aligned16(p); }

// B, H, head_dim, t, c, dtype, scale: shared by all entry points
int check_common(int B, int H, int head_dim, int t, int c, float scale, int dtype) {
    if (B < 1 || H < 1 || t < 1 || c < 1) return LOMA_ERR_INVALID_ARG;
    if (!(scale > 0.f) || !std::isfinite(scale)) return LOMA_ERR_INVALID_ARG;
    if (dtype != LOMA_F32 && dtype != LOMA_BF16) return LOMA_ERR_UNSUPPORTED;
    if (head_dim < 8 || head_dim > 256 || head_dim % 8 != 0) return LOMA_ERR_UNSUPPORTED;
    if ((long long)B * H > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    if ((long long)t * c > (1 << 24)) return LOMA_ERR_UNSUPPORTED;
    return LOMA_OK;
}

}  // namespace

extern "C" {

const char* loma_status_string(int status) {
    switch (status) {
        case LOMA_OK: return "ok";
        case LOMA_ERR_INVALID_ARG: return "invalid argument";
        case LOMA_ERR_UNSUPPORTED: return "unsupported dtype, head_dim or size";
        case LOMA_ERR_WORKSPACE: return "workspace missing or too small";
        case LOMA_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

int loma_abi_version(void) { return 1; }

int loma_mask_attn_fwd(const void* q, const void* k, const void* v, void* out, float* lse,
                       int B, int H, int head_dim, int t, int c, int n_chunks,
                       float scale, int dtype, void* stream) {
    if (int rc = check_common(B, H, head_dim, t, c, scale, dtype)) return rc;
    if (n_chunks < 1) return LOMA_ERR_INVALID_ARG;
    if (!good_ptr(q) || !good_ptr(k) || !good_ptr(v) || !good_ptr(out)) return LOMA_ERR_INVALID_ARG;
    if (lse != nullptr && (reinterpret_cast<uintptr_t>(lse) & 3u)) return LOMA_ERR_INVALID_ARG;
    Geometry g;
    g.t = t; g.c = c; g.n = n_chunks; g.R = t * c; g.s = t * (2 * c + 1);
    const long long S = (long long)n_chunks * g.s;
    if (S > (1LL << 30)) return LOMA_ERR_UNSUPPORTED;
    g.S = (int)S;
    const int nbh = B * H;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (loma::use_mfma_path(dtype, head_dim) && loma::mask_attn_mfma_fits(g))
        return loma::launch_mask_attn_mfma(q, k, v, out, lse, nbh, head_dim, g, scale, st);
    return loma::launch_mask_attn_generic(q, k, v, out, lse, nbh, head_dim, g, scale, dtype, st);
}

size_t loma_mask_attn_bwd_workspace_bytes(int B, int H, int head_dim, int t, int c, int n_chunks, int dtype) {
    if (check_common(B, H, head_dim, t, c, 1.f, dtype) != LOMA_OK || n_chunks < 1) return 0;
    const long long S = (long long)n_chunks * t * (2 * c + 1);
    if (S > (1LL << 30)) return 0;
    if (loma::use_mfma_path(dtype, head_dim)) {
        Geometry g;
        g.t = t; g.c = c; g.n = n_chunks; g.R = t * c; g.s = t * (2 * c + 1); g.S = (int)S;
        if (loma::mask_attn_bwd_mfma_fits(g))
            return loma::mask_attn_bwd_mfma_workspace_floats(B * H, head_dim, g) * sizeof(float);
    }
    return (size_t)B * H * (size_t)S * 2 * sizeof(float);   // per row: dout . out and -lse * log2(e)
}

int loma_mask_attn_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse,
                       const void* dout, void* dq, void* dk, void* dv,
                       int B, int H, int head_dim, int t, int c, int n_chunks,
                       float scale, int dtype,
                       void* workspace, size_t workspace_bytes, void* stream) {
    if (int rc = check_common(B, H, head_dim, t, c, scale, dtype)) return rc;
    if (n_chunks < 1) return LOMA_ERR_INVALID_ARG;
    if (!good_ptr(q) || !good_ptr(k) || !good_ptr(v) || !good_ptr(out) || !good_ptr(dout) || !good_ptr(dq) ||
        !good_ptr(dk) || !good_ptr(dv))
        return LOMA_ERR_INVALID_ARG;
    if (lse == nullptr || (reinterpret_cast<uintptr_t>(lse) & 3u)) return LOMA_ERR_INVALID_ARG;
    for (const void* o : {(const void*)dq, (const void*)dk, (const void*)dv}) {
        for (const void* i : {q, k, v, out, dout}) if (o == i) return LOMA_ERR_INVALID_ARG;
    }
    if (dq == dk || dq == dv || dk == dv) return LOMA_ERR_INVALID_ARG;
    Geometry g;
    g.t = t; g.c = c; g.n = n_chunks; g.R = t * c; g.s = t * (2 * c + 1);
    const long long S = (long long)n_chunks * g.s;
    if (S > (1LL << 30)) return LOMA_ERR_UNSUPPORTED;
    g.S = (int)S;
    const size_t need = loma_mask_attn_bwd_workspace_bytes(B, H, head_dim, t, c, n_chunks, dtype);
    if (workspace == nullptr || workspace_bytes < need || !aligned16(workspace)) return LOMA_ERR_WORKSPACE;
    const int nbh = B * H;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (loma::use_mfma_path(dtype, head_dim) && loma::mask_attn_bwd_mfma_fits(g))
        return loma::launch_mask_attn_bwd_mfma(q, k, v, out, lse, dout, dq, dk, dv, static_cast<float*>(workspace),
                                               nbh, head_dim, g, scale, st);
    return loma::launch_mask_attn_bwd_generic(q, k, v, out, lse, dout, dq, dk, dv, static_cast<float*>(workspace),
                                              nbh, head_dim, g, scale, dtype, st);
}

}  // extern "C" (reopened below)

namespace {

bool good_rope(int pos_first, int pos_stride, float theta) {
    return pos_first >= 0 && pos_stride >= 0 && theta > 0.f && std::isfinite(theta);
}

int compress_step_impl(const void* q_mem, const void* k_mem, const void* v_mem,
                       const void* k_read, const void* v_read,
                       void* k_memcache, void* v_memcache, void* out,
                       int B, int H, int head_dim, int t, int c,
                       int n_mem_chunks, int mem_capacity,
                       float scale, int dtype, void* stream, const loma::RopeTable* rope) {
    if (int rc = check_common(B, H, head_dim, t, c, scale, dtype)) return rc;
    if (n_mem_chunks < 0 || mem_capacity < 1) return LOMA_ERR_INVALID_ARG;
    if (((long long)n_mem_chunks + 1) * t > mem_capacity) return LOMA_ERR_INVALID_ARG;
    if (!good_ptr(q_mem) || !good_ptr(k_mem) || !good_ptr(v_mem) || !good_ptr(k_read) || !good_ptr(v_read) ||
        !good_ptr(k_memcache) || !good_ptr(v_memcache) || !good_ptr(out))
        return LOMA_ERR_INVALID_ARG;
    if (rope != nullptr && out == q_mem) return LOMA_ERR_INVALID_ARG;   // out holds the rotated queries meanwhile
    const int nbh = B * H;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (loma::use_mfma_path(dtype, head_dim))
        return loma::launch_compress_mfma(q_mem, k_mem, v_mem, k_read, v_read, k_memcache, v_memcache, out,
                                          nbh, head_dim, t, c, n_mem_chunks, mem_capacity, scale, st, rope);
    if (rope != nullptr) return LOMA_ERR_UNSUPPORTED;
    return loma::launch_compress_generic(q_mem, k_mem, v_mem, k_read, v_read, k_memcache, v_memcache, out,
                                         nbh, head_dim, t, c, n_mem_chunks, mem_capacity, scale, dtype, st);
}

}  // namespace

extern "C" {

int loma_compress_step(const void* q_mem, const void* k_mem, const void* v_mem,
                       const void* k_read, const void* v_read,
                       void* k_memcache, void* v_memcache, void* out,
                       int B, int H, int head_dim, int t, int c,
                       int n_mem_chunks, int mem_capacity,
                       float scale, int dtype, void* stream) {
    return compress_step_impl(q_mem, k_mem, v_mem, k_read, v_read, k_memcache, v_memcache, out, B, H, head_dim, t, c,
                              n_mem_chunks, mem_capacity, scale, dtype, stream, nullptr);
}

int loma_compress_step_rope(const void* q_mem, const void* k_mem, const void* v_mem,
                            const void* k_read, const void* v_read,
                            void* k_memcache, void* v_memcache, void* out,
                            int B, int H, int head_dim, int t, int c,
                            int n_mem_chunks, int mem_capacity,
                            float scale, int dtype,
                            int pos_first, int pos_stride, float rope_theta, void* stream) {
    if (!good_rope(pos_first, pos_stride, rope_theta)) return LOMA_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return LOMA_ERR_UNSUPPORTED;
    const loma::RopeTable rt = loma::make_rope_table(head_dim, rope_theta, pos_first, pos_stride);
    return compress_step_impl(q_mem, k_mem, v_mem, k_read, v_read, k_memcache, v_memcache, out, B, H, head_dim, t, c,
                              n_mem_chunks, mem_capacity, scale, dtype, stream, &rt);
}

int loma_memory_position_ids(int t, int c, int chunk, int position_type, int* ids) {
    if (t < 1 || c < 1 || chunk < 0 || ids == nullptr) return LOMA_ERR_INVALID_ARG;
    if (position_type != LOMA_POS_INTERMITTENT && position_type != LOMA_POS_CONTIGUOUS) return LOMA_ERR_INVALID_ARG;
    const long long R = (long long)t * c;
    if (((long long)chunk + 1) * R > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    for (int j = 0; j < t; ++j)
        ids[j] = position_type == LOMA_POS_INTERMITTENT ? (int)(chunk * R + (long long)(j + 1) * c - 1)   // Eq. 14
                                                         : chunk * t + j;                                  // mem_cursor + j
    return LOMA_OK;
}

int loma_sample_position_ids(int t, int c, int n_chunks, int position_type, int* ids) {
    if (t < 1 || c < 1 || n_chunks < 1 || ids == nullptr) return LOMA_ERR_INVALID_ARG;
    if (position_type != LOMA_POS_INTERMITTENT && position_type != LOMA_POS_CONTIGUOUS) return LOMA_ERR_INVALID_ARG;
    const long long R = (long long)t * c, s = 2 * R + t;
    if (n_chunks * s > (1LL << 30)) return LOMA_ERR_UNSUPPORTED;
    for (int y = 0; y < n_chunks; ++y) {
        int* row = ids + y * s;
        for (int j = 0; j < R; ++j) row[j] = row[R + t + j] = (int)(y * R + j);   // <r> tokens: the ids of the tokens they reproduce
        if (int rc = loma_memory_position_ids(t, c, y, position_type, row + R)) return rc;
    }
    return LOMA_OK;
}

size_t loma_decode_workspace_bytes(int B, int H, int head_dim, int t, int c, int n_mem_chunks, int dtype) {
    if (check_common(B, H, head_dim, t, c, 1.f, dtype) != LOMA_OK || n_mem_chunks < 0) return 0;
    if (!loma::use_mfma_path(dtype, head_dim)) return 0;
    const long long nmax = (long long)n_mem_chunks * t + (long long)t * c;
    if (nmax > 0x7fffffffLL) return 0;
    return loma::decode_workspace_bytes(B * H, head_dim, (int)nmax);
}

}  // extern "C" (reopened below)

namespace {

// Argument checks shared by the forms of the decode step (everything except the tensors' own pointers).
int check_decode_state(int B, int H, int head_dim, int t, int c, int n_mem_chunks, int mem_capacity, int read_fill,
                       bool has_new, float scale, int dtype, long long* n_mem_keys) {
    if (int rc = check_common(B, H, head_dim, t, c, scale, dtype)) return rc;
    const int R = t * c;
    if (n_mem_chunks < 0 || mem_capacity < 0 || read_fill < 0) return LOMA_ERR_INVALID_ARG;
    *n_mem_keys = (long long)n_mem_chunks * t;
    if (*n_mem_keys > mem_capacity) return LOMA_ERR_INVALID_ARG;
    // Appendix A keeps the reading zone shorter than t*c whenever a token is fed
    if (has_new ? read_fill >= R : read_fill > R) return LOMA_ERR_INVALID_ARG;
    if (*n_mem_keys + read_fill + (has_new ? 1 : 0) < 1) return LOMA_ERR_INVALID_ARG;
    return LOMA_OK;
}

int decode_attn_impl(const void* q, const void* k_new, const void* v_new,
                     const void* k_memcache, const void* v_memcache,
                     void* k_read, void* v_read, void* out,
                     int B, int H, int head_dim, int t, int c,
                     int n_mem_chunks, int mem_capacity, int read_fill,
                     float scale, int dtype, bool static_scratch,
                     void* workspace, size_t workspace_bytes, void* stream, const loma::RopeTable* rope = nullptr) {
    if ((k_new == nullptr) != (v_new == nullptr)) return LOMA_ERR_INVALID_ARG;
    const bool has_new = k_new != nullptr;
    long long n_mem_keys = 0;
    if (int rc = check_decode_state(B, H, head_dim, t, c, n_mem_chunks, mem_capacity, read_fill, has_new, scale, dtype,
                                    &n_mem_keys))
        return rc;
    const int R = t * c;
    if (!good_ptr(q) || !good_ptr(out) || !good_ptr(k_read) || !good_ptr(v_read)) return LOMA_ERR_INVALID_ARG;
    if (has_new && (!aligned16(k_new) || !aligned16(v_new))) return LOMA_ERR_INVALID_ARG;
    if (n_mem_chunks > 0 && (!good_ptr(k_memcache) || !good_ptr(v_memcache))) return LOMA_ERR_INVALID_ARG;
    const int nbh = B * H;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (loma::use_mfma_path(dtype, head_dim)) {
        const size_t need = loma::decode_workspace_bytes(nbh, head_dim, (int)n_mem_keys + R);
        if (nbh > 65535) return LOMA_ERR_UNSUPPORTED;
        if (static_scratch) {
            if (need > loma::decode_static_scratch_bytes()) return LOMA_ERR_UNSUPPORTED;
            workspace = nullptr;
            if (need > 0 && (workspace = loma::decode_static_scratch_ptr()) == nullptr) return LOMA_ERR_LAUNCH;
        } else if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned16(workspace))) {
            return LOMA_ERR_WORKSPACE;
        }
        return loma::launch_decode_splitk(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, nbh,
                                          head_dim, R, (int)n_mem_keys, mem_capacity, read_fill, scale,
                                          need > 0 ? workspace : nullptr, st, rope);
    }
    if (rope != nullptr) return LOMA_ERR_UNSUPPORTED;
    return loma::launch_decode_generic(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, nbh,
                                       head_dim, R, (int)n_mem_keys, mem_capacity, read_fill, scale, dtype, st);
}

}  // namespace

extern "C" {

int loma_decode_attn(const void* q, const void* k_new, const void* v_new,
                     const void* k_memcache, const void* v_memcache,
                     void* k_read, void* v_read, void* out,
                     int B, int H, int head_dim, int t, int c,
                     int n_mem_chunks, int mem_capacity, int read_fill,
                     float scale, int dtype,
                     void* workspace, size_t workspace_bytes, void* stream) {
    return decode_attn_impl(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, B, H, head_dim, t, c,
                            n_mem_chunks, mem_capacity, read_fill, scale, dtype, false, workspace, workspace_bytes, stream);
}

int loma_decode_attn_static(const void* q, const void* k_new, const void* v_new,
                            const void* k_memcache, const void* v_memcache,
                            void* k_read, void* v_read, void* out,
                            int B, int H, int head_dim, int t, int c,
                            int n_mem_chunks, int mem_capacity, int read_fill,
                            float scale, int dtype, void* stream) {
    return decode_attn_impl(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, B, H, head_dim, t, c,
                            n_mem_chunks, mem_capacity, read_fill, scale, dtype, true, nullptr, 0, stream);
}

int loma_decode_attn_rope(const void* q, const void* k_new, const void* v_new,
                          const void* k_memcache, const void* v_memcache,
                          void* k_read, void* v_read, void* out,
                          int B, int H, int head_dim, int t, int c,
                          int n_mem_chunks, int mem_capacity, int read_fill,
                          float scale, int dtype, int pos, float rope_theta,
                          void* workspace, size_t workspace_bytes, void* stream) {
    if (!good_rope(pos, 0, rope_theta)) return LOMA_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return LOMA_ERR_UNSUPPORTED;
    const loma::RopeTable rt = loma::make_rope_table(head_dim, rope_theta, pos, 0);
    return decode_attn_impl(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, B, H, head_dim, t, c,
                            n_mem_chunks, mem_capacity, read_fill, scale, dtype, false, workspace, workspace_bytes, stream,
                            &rt);
}

static bool good_gqa_heads(int H, int H_kv) {
    if (H < 1 || H_kv < 1 || H % H_kv != 0) return false;
    return true;
}

size_t loma_decode_gqa_workspace_bytes(int B, int H, int H_kv, int head_dim, int dtype) {
    if (B < 1 || !good_gqa_heads(H, H_kv) || !loma::use_mfma_path(dtype, head_dim)) return 0;
    if ((long long)B * H_kv > 65535) return 0;
    return loma::decode_gqa_workspace_bytes(B * H_kv, H / H_kv, head_dim);
}

int loma_decode_attn_gqa(const void* q, const void* k_new, const void* v_new,
                         const void* k_memcache, const void* v_memcache,
                         void* k_read, void* v_read, void* out,
                         int B, int H, int H_kv, int head_dim, int t, int c,
                         int n_mem_chunks, int mem_capacity, int read_fill,
                         float scale, int dtype,
                         void* workspace, size_t workspace_bytes, void* stream) {
    if ((k_new == nullptr) != (v_new == nullptr)) return LOMA_ERR_INVALID_ARG;
    if (!good_gqa_heads(H, H_kv)) return LOMA_ERR_INVALID_ARG;
    const bool has_new = k_new != nullptr;
    long long n_mem_keys = 0;
    // the cache state is that of B * H_kv sequences
    if (int rc = check_decode_state(B, H_kv, head_dim, t, c, n_mem_chunks, mem_capacity, read_fill, has_new, scale, dtype,
                                    &n_mem_keys))
        return rc;
    if (!good_ptr(q) || !good_ptr(out) || !good_ptr(k_read) || !good_ptr(v_read)) return LOMA_ERR_INVALID_ARG;
    if (has_new && (!aligned16(k_new) || !aligned16(v_new))) return LOMA_ERR_INVALID_ARG;
    if (n_mem_chunks > 0 && (!good_ptr(k_memcache) || !good_ptr(v_memcache))) return LOMA_ERR_INVALID_ARG;
    const int G = H / H_kv;
    if (G != 1 && G != 2 && G != 4 && G != 8) return LOMA_ERR_UNSUPPORTED;
    if (!loma::use_mfma_path(dtype, head_dim)) return LOMA_ERR_UNSUPPORTED;
    if ((long long)B * H_kv > 65535) return LOMA_ERR_UNSUPPORTED;
    const int nbh_kv = B * H_kv;
    const size_t need = loma::decode_gqa_workspace_bytes(nbh_kv, G, head_dim);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned16(workspace))) return LOMA_ERR_WORKSPACE;
    return loma::launch_decode_gqa(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, nbh_kv, G, head_dim,
                                   t * c, (int)n_mem_keys, mem_capacity, read_fill, scale, need > 0 ? workspace : nullptr,
                                   static_cast<hipStream_t>(stream));
}

int loma_decode_attn_gqa_layers(const void* const* q, const void* const* k_new, const void* const* v_new,
                                const void* const* k_memcache, const void* const* v_memcache,
                                void* const* k_read, void* const* v_read, void* const* out,
                                int n_layers, int B, int H, int H_kv, int head_dim, int t, int c,
                                int n_mem_chunks, int mem_capacity, int read_fill,
                                float scale, int dtype,
                                void* workspace, size_t workspace_bytes, void* stream) {
    if (n_layers < 1) return LOMA_ERR_INVALID_ARG;
    if ((k_new == nullptr) != (v_new == nullptr)) return LOMA_ERR_INVALID_ARG;
    if (!good_gqa_heads(H, H_kv)) return LOMA_ERR_INVALID_ARG;
    const bool has_new = k_new != nullptr;
    long long n_mem_keys = 0;
    if (int rc = check_decode_state(B, H_kv, head_dim, t, c, n_mem_chunks, mem_capacity, read_fill, has_new, scale, dtype,
                                    &n_mem_keys))
        return rc;
    auto good_table = [](const void* p) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 7u) == 0; };
    if (!good_table(q) || !good_table(out) || !good_table(k_read) || !good_table(v_read)) return LOMA_ERR_INVALID_ARG;
    if (has_new && (!good_table(k_new) || !good_table(v_new))) return LOMA_ERR_INVALID_ARG;
    if (n_mem_chunks > 0 && (!good_table(k_memcache) || !good_table(v_memcache))) return LOMA_ERR_INVALID_ARG;
    const int G = H / H_kv;
    if (G != 1 && G != 2 && G != 4 && G != 8) return LOMA_ERR_UNSUPPORTED;
    if (!loma::use_mfma_path(dtype, head_dim)) return LOMA_ERR_UNSUPPORTED;
    if ((long long)B * H_kv > 65535 || n_layers > 65535) return LOMA_ERR_UNSUPPORTED;
    const int nbh_kv = B * H_kv;
    const size_t need = (size_t)n_layers * loma::decode_gqa_workspace_bytes(nbh_kv, G, head_dim);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned16(workspace))) return LOMA_ERR_WORKSPACE;
    const void* const* tables[8] = {q, k_new, v_new, k_memcache, v_memcache,
                                    const_cast<const void* const*>(k_read), const_cast<const void* const*>(v_read),
                                    const_cast<const void* const*>(out)};
    return loma::launch_decode_gqa_layers(tables, has_new, n_layers, nbh_kv, G, head_dim, t * c, (int)n_mem_keys, mem_capacity,
                                          read_fill, scale, need > 0 ? workspace : nullptr, static_cast<hipStream_t>(stream));
}

size_t loma_decode_static_scratch_bytes(void) { return loma::decode_static_scratch_bytes(); }

size_t loma_decode_layers_workspace_bytes(int n_layers, int B, int H, int head_dim, int t, int c,
                                          int n_mem_chunks, int dtype) {
    if (n_layers < 1) return 0;
    return (size_t)n_layers * loma_decode_workspace_bytes(B, H, head_dim, t, c, n_mem_chunks, dtype);
}

int loma_decode_attn_layers(const void* const* q, const void* const* k_new, const void* const* v_new,
                            const void* const* k_memcache, const void* const* v_memcache,
                            void* const* k_read, void* const* v_read, void* const* out,
                            int n_layers, int B, int H, int head_dim, int t, int c,
                            int n_mem_chunks, int mem_capacity, int read_fill,
                            float scale, int dtype,
                            void* workspace, size_t workspace_bytes, void* stream) {
    if (n_layers < 1) return LOMA_ERR_INVALID_ARG;
    if ((k_new == nullptr) != (v_new == nullptr)) return LOMA_ERR_INVALID_ARG;
    const bool has_new = k_new != nullptr;
    long long n_mem_keys = 0;
    if (int rc = check_decode_state(B, H, head_dim, t, c, n_mem_chunks, mem_capacity, read_fill, has_new, scale, dtype,
                                    &n_mem_keys))
        return rc;
    auto good_table = [](const void* p) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 7u) == 0; };
    if (!good_table(q) || !good_table(out) || !good_table(k_read) || !good_table(v_read)) return LOMA_ERR_INVALID_ARG;
    if (has_new && (!good_table(k_new) || !good_table(v_new))) return LOMA_ERR_INVALID_ARG;
    if (n_mem_chunks > 0 && (!good_table(k_memcache) || !good_table(v_memcache))) return LOMA_ERR_INVALID_ARG;
    if (!loma::use_mfma_path(dtype, head_dim)) return LOMA_ERR_UNSUPPORTED;
    const int nbh = B * H, R = t * c;
    if (nbh > 65535 || n_layers > 65535) return LOMA_ERR_UNSUPPORTED;
    const size_t need = (size_t)n_layers * loma::decode_workspace_bytes(nbh, head_dim, (int)n_mem_keys + R);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned16(workspace))) return LOMA_ERR_WORKSPACE;
    const void* const* tables[8] = {q, k_new, v_new, k_memcache, v_memcache,
                                    const_cast<const void* const*>(k_read), const_cast<const void* const*>(v_read),
                                    const_cast<const void* const*>(out)};
    return loma::launch_decode_splitk_layers(tables, has_new, n_layers, nbh, head_dim, R, (int)n_mem_keys, mem_capacity,
                                             read_fill, scale, need > 0 ? workspace : nullptr,
                                             static_cast<hipStream_t>(stream));
}

int loma_prefill_attn(const void* q, const void* k_new, const void* v_new,
                      const void* k_memcache, const void* v_memcache,
                      void* k_read, void* v_read, void* out, float* lse,
                      int B, int H, int head_dim, int t, int c,
                      int n_mem_chunks, int mem_capacity, int read_fill, int n_new,
                      float scale, int dtype, void* stream) {
    if (int rc = check_common(B, H, head_dim, t, c, scale, dtype)) return rc;
    const int R = t * c;
    if (n_mem_chunks < 0 || mem_capacity < 0 || read_fill < 0 || n_new < 1) return LOMA_ERR_INVALID_ARG;
    const long long n_mem_keys = (long long)n_mem_chunks * t;
    if (n_mem_keys > mem_capacity || n_mem_keys > 0x3fffffffLL) return LOMA_ERR_INVALID_ARG;
    if ((long long)read_fill + n_new > R) return LOMA_ERR_INVALID_ARG;
    if (!good_ptr(q) || !good_ptr(k_new) || !good_ptr(v_new) || !good_ptr(out) || !good_ptr(k_read) || !good_ptr(v_read))
        return LOMA_ERR_INVALID_ARG;
    if (n_mem_chunks > 0 && (!good_ptr(k_memcache) || !good_ptr(v_memcache))) return LOMA_ERR_INVALID_ARG;
    if (lse != nullptr && (reinterpret_cast<uintptr_t>(lse) & 3u)) return LOMA_ERR_INVALID_ARG;
    const int nbh = B * H;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (loma::use_mfma_path(dtype, head_dim))
        return loma::launch_prefill_mfma(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, lse, nbh,
                                         head_dim, R, (int)n_mem_keys, mem_capacity, read_fill, n_new, scale, st);
    return loma::launch_prefill_generic(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, lse, nbh,
                                        head_dim, R, (int)n_mem_keys, mem_capacity, read_fill, n_new, scale, dtype, st);
}

long long loma_mask_schedule_size(int B, int H, int head_dim, int t, int c, int n_chunks, int dtype) {
    if (check_common(B, H, head_dim, t, c, 1.f, dtype) != LOMA_OK || n_chunks < 1) return 0;
    if (!loma::use_mfma_path(dtype, head_dim)) return 0;
    const long long S = (long long)n_chunks * t * (2 * c + 1);
    if (S > (1LL << 30)) return 0;
    Geometry g;
    g.t = t; g.c = c; g.n = n_chunks; g.R = t * c; g.s = t * (2 * c + 1); g.S = (int)S;
    if (!loma::mask_attn_mfma_fits(g)) return 0;
    return loma::MaskSchedule::make(B * H, t, c, n_chunks, loma::mask_block_rows(t * c, t)).size();
}

int loma_mask_schedule_item(int B, int H, int head_dim, int t, int c, int n_chunks, int dtype,
                            long long block, int item[6]) {
    if (int rc = check_common(B, H, head_dim, t, c, 1.f, dtype)) return rc;
    if (n_chunks < 1 || item == nullptr) return LOMA_ERR_INVALID_ARG;
    if (!loma::use_mfma_path(dtype, head_dim)) return LOMA_ERR_UNSUPPORTED;
    const loma::MaskSchedule sch = loma::MaskSchedule::make(B * H, t, c, n_chunks, loma::mask_block_rows(t * c, t));
    if (block < 0 || block >= sch.size()) return LOMA_ERR_INVALID_ARG;
    const loma::MaskJob j = sch.decode(block);
    item[0] = j.bh; item[1] = j.y; item[2] = j.zone; item[3] = j.o0; item[4] = j.rows; item[5] = j.nkeys;
    return 1;
}

}  // extern "C"
