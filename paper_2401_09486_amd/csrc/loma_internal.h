// Internal declarations shared by the translation units of libloma (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/loma.h"

namespace loma {

// Geometry of a restructured sample (Sec. 4.1): chunk = [R reading | t memory | R repetition].
struct Geometry {
    int t, c, n;
    int R;  // t*c
    int s;  // t*(2c+1)
    int S;  // n*s
};

enum Zone : int { ZONE_READ = 0, ZONE_MEM = 1, ZONE_REP = 2 };

// One workgroup's share of the mask pass: `rows` query rows of one zone of one chunk.
struct MaskJob {
    int bh;     // b*H + h
    int y;      // chunk
    int zone;   // Zone
    int o0;     // first row inside the zone
    int rows;   // rows handled (<= block rows)
    int nkeys;  // keys this workgroup walks over (visible to its last row)
};

// Tile-schedule arithmetic, identical on host (tests, grid sizing) and device (job decode).
// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  With B*H a multiple of 8
// workgroup id -> XCD id % 8, and every XCD walks its own (b,h) pairs ONE AFTER THE OTHER, so
// the memory-zone K/V of a (b,h), re-read by every later chunk, stays in that L2 (about 1 MB
// per (b,h) at the long-context shape, against 4 MB of L2).  Inside a (b,h): chunk-major from
// the last chunk to the first (reading blocks of late chunks see the most keys: longest
// first), and within a chunk reading blocks, memory blocks, repetition blocks side by side,
// so the MFMA-heavy reading blocks and the HBM-heavy repetition blocks share the CUs.
struct MaskSchedule {
    int nbh, n, t, R, s, bm;
    int nRB, nMB;        // row blocks per reading (= repetition) zone, per memory zone
    int jobs_per_chunk, jobs_per_bh;

    __host__ __device__ static MaskSchedule make(int nbh, int t, int c, int n, int bm) {
        MaskSchedule m;
        m.nbh = nbh; m.n = n; m.t = t; m.R = t * c; m.s = t * (2 * c + 1); m.bm = bm;
        m.nRB = (m.R + bm - 1) / bm;
        m.nMB = (t + bm - 1) / bm;
        m.jobs_per_chunk = 2 * m.nRB + m.nMB;
        m.jobs_per_bh = n * m.jobs_per_chunk;
        return m;
    }
    __host__ __device__ long long size() const { return (long long)nbh * jobs_per_bh; }

    __host__ __device__ MaskJob decode(long long id) const {
        MaskJob j;
        int w;
        if (nbh % 8 == 0) {
            const int xcd = (int)(id % 8);
            const long long k = id / 8;
            j.bh = xcd + 8 * (int)(k / jobs_per_bh);
            w = (int)(k % jobs_per_bh);
        } else {
            j.bh = (int)(id % nbh);
            w = (int)(id / nbh);
        }
        j.y = n - 1 - w / jobs_per_chunk;
        int u = w % jobs_per_chunk;
        if (u < nRB) {
            j.zone = ZONE_READ;
            j.o0 = (nRB - 1 - u) * bm;
            j.rows = (R - j.o0 < bm) ? R - j.o0 : bm;
            j.nkeys = j.y * t + j.o0 + j.rows;
        } else if (u < nRB + nMB) {
            u -= nRB;
            j.zone = ZONE_MEM;
            j.o0 = u * bm;
            j.rows = (t - j.o0 < bm) ? t - j.o0 : bm;
            j.nkeys = R + t;
        } else {
            u -= nRB + nMB;
            j.zone = ZONE_REP;
            j.o0 = u * bm;
            j.rows = (R - j.o0 < bm) ? R - j.o0 : bm;
            j.nkeys = t;  // + the row itself, handled outside the key walk
        }
        return j;
    }
};

// Rows per workgroup of the MFMA mask-pass kernels for a reading zone of R rows and a memory zone of t rows.
inline int mask_block_rows(int R, int t) { (void)t; return R >= 128 ? 128 : (R >= 64 ? 64 : 32); }
// Rows per workgroup of the gradient kernels.
inline int mask_bwd_block_rows(int R) { return R >= 128 ? 128 : (R >= 64 ? 64 : 32); }

inline bool use_mfma_path(int dtype, int head_dim) {
    return dtype == LOMA_BF16 && (head_dim == 64 || head_dim == 128);
}

// The MFMA mask-pass kernels find the chunk of memory key j (j < (n-1)*t) with a multiply-high by
// floor(2^32 / t) + 1, which is exact only while j * t < 2^32; longer samples take the generic kernels.
inline bool mask_attn_mfma_fits(const Geometry& g) {
    return (unsigned long long)(g.n - 1) * (unsigned long long)g.t * (unsigned long long)g.t < (1ULL << 32);
}

// ---- launchers (each returns LOMA_OK or LOMA_ERR_LAUNCH) -----------------------------------
int launch_mask_attn_mfma(const void* q, const void* k, const void* v, void* out, float* lse,
                          int nbh, int D, const Geometry& g, float scale, hipStream_t st);
int launch_compress_mfma(const void* q_mem, const void* k_mem, const void* v_mem,
                         const void* k_read, const void* v_read, void* k_memcache, void* v_memcache,
                         void* out, int nbh, int D, int t, int c, int n_mem_chunks, int mem_capacity,
                         float scale, hipStream_t st, const struct RopeTable* rope = nullptr);

int launch_mask_attn_generic(const void* q, const void* k, const void* v, void* out, float* lse,
                             int nbh, int D, const Geometry& g, float scale, int dtype, hipStream_t st);
int launch_compress_generic(const void* q_mem, const void* k_mem, const void* v_mem,
                            const void* k_read, const void* v_read, void* k_memcache, void* v_memcache,
                            void* out, int nbh, int D, int t, int c, int n_mem_chunks, int mem_capacity,
                            float scale, int dtype, hipStream_t st);
int launch_decode_generic(const void* q, const void* k_new, const void* v_new,
                          const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                          void* out, int nbh, int D, int R, int n_mem_keys, int mem_capacity, int read_fill,
                          float scale, int dtype, hipStream_t st);

// Gradients of the mask pass; the caller's workspace holds two floats per row (the generic kernels use the first nbh*S).
int launch_mask_attn_bwd_generic(const void* q, const void* k, const void* v, const void* out, const float* lse,
                                 const void* dout, void* dq, void* dk, void* dv, float* delta,
                                 int nbh, int D, const Geometry& g, float scale, int dtype, hipStream_t st);

bool mask_attn_bwd_mfma_fits(const Geometry& g);
size_t mask_attn_bwd_mfma_workspace_floats(int nbh, int D, const Geometry& g);   // what `workspace` below must hold
int launch_mask_attn_bwd_mfma(const void* q, const void* k, const void* v, const void* out, const float* lse,
                              const void* dout, void* dq, void* dk, void* dv, float* workspace,
                              int nbh, int D, const Geometry& g, float scale, hipStream_t st);

// Several new tokens against the cache: memory keys and live reading rows in full, new tokens causally.
int launch_prefill_mfma(const void* q, const void* k_new, const void* v_new,
                        const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                        void* out, float* lse, int nbh, int D, int R, int n_mem_keys, int mem_capacity,
                        int read_fill, int n_new, float scale, hipStream_t st);
int launch_prefill_generic(const void* q, const void* k_new, const void* v_new,
                           const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                           void* out, float* lse, int nbh, int D, int R, int n_mem_keys, int mem_capacity,
                           int read_fill, int n_new, float scale, int dtype, hipStream_t st);

// Split-K decode over [memory cache || reading zone || new token].
int decode_num_splits(int nbh, int n_keys);
size_t decode_workspace_bytes(int nbh, int D, int n_keys_max);
struct RopeTable;   // loma_rope.h: rotary frequencies and the position ids of the rows to rotate; nullptr = no rotation
int launch_decode_splitk(const void* q, const void* k_new, const void* v_new,
                         const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                         void* out, int nbh, int D, int R, int n_mem_keys, int mem_capacity, int read_fill,
                         float scale, void* workspace, hipStream_t st, const RopeTable* rope = nullptr);

// The same for n_layers independent caches in ONE launch: tables[i] is a DEVICE array of n_layers device pointers
// (q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out); shapes and cache state are shared by the layers.
// The workspace holds n_layers blocks of decode_workspace_bytes() each.
int launch_decode_splitk_layers(const void* const* tables[8], bool has_new, int n_layers, int nbh, int D, int R,
                                int n_mem_keys, int mem_capacity, int read_fill, float scale, void* workspace,
                                hipStream_t st);
// Grouped-query decode: G = H / H_kv consecutive query heads share a KV head (G in {1, 2, 4, 8}); q and out hold
// nbh_kv * G rows, every cache tensor nbh_kv sequences.  The workspace holds decode_gqa_workspace_bytes().
size_t decode_gqa_workspace_bytes(int nbh_kv, int G, int D);
int launch_decode_gqa(const void* q, const void* k_new, const void* v_new,
                      const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                      void* out, int nbh_kv, int G, int D, int R, int n_mem_keys, int mem_capacity, int read_fill,
                      float scale, void* workspace, hipStream_t st);
// ... and for n_layers caches in one launch (pointer tables as in launch_decode_splitk_layers; the workspace holds n_layers
// blocks of decode_gqa_workspace_bytes() each)
int launch_decode_gqa_layers(const void* const* tables[8], bool has_new, int n_layers, int nbh_kv, int G, int D, int R,
                             int n_mem_keys, int mem_capacity, int read_fill, float scale, void* workspace, hipStream_t st);
// Fixed split-K scratch inside the library's device image (for callers that cannot allocate): its size, and its
// address on the current device (nullptr if the runtime cannot resolve it).
size_t decode_static_scratch_bytes();
void* decode_static_scratch_ptr();

}  // namespace loma
