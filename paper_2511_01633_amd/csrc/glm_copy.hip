// Block copies driven by the cache manager: copy-on-write of a partly filled block when a
// branch forks, and whole-block gather for eviction to a staging area / re-admission.
// Both are pure HBM traffic: 16-byte vector loads and stores, several in flight per lane.
#include <algorithm>
#include <vector>

#include "glm_internal.h"

namespace glm {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 256;
constexpr int kCopyUnroll = 4;                                   // 16-byte pieces in flight per thread
constexpr int kCopySpan = kCopyThreads * kCopyUnroll;            // pieces one workgroup moves

// grid = (ceil(pieces_per_block / kCopySpan), n)
__global__ void __launch_bounds__(kCopyThreads) gather_kernel(const u32x4 *__restrict__ src, const int32_t *__restrict__ src_ids,
                                                              u32x4 *__restrict__ dst, const int32_t *__restrict__ dst_ids,
                                                              int64_t pieces_per_block) {
    const int k = blockIdx.y;
    const int64_t s = src_ids ? src_ids[k] : k;
    const int64_t d = dst_ids ? dst_ids[k] : k;
    const u32x4 *sp = src + s * pieces_per_block;
    u32x4 *dp = dst + d * pieces_per_block;
    const int64_t base = (int64_t)blockIdx.x * kCopySpan + threadIdx.x;
    u32x4 v[kCopyUnroll];
#pragma unroll
    for (int i = 0; i < kCopyUnroll; ++i) {
        const int64_t p = base + (int64_t)i * kCopyThreads;
        if (p < pieces_per_block) v[i] = __builtin_nontemporal_load(sp + p);
    }
#pragma unroll
    for (int i = 0; i < kCopyUnroll; ++i) {
        const int64_t p = base + (int64_t)i * kCopyThreads;
        if (p < pieces_per_block) __builtin_nontemporal_store(v[i], dp + p);
    }
}

// grid = (2 * Hkv, n_pairs): one workgroup copies the first n_tokens rows of one (plane, kv head).
// A row is row_pieces 16-byte pieces and the rows of a (plane, head) slab are contiguous.
__global__ void __launch_bounds__(kCopyThreads) fork_copy_kernel(u32x4 *__restrict__ pool, const int32_t *__restrict__ src_ids,
                                                                 const int32_t *__restrict__ dst_ids,
                                                                 const int32_t *__restrict__ n_tokens, int row_pieces,
                                                                 int64_t pieces_per_block, int num_blocks) {
    const int k = blockIdx.y;
    const int n = min(max(n_tokens[k], 0), kBlockSize);
    const int64_t s = min(max(src_ids[k], 0), num_blocks - 1);
    const int64_t d = min(max(dst_ids[k], 0), num_blocks - 1);
    const int64_t slab = (int64_t)blockIdx.x * kBlockSize * row_pieces;
    const u32x4 *sp = pool + s * pieces_per_block + slab;
    u32x4 *dp = pool + d * pieces_per_block + slab;
    const int total = n * row_pieces;
    for (int p = threadIdx.x; p < total; p += kCopyThreads) dp[p] = sp[p];
}

// grid = n_tokens: one workgroup scatters one token's K and V rows (2 * Hkv * row_pieces 16-byte pieces)
// to its slot; piece p = (plane, head, c) goes to block + (plane*Hkv + head) * slab + offset * row + c.
__global__ void __launch_bounds__(kCopyThreads) append_kernel(u32x4 *__restrict__ pool, const u32x4 *__restrict__ k_new,
                                                              const u32x4 *__restrict__ v_new,
                                                              const int64_t *__restrict__ slots, int hkv, int row_pieces,
                                                              int64_t pieces_per_block, int64_t num_slots) {
    const int64_t tok = blockIdx.x;
    const int64_t slot = slots[tok];
    if (slot < 0 || slot >= num_slots) return;                    // padding, or out of range: never write outside the pool
    const int64_t blk = slot / kBlockSize;
    const int off = (int)(slot % kBlockSize);
    const int per_plane = hkv * row_pieces;
    for (int p = threadIdx.x; p < 2 * per_plane; p += kCopyThreads) {
        const int plane = p / per_plane, q = p % per_plane;
        const int head = q / row_pieces, c = q % row_pieces;
        const u32x4 v = (plane ? v_new : k_new)[tok * per_plane + q];
        pool[blk * pieces_per_block + ((int64_t)(plane * hkv + head) * kBlockSize + off) * row_pieces + c] = v;
    }
}

// grid = (ceil(max_seq_len / 16), B): one workgroup moves one logical block of one request; a (plane, head) slab
// of n rows is contiguous both in the block and in the request's dense [2][Hkv][L][d] slab.
__global__ void __launch_bounds__(kCopyThreads) gather_tokens_kernel(const u32x4 *__restrict__ pool, const int32_t *__restrict__ tables,
                                                                     const int32_t *__restrict__ seq_lens,
                                                                     const int64_t *__restrict__ dst_offsets, u32x4 *__restrict__ dst,
                                                                     int max_blocks, int hkv, int row_pieces, int num_blocks) {
    const int r = blockIdx.y, b = blockIdx.x;
    const int64_t L = min(max(seq_lens[r], 0), max_blocks * kBlockSize);
    const int rows = (int)min((int64_t)kBlockSize, L - (int64_t)b * kBlockSize);
    if (rows <= 0) return;
    const int id = min(max(tables[(int64_t)r * max_blocks + b], 0), num_blocks - 1);     // never reads outside the pool
    const int slab = kBlockSize * row_pieces;                       // pieces of one (plane, head) slab of a block
    const u32x4 *sp = pool + (int64_t)id * 2 * hkv * slab;
    u32x4 *dp = dst + dst_offsets[r] / 8;
    const int n = rows * row_pieces;
    for (int ph = 0; ph < 2 * hkv; ++ph) {
        u32x4 *d = dp + ((int64_t)ph * L + (int64_t)b * kBlockSize) * row_pieces;
        const u32x4 *sph = sp + (int64_t)ph * slab;
        for (int p = threadIdx.x; p < n; p += kCopyThreads) d[p] = sph[p];
    }
}

namespace {

int validate_ids(const int32_t *ids_dev, int32_t n, int64_t upper, bool distinct, std::vector<int32_t> *keep,
                 hipStream_t st) {
    if (!ids_dev) return GLM_OK;
    try {
        std::vector<int32_t> h(n);
        hipError_t e = hipStreamSynchronize(st);
        if (e == hipSuccess) e = hipMemcpy(h.data(), ids_dev, (size_t)n * 4, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return set_hip_error(e);
        for (int32_t v : h)
            if (v < 0 || (upper >= 0 && v >= upper)) return GLM_ERR_RANGE;
        if (keep) *keep = h;
        if (distinct) {
            std::sort(h.begin(), h.end());
            if (std::adjacent_find(h.begin(), h.end()) != h.end()) return GLM_ERR_RANGE;
        }
    } catch (...) {
        return GLM_ERR_ALLOC;
    }
    return GLM_OK;
}

}  // namespace
}  // namespace glm

using namespace glm;

extern "C" {

int glm_kv_gather(glm_geom g, const void *src_base_dev, const int32_t *src_ids_dev, void *dst_base_dev,
                  const int32_t *dst_ids_dev, int32_t n, void *hip_stream) {
    if (int st = check_geom(g)) return st;
    if (n < 0) return GLM_ERR_GEOM;
    if (n == 0) return GLM_OK;
    if (!src_base_dev || !dst_base_dev) return GLM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(src_base_dev) | reinterpret_cast<uintptr_t>(dst_base_dev)) & 15u) return GLM_ERR_ALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    if (validate_enabled()) {
        if (int v = validate_ids(src_ids_dev, n, -1, false, nullptr, st)) return v;
        if (int v = validate_ids(dst_ids_dev, n, -1, true, nullptr, st)) return v;
    }
    const int64_t pieces = 2LL * g.num_kv_heads * g.block_size * g.head_dim * 2 / 16;
    const int gx = (int)((pieces + kCopySpan - 1) / kCopySpan);
    for (int32_t done = 0; done < n; done += 65535) {             // grid.y limit
        const int32_t cnt = std::min<int32_t>(65535, n - done);
        const int64_t off_s = src_ids_dev ? 0 : (int64_t)done * pieces;
        const int64_t off_d = dst_ids_dev ? 0 : (int64_t)done * pieces;
        ProfileScope prof(kKernelGather, st);
        hipLaunchKernelGGL(gather_kernel, dim3(gx, cnt), dim3(kCopyThreads), 0, st,
                           (const u32x4 *)src_base_dev + off_s, src_ids_dev ? src_ids_dev + done : nullptr,
                           (u32x4 *)dst_base_dev + off_d, dst_ids_dev ? dst_ids_dev + done : nullptr, pieces);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return set_hip_error(e);
    }
    return GLM_OK;
}

int glm_kv_fork_copy(glm_geom g, void *kv_pool_dev, const int32_t *src_ids_dev, const int32_t *dst_ids_dev,
                     const int32_t *n_tokens_dev, int32_t n_pairs, void *hip_stream) {
    if (int st = check_geom(g)) return st;
    if (n_pairs < 0) return GLM_ERR_GEOM;
    if (n_pairs == 0) return GLM_OK;
    if (!kv_pool_dev || !src_ids_dev || !dst_ids_dev || !n_tokens_dev) return GLM_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(kv_pool_dev) & 15u) return GLM_ERR_ALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    if (validate_enabled()) {
        std::vector<int32_t> src, dst;
        if (int v = validate_ids(src_ids_dev, n_pairs, g.num_blocks, false, &src, st)) return v;
        if (int v = validate_ids(dst_ids_dev, n_pairs, g.num_blocks, true, &dst, st)) return v;
        if (int v = validate_ids(n_tokens_dev, n_pairs, g.block_size + 1, false, nullptr, st)) return v;
        std::sort(src.begin(), src.end());
        for (int32_t d : dst)
            if (std::binary_search(src.begin(), src.end(), d)) return GLM_ERR_RANGE;
    }
    const int row_pieces = g.head_dim * 2 / 16;
    const int64_t pieces = 2LL * g.num_kv_heads * g.block_size * row_pieces;
    for (int32_t done = 0; done < n_pairs; done += 65535) {
        const int32_t cnt = std::min<int32_t>(65535, n_pairs - done);
        ProfileScope prof(kKernelFork, st);
        hipLaunchKernelGGL(fork_copy_kernel, dim3(2 * g.num_kv_heads, cnt), dim3(kCopyThreads), 0, st,
                           (u32x4 *)kv_pool_dev, src_ids_dev + done, dst_ids_dev + done, n_tokens_dev + done, row_pieces,
                           pieces, g.num_blocks);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return set_hip_error(e);
    }
    return GLM_OK;
}

}  // extern "C"

extern "C" int glm_kv_append(glm_geom g, void *kv_pool_dev, const void *k_new_dev, const void *v_new_dev,
                             const int64_t *slot_mapping_dev, int32_t n_tokens, void *hip_stream) {
    if (int st = check_geom(g)) return st;
    if (n_tokens < 0) return GLM_ERR_GEOM;
    if (n_tokens == 0) return GLM_OK;
    if (!kv_pool_dev || !k_new_dev || !v_new_dev || !slot_mapping_dev) return GLM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(kv_pool_dev) | reinterpret_cast<uintptr_t>(k_new_dev) |
         reinterpret_cast<uintptr_t>(v_new_dev)) & 15u)
        return GLM_ERR_ALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t num_slots = (int64_t)g.num_blocks * g.block_size;
    if (validate_enabled()) {
        try {
            std::vector<int64_t> h(n_tokens);
            hipError_t e = hipStreamSynchronize(st);
            if (e == hipSuccess) e = hipMemcpy(h.data(), slot_mapping_dev, (size_t)n_tokens * 8, hipMemcpyDeviceToHost);
            if (e != hipSuccess) return set_hip_error(e);
            std::vector<int64_t> used;
            for (int64_t v : h) {
                if (v >= num_slots) return GLM_ERR_RANGE;
                if (v >= 0) used.push_back(v);
            }
            std::sort(used.begin(), used.end());
            if (std::adjacent_find(used.begin(), used.end()) != used.end()) return GLM_ERR_RANGE;
        } catch (...) {
            return GLM_ERR_ALLOC;
        }
    }
    const int row_pieces = g.head_dim * 2 / 16;
    const int64_t pieces = 2LL * g.num_kv_heads * g.block_size * row_pieces;
    ProfileScope prof(kKernelAppend, st);
    hipLaunchKernelGGL(append_kernel, dim3(n_tokens), dim3(kCopyThreads), 0, st, (u32x4 *)kv_pool_dev,
                       (const u32x4 *)k_new_dev, (const u32x4 *)v_new_dev, slot_mapping_dev, g.num_kv_heads, row_pieces,
                       pieces, num_slots);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? GLM_OK : set_hip_error(e);
}

extern "C" int glm_kv_gather_tokens(glm_geom g, const void *kv_pool_dev, const int32_t *block_tables_dev, int32_t max_blocks,
                                    const int32_t *seq_lens_dev, const int64_t *dst_offsets_dev, int32_t B, int32_t max_seq_len,
                                    void *dst_dev, void *hip_stream) {
    if (int st = check_geom(g)) return st;
    if (B < 0 || max_blocks <= 0 || max_seq_len < 0) return GLM_ERR_GEOM;
    if (B == 0 || max_seq_len == 0) return GLM_OK;
    if (!kv_pool_dev || !block_tables_dev || !seq_lens_dev || !dst_offsets_dev || !dst_dev) return GLM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(kv_pool_dev) | reinterpret_cast<uintptr_t>(dst_dev)) & 15u) return GLM_ERR_ALIGN;
    if (B > 65535) return GLM_ERR_GEOM;                       // grid.y
    hipStream_t st = (hipStream_t)hip_stream;
    if (validate_enabled()) {
        try {
            std::vector<int32_t> lens(B), tab((size_t)B * max_blocks);
            std::vector<int64_t> offs(B);
            hipError_t e = hipStreamSynchronize(st);
            if (e == hipSuccess) e = hipMemcpy(lens.data(), seq_lens_dev, (size_t)B * 4, hipMemcpyDeviceToHost);
            if (e == hipSuccess) e = hipMemcpy(tab.data(), block_tables_dev, tab.size() * 4, hipMemcpyDeviceToHost);
            if (e == hipSuccess) e = hipMemcpy(offs.data(), dst_offsets_dev, (size_t)B * 8, hipMemcpyDeviceToHost);
            if (e != hipSuccess) return set_hip_error(e);
            for (int32_t r = 0; r < B; ++r) {
                if (lens[r] < 0 || lens[r] > max_seq_len || (int64_t)lens[r] > (int64_t)max_blocks * g.block_size) return GLM_ERR_RANGE;
                if (offs[r] < 0 || (offs[r] & 7)) return GLM_ERR_RANGE;
                for (int32_t b = 0; b < (lens[r] + g.block_size - 1) / g.block_size; ++b) {
                    const int32_t id = tab[(size_t)r * max_blocks + b];
                    if (id < 0 || id >= g.num_blocks) return GLM_ERR_RANGE;
                }
            }
        } catch (...) {
            return GLM_ERR_ALLOC;
        }
    }
    const int nb = std::min((max_seq_len + g.block_size - 1) / g.block_size, max_blocks);
    ProfileScope prof(kKernelGatherTokens, st);
    hipLaunchKernelGGL(gather_tokens_kernel, dim3(nb, B), dim3(kCopyThreads), 0, st, (const u32x4 *)kv_pool_dev, block_tables_dev,
                       seq_lens_dev, dst_offsets_dev, (u32x4 *)dst_dev, max_blocks, g.num_kv_heads, g.head_dim * 2 / 16,
                       g.num_blocks);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? GLM_OK : set_hip_error(e);
}
