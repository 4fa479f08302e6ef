// Store side and bulk copies of the unified pool:
//   append_kernel : scatters each request's new K/V token into its pages and writes the call's new
//                   page-table entries;  patch_kernel : page-table entries alone (used when a token
//                   spans more than four pages);
//   copy_tokens_kernel : paged <-> contiguous copy of whole requests (gather / scatter);
//   stage_copy_kernel : uploads a call's plan from pinned host memory.
#include "ukv_device.h"

namespace ukv {

__global__ void patch_kernel(int32_t *page_table, const uint64_t *entry, const int32_t *page, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        page_table[entry[i]] = page[i];
}

// Opt-in check (UKV_PARAM_VALIDATE): every table entry a call is about to use must name a page of the pool.  One
// workgroup per request; the first bad entry found is reported in pinned host memory, and its flag makes the call's
// compute kernels leave at once.  The check only reads the table.
__global__ void __launch_bounds__(256) validate_kernel(const int32_t *page_table, const ValRec *recs, uint64_t n_pages,
                                                       ValReport *report, uint32_t *flag_dev) {
    const ValRec r = recs[blockIdx.x];
    for (uint64_t e = threadIdx.x; e < r.n_entries; e += blockDim.x) {
        const int64_t pg = page_table[r.table_off + e];
        if (pg < 0 || (uint64_t)pg >= n_pages) {
            *flag_dev = 1u; // what the kernels of this and later calls read, until the host has reported
            if (atomicCAS_system(&report->bad, 0u, 1u) == 0u) { // the first one to find something describes it
                report->req = r.req;
                report->entry = r.table_off + e;
                report->page = pg;
            }
        }
    }
}

// The flag of that check (device memory), read by the kernels of the checked call: one load per workgroup.
__device__ __forceinline__ bool tables_bad(const uint32_t *bad) {
    return bad != nullptr && *reinterpret_cast<const volatile uint32_t *>(bad) != 0;
}

// Workgroups [0, n_requests): one per request; each lane moves 16-byte pieces of the new token
// row.  Page ids of table entries that are being patched in the same call come with the record
// (r.page[k] >= 0 for the k-th page the token touches), so no workgroup reads an entry another one
// is writing.  Workgroups [n_requests, ...): write the patched page-table entries.
__global__ void __launch_bounds__(256) append_kernel(unsigned char *pool_base, uint32_t lg, int32_t *page_table,
                                                     const AppendRec *recs, uint32_t n_requests,
                                                     const ClassRec *classes, const uint16_t *new_k,
                                                     const uint16_t *new_v, const uint64_t *patch_entry,
                                                     const int32_t *patch_page, uint32_t n_patches,
                                                     const uint32_t *bad) {
    if (tables_bad(bad))
        return;
    if (blockIdx.x >= n_requests) {
        const uint32_t i = (blockIdx.x - n_requests) * blockDim.x + threadIdx.x;
        if (i < n_patches)
            page_table[patch_entry[i]] = patch_page[i];
        return;
    }
    const AppendRec r = recs[blockIdx.x];
    if (r.ctx_len == 0)
        return;
    const ClassRec c = classes[r.cls];
    const uint32_t pieces_per_row = c.row_bytes / 16, half = pieces_per_row / 2;
    const uint32_t n_pieces = c.token_bytes / 16;
    const uint64_t stream0 = (uint64_t)(r.ctx_len - 1) * c.token_bytes;
    const uint64_t first_slot = stream0 >> lg;
    const uint64_t page_mask = (1ull << lg) - 1;
    for (uint32_t pc = threadIdx.x; pc < n_pieces; pc += blockDim.x) {
        const uint32_t h = pc / pieces_per_row, w = pc % pieces_per_row;
        const uint16_t *src = (w < half ? new_k : new_v) + r.new_off + (uint64_t)h * c.d + (w % half) * 8;
        const uint64_t off = stream0 + (uint64_t)pc * 16;
        const uint64_t slot = off >> lg;
        const uint32_t k = (uint32_t)(slot - first_slot);
        int32_t pg = k < 4 ? r.page[k] : -1;
        if (pg < 0)
            pg = page_table[r.table_off + slot];
        uint4 *dst = reinterpret_cast<uint4 *>(pool_base + ((uint64_t)(uint32_t)pg << lg) + (off & page_mask));
        *dst = *reinterpret_cast<const uint4 *>(src);
    }
}

// Paged <-> contiguous copy.  One workgroup per record = tokens [t0, t1) of one request (the
// host cuts requests into chunks of about 1 MiB); the (token, 16-byte piece) pairs of the chunk
// are spread over the lanes, four in flight per lane.  TO_POOL = false gathers (pool ->
// k_io/v_io), true scatters (k_io/v_io -> pool).
template <bool TO_POOL>
__global__ void __launch_bounds__(256) copy_tokens_kernel(unsigned char *pool_base, uint32_t lg,
                                                          const int32_t *page_table, const GatherRec *recs,
                                                          const ClassRec *classes, uint16_t *k_io, uint16_t *v_io,
                                                          const uint32_t *bad) {
    if (tables_bad(bad))
        return;
    const GatherRec r = recs[blockIdx.x];
    const ClassRec c = classes[r.cls];
    const uint32_t pieces_per_row = c.row_bytes / 16, half = pieces_per_row / 2;
    const uint32_t n_pieces = c.token_bytes / 16;
    const uint64_t page_mask = (1ull << lg) - 1;
    const uint64_t total = (uint64_t)(r.t1 - r.t0) * n_pieces;
    auto addrs = [&](uint64_t idx, uint4 *&in_pool, uint4 *&flat) {
        const uint32_t t = r.t0 + (uint32_t)(idx / n_pieces), pc = (uint32_t)(idx % n_pieces);
        const uint32_t h = pc / pieces_per_row, w = pc % pieces_per_row;
        const uint64_t off = (uint64_t)t * c.token_bytes + (uint64_t)pc * 16;
        const int32_t pg = page_table[r.table_off + (off >> lg)];
        in_pool = reinterpret_cast<uint4 *>(pool_base + ((uint64_t)(uint32_t)pg << lg) + (off & page_mask));
        flat = reinterpret_cast<uint4 *>((w < half ? k_io : v_io) + r.kv_off + ((uint64_t)(t - r.flat_t0) * c.n_kv + h) * c.d +
                                         (w % half) * 8);
    };
    uint64_t idx = threadIdx.x;
    for (; idx + 3 * 256 < total; idx += 4 * 256) {
        uint4 *pp[4], *ff[4], x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            addrs(idx + u * 256, pp[u], ff[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            x[u] = TO_POOL ? *ff[u] : *pp[u];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            *(TO_POOL ? pp[u] : ff[u]) = x[u];
    }
    for (; idx < total; idx += 256) {
        uint4 *p1, *f1;
        addrs(idx, p1, f1);
        if (TO_POOL)
            *p1 = *f1;
        else
            *f1 = *p1;
    }
}

// Plan upload: copies 16-byte pieces from pinned, device-mapped host memory into the workspace.
// Workgroups past the copy write the step's new page-table entries (fused append), so that the
// decode launch that follows finds them in place.
__global__ void __launch_bounds__(256) stage_copy_kernel(uint4 *dst, const uint4 *src, uint32_t n16,
                                                         int32_t *page_table, const uint64_t *patch_entry,
                                                         const int32_t *patch_page, uint32_t n_patches) {
    const uint32_t copy_blocks = (n16 + 255) / 256;
    if (blockIdx.x >= copy_blocks) {
        const uint32_t i = (blockIdx.x - copy_blocks) * blockDim.x + threadIdx.x;
        if (i < n_patches)
            page_table[patch_entry[i]] = patch_page[i];
        return;
    }
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n16)
        dst[i] = src[i];
}

// ------------------------------------------------------------------ launchers
hipError_t launch_stage_copy(void *dst, const void *src_mapped, size_t bytes, int32_t *page_table,
                             const uint64_t *patch_entry, const int32_t *patch_page, uint32_t n_patches,
                             hipStream_t s) {
    const uint32_t n16 = (uint32_t)((bytes + 15) / 16);
    const uint32_t blocks = (n16 + 255) / 256 + (n_patches + 255) / 256;
    if (blocks == 0)
        return hipSuccess;
    hipLaunchKernelGGL(stage_copy_kernel, dim3(blocks), dim3(256), 0, s, static_cast<uint4 *>(dst),
                       static_cast<const uint4 *>(src_mapped), n16, page_table, patch_entry, patch_page, n_patches);
    return hipGetLastError();
}

hipError_t launch_validate(const int32_t *page_table, const ValRec *recs, uint32_t n, uint64_t n_pages,
                           ValReport *report, uint32_t *flag_dev, hipStream_t s) {
    if (n == 0)
        return hipSuccess;
    hipLaunchKernelGGL(validate_kernel, dim3(n), dim3(256), 0, s, page_table, recs, n_pages, report, flag_dev);
    return hipGetLastError();
}

hipError_t launch_patch(int32_t *page_table, const uint64_t *entry, const int32_t *page, uint32_t n,
                        hipStream_t s) {
    if (n == 0)
        return hipSuccess;
    hipLaunchKernelGGL(patch_kernel, dim3((n + 255) / 256), dim3(256), 0, s, page_table, entry, page, n);
    return hipGetLastError();
}

hipError_t launch_append(unsigned char *pool_base, uint32_t log2_page, int32_t *page_table, const AppendRec *recs,
                         uint32_t n, const ClassRec *classes, const void *new_k, const void *new_v,
                         const uint64_t *patch_entry, const int32_t *patch_page, uint32_t n_patches,
                         const uint32_t *bad, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
    const uint32_t blocks = n + (n_patches + 255) / 256;
    if (blocks == 0)
        return hipSuccess;
    hipExtLaunchKernelGGL(append_kernel, dim3(blocks), dim3(256), 0, s, ev0, ev1, 0, pool_base, log2_page, page_table,
                          recs, n, classes, static_cast<const uint16_t *>(new_k),
                          static_cast<const uint16_t *>(new_v), patch_entry, patch_page, n_patches, bad);
    return hipGetLastError();
}

hipError_t launch_copy_tokens(bool to_pool, unsigned char *pool_base, uint32_t log2_page, const int32_t *page_table,
                              const GatherRec *recs, uint32_t n, const ClassRec *classes, void *k_io, void *v_io,
                              const uint32_t *bad, hipStream_t s) {
    if (n == 0)
        return hipSuccess;
    if (to_pool)
        hipLaunchKernelGGL(copy_tokens_kernel<true>, dim3(n), dim3(256), 0, s, pool_base, log2_page, page_table,
                           recs, classes, static_cast<uint16_t *>(k_io), static_cast<uint16_t *>(v_io), bad);
    else
        hipLaunchKernelGGL(copy_tokens_kernel<false>, dim3(n), dim3(256), 0, s, pool_base, log2_page, page_table,
                           recs, classes, static_cast<uint16_t *>(k_io), static_cast<uint16_t *>(v_io), bad);
    return hipGetLastError();
}

} // namespace ukv
