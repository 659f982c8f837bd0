// Moving one request's paged K/V between the pool and host memory (Algorithm 2, memory-aware
// execution: a task that has waited T_max for memory has its KV cache offloaded to the host and
// resumes from that copy).  A request's pages are scattered over the pool, so a gather kernel
// packs them (all layers, K and V) into one contiguous device buffer, which then crosses PCIe
// in a single copy; reloading is the same in reverse, into whatever pages the block table
// assigns to the request by then.  Pure byte movement: results are bit-exact.
//   packed[layer][0 = K, 1 = V][j][head][slot][head_dim] = pool[layer][block_table[b][j]][head][slot][:]
#include "common.h"

namespace {

// one workgroup per (page j, K/V, layer); a page of one layer is h * page * dh contiguous elements
template <bool TO_POOL>
__global__ __launch_bounds__(256) void kv_pack_kernel(char* k_pool, char* v_pool, const int32_t* table_row,
                                                      char* packed, size_t page_bytes, size_t layer_slab_bytes,
                                                      int n_req_pages) {
  const int j = blockIdx.x, which = blockIdx.y, l = blockIdx.z;
  char* pool = (which == 0 ? k_pool : v_pool) + (size_t)l * layer_slab_bytes + (size_t)table_row[j] * page_bytes;
  char* pk = packed + (((size_t)l * 2 + which) * n_req_pages + j) * page_bytes;
  for (size_t i = (size_t)threadIdx.x * 16; i < page_bytes; i += 256 * 16) {
    if (TO_POOL) *(u32x4*)(pool + i) = *(const u32x4*)(pk + i);
    else *(u32x4*)(pk + i) = *(const u32x4*)(pool + i);
  }
}

struct Geom {
  size_t page_bytes, layer_slab_bytes, total_bytes;
  int n_req_pages;
};

ls_status geometry(const ls_config* c, const ls_kv* kv, int request, int n_tokens, Geom* g) {
  LS_REQUIRE(c && kv && kv->k_pool && kv->v_pool && kv->block_table, "kv offload: null argument");
  LS_REQUIRE(request >= 0, "kv offload: negative request index");
  LS_REQUIRE(n_tokens >= 0, "kv offload: negative token count");
  const int npg = (n_tokens + c->page_size - 1) / c->page_size;
  LS_REQUIRE(npg <= kv->max_pages_per_req, "kv offload: %d tokens need %d pages, the block table holds %d", n_tokens,
             npg, kv->max_pages_per_req);
  const size_t esz = dtype_size(c->mma_dtype);
  g->page_bytes = (size_t)c->n_heads * c->page_size * c->head_dim * esz;
  g->layer_slab_bytes = (size_t)kv->n_pages * g->page_bytes;
  g->n_req_pages = npg;
  g->total_bytes = (size_t)c->n_layers * 2 * npg * g->page_bytes;
  LS_REQUIRE(g->page_bytes % 16 == 0, "kv offload: a page must be a multiple of 16 bytes");
  return LS_OK;
}

}  // namespace

extern "C" {

size_t lsk_kv_packed_bytes(const ls_config* c, int n_tokens) {
  if (!c || n_tokens <= 0) return 0;
  const size_t npg = (size_t)(n_tokens + c->page_size - 1) / c->page_size;
  return (size_t)c->n_layers * 2 * npg * c->n_heads * c->page_size * c->head_dim * dtype_size(c->mma_dtype);
}

// pool -> staging (device, lsk_kv_packed_bytes) -> host (pinned for an asynchronous copy)
ls_status lsk_kv_offload(const ls_config* c, const ls_kv* kv, int request, int n_tokens, void* staging, void* host,
                         void* stream) {
  Geom g;
  LS_TRY(geometry(c, kv, request, n_tokens, &g));
  if (g.n_req_pages == 0) return LS_OK;
  LS_REQUIRE(staging && host, "kv offload: null buffer");
  hipStream_t st = (hipStream_t)stream;
  const int32_t* row = kv->block_table + (size_t)request * kv->max_pages_per_req;
  kv_pack_kernel<false><<<dim3(g.n_req_pages, 2, c->n_layers), 256, 0, st>>>((char*)kv->k_pool, (char*)kv->v_pool, row,
                                                                            (char*)staging, g.page_bytes,
                                                                            g.layer_slab_bytes, g.n_req_pages);
  LS_CHECK_LAUNCH();
  LS_CHECK_HIP(hipMemcpyAsync(host, staging, g.total_bytes, hipMemcpyDeviceToHost, st));
  return LS_OK;
}

// host -> staging -> the pages the block table assigns to the request now
ls_status lsk_kv_reload(const ls_config* c, const ls_kv* kv, int request, int n_tokens, const void* host,
                        void* staging, void* stream) {
  Geom g;
  LS_TRY(geometry(c, kv, request, n_tokens, &g));
  if (g.n_req_pages == 0) return LS_OK;
  LS_REQUIRE(staging && host, "kv reload: null buffer");
  hipStream_t st = (hipStream_t)stream;
  LS_CHECK_HIP(hipMemcpyAsync(staging, host, g.total_bytes, hipMemcpyHostToDevice, st));
  const int32_t* row = kv->block_table + (size_t)request * kv->max_pages_per_req;
  kv_pack_kernel<true><<<dim3(g.n_req_pages, 2, c->n_layers), 256, 0, st>>>((char*)kv->k_pool, (char*)kv->v_pool, row,
                                                                           (char*)staging, g.page_bytes,
                                                                           g.layer_slab_bytes, g.n_req_pages);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

// Algorithm 2's MemoryAvailable: may a task that needs `need_bytes` more device memory start,
// given the profiled threshold?  used = total - free as the driver reports it.
ls_status lsk_memory_available(size_t need_bytes, size_t threshold_bytes, int* available, size_t* used_bytes) {
  LS_REQUIRE(available, "memory_available: null result");
  size_t free_b = 0, total_b = 0;
  LS_CHECK_HIP(hipMemGetInfo(&free_b, &total_b));
  const size_t used = total_b - free_b;
  if (used_bytes) *used_bytes = used;
  *available = used + need_bytes <= threshold_bytes ? 1 : 0;
  return LS_OK;
}

}  // extern "C"
