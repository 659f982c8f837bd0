// Continuous-batching loop of one stage (Algorithm 3): batcher, page allocator
// and per-request progress on the host; one hybrid stage_step per pass.
#include <algorithm>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/lemix_sched.h"
#include "../../include/lemix_serve.h"
#include "common.h"

namespace {

// one workgroup per row; rows are whole 16-byte pieces.  to_batch: request row -> batch row
// `blockIdx.x`, else the reverse.
__global__ void rows_copy_kernel(const uint64_t* ptrs, char* batch, int row_bytes, int to_batch) {
  char* a = batch + (size_t)blockIdx.x * row_bytes;
  char* b = (char*)ptrs[blockIdx.x];
  const uint4* src = (const uint4*)(to_batch ? b : a);
  uint4* dst = (uint4*)(to_batch ? a : b);
  for (int i = threadIdx.x; i < row_bytes / 16; i += blockDim.x) dst[i] = src[i];
}

struct Request {
  const char* X;
  char* Y;
  int prompt_len, total, done;
  int reserved = 0;   // pages set aside for the whole sequence once the request has started (0: not started)
  std::vector<int32_t> pages;
};

constexpr int kSlots = 2;

}  // namespace

struct ls_server {
  ls_stage* stage;
  ls_config c;
  ls_server_config cfg;
  void *k_pool, *v_pool;
  ls_batcher* batcher = nullptr;
  std::unordered_map<int64_t, Request> req;
  std::vector<int32_t> free_pages;
  int unreserved = 0;   // pages of the pool that no started request has set aside
  int row_bytes;
  // per pass: [block table B x maxp][ctx_len B] int32, then [x ptr rows][y ptr rows] u64
  size_t stage_bytes, ptr_off;
  char* host_stage[kSlots] = {nullptr, nullptr};
  char* dev_stage[kSlots] = {nullptr, nullptr};
  hipEvent_t copied[kSlots] = {nullptr, nullptr};
  bool used[kSlots] = {false, false};
  int slot = 0;
  char *xb = nullptr, *yb = nullptr;
};

extern "C" {

void ls_server_destroy(ls_server* sv) {
  if (!sv) return;
  for (int i = 0; i < kSlots; ++i) {
    if (sv->copied[i]) { (void)hipEventSynchronize(sv->copied[i]); (void)hipEventDestroy(sv->copied[i]); }
    if (sv->host_stage[i]) (void)hipHostFree(sv->host_stage[i]);
    if (sv->dev_stage[i]) (void)hipFree(sv->dev_stage[i]);
  }
  if (sv->xb) (void)hipFree(sv->xb);
  if (sv->yb) (void)hipFree(sv->yb);
  ls_batcher_destroy(sv->batcher);
  delete sv;
}

ls_status ls_server_create(ls_stage* s, const ls_server_config* cfg, void* k_pool, void* v_pool, ls_server** out) {
  LS_REQUIRE(s && cfg && k_pool && v_pool && out, "server_create: null argument");
  LS_REQUIRE(cfg->max_batch >= 1 && cfg->max_batch <= 256, "server_create: max_batch %d outside 1..256", cfg->max_batch);
  LS_REQUIRE(cfg->max_wait >= 0, "server_create: max_wait must be non-negative");
  LS_REQUIRE(cfg->n_pages >= 1 && cfg->max_pages_per_req >= 1, "server_create: non-positive page counts");
  LS_REQUIRE(cfg->max_chunk >= 1, "server_create: max_chunk must be at least 1");
  LS_REQUIRE(cfg->max_tokens >= cfg->max_batch, "server_create: max_tokens %d cannot hold a decode row of each of %d requests",
             cfg->max_tokens, cfg->max_batch);
  ls_server* sv = new (std::nothrow) ls_server();
  if (!sv) { ls_set_error("host allocation failed"); return LS_ENOMEM; }
  sv->stage = s;
  sv->cfg = *cfg;
  sv->k_pool = k_pool;
  sv->v_pool = v_pool;
  ls_status rc = ls_get_config(s, &sv->c);
  if (rc == LS_OK) rc = ls_batcher_create(cfg->max_batch, cfg->max_wait, &sv->batcher);
  if (rc != LS_OK) { ls_server_destroy(sv); return rc; }
  sv->row_bytes = sv->c.d_model * (int)dtype_size(sv->c.io_dtype);
  sv->free_pages.resize(cfg->n_pages);
  for (int i = 0; i < cfg->n_pages; ++i) sv->free_pages[i] = cfg->n_pages - 1 - i;  // page 0 is handed out first
  sv->unreserved = cfg->n_pages;
  sv->ptr_off = align_up(((size_t)cfg->max_batch * cfg->max_pages_per_req + cfg->max_batch) * sizeof(int32_t), 16);
  sv->stage_bytes = sv->ptr_off + 2 * (size_t)cfg->max_tokens * sizeof(uint64_t);
  bool ok = true;
  for (int i = 0; i < kSlots && ok; ++i) {
    ok = hipHostMalloc((void**)&sv->host_stage[i], sv->stage_bytes, hipHostMallocDefault) == hipSuccess &&
         hipMalloc((void**)&sv->dev_stage[i], sv->stage_bytes) == hipSuccess &&
         hipEventCreateWithFlags(&sv->copied[i], hipEventDisableTiming) == hipSuccess;
  }
  const size_t batch_bytes = (size_t)cfg->max_tokens * sv->row_bytes;
  ok = ok && hipMalloc((void**)&sv->xb, batch_bytes) == hipSuccess && hipMalloc((void**)&sv->yb, batch_bytes) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    ls_server_destroy(sv);
    ls_set_error("server_create: allocation of the staging buffers failed");
    return LS_ENOMEM;
  }
  *out = sv;
  return LS_OK;
}

ls_status ls_server_submit(ls_server* sv, int64_t id, const void* X, void* Y, int prompt_len, int n_decode) {
  LS_REQUIRE(sv && X && Y, "server_submit: null argument");
  LS_REQUIRE(id >= 0, "server_submit: request ids are non-negative");
  LS_REQUIRE(prompt_len >= 1 && n_decode >= 0, "server_submit: prompt_len %d, n_decode %d", prompt_len, n_decode);
  LS_REQUIRE(!sv->req.count(id), "server_submit: request %lld is already in flight", (long long)id);
  const long total = (long)prompt_len + n_decode;
  const int P = sv->c.page_size;
  LS_REQUIRE((total + P - 1) / P <= sv->cfg.max_pages_per_req,
             "server_submit: %ld tokens need more than %d pages of %d", total, sv->cfg.max_pages_per_req, P);
  LS_REQUIRE((total + P - 1) / P <= sv->cfg.n_pages, "server_submit: %ld tokens exceed the whole pool", total);
  LS_REQUIRE(sv->c.block != LS_BLOCK_LLAMA || total <= sv->c.max_pos, "server_submit: %ld tokens exceed max_pos %d",
             total, sv->c.max_pos);
  LS_REQUIRE((uintptr_t)X % 16 == 0 && (uintptr_t)Y % 16 == 0, "server_submit: X and Y must be 16-byte aligned");
  LS_TRY(ls_batcher_push(sv->batcher, id, 0));
  Request r;
  r.X = (const char*)X;
  r.Y = (char*)Y;
  r.prompt_len = prompt_len;
  r.total = (int)total;
  r.done = 0;
  sv->req.emplace(id, std::move(r));
  return LS_OK;
}

int ls_server_in_flight(const ls_server* sv) { return sv ? (int)sv->req.size() : 0; }

ls_status ls_server_pass(ls_server* sv, double now, void* workspace, void* stream, ls_pass_report* report,
                         int64_t* ran_ids, int64_t* finished_ids) {
  LS_REQUIRE(sv && workspace, "server_pass: null argument");
  hipStream_t st = (hipStream_t)stream;
  const int P = sv->c.page_size, maxp = sv->cfg.max_pages_per_req;
  std::vector<int64_t> batch(sv->cfg.max_batch);
  int n_batch = 0, n_new = 0, blocked = 0;
  LS_TRY(ls_batcher_form(sv->batcher, now, batch.data(), &n_batch, &n_new, &blocked));
  ls_pass_report rep = {n_batch, n_new, 0, 0, 0, 0, 0, 0, 0};

  // the pass's members: decode rows first, then prompt chunks, each in batch order
  struct Member { int64_t id; int rows; };
  std::vector<Member> dec, pre;
  int rows_left = sv->cfg.max_tokens;
  // A request starts only when the pages of its whole sequence can be set aside: members that have started
  // then always find the pages their next rows need, so every one of them finishes and the pool cannot fill
  // up with partly served requests that all wait for each other.  (One request alone always fits: submit
  // checks it.)  The pages themselves are still taken from the free list just before the rows that need them.
  auto take_pages = [&](Request& r, int rows) {
    if (r.reserved == 0) {
      const int whole = (r.total + P - 1) / P;
      if (whole > sv->unreserved) return false;
      r.reserved = whole;
      sv->unreserved -= whole;
    }
    const int need = (r.done + rows + P - 1) / P - (int)r.pages.size();
    for (int i = 0; i < need; ++i) { r.pages.push_back(sv->free_pages.back()); sv->free_pages.pop_back(); }
    return true;
  };
  for (int i = 0; i < n_batch; ++i) {
    Request& r = sv->req.at(batch[i]);
    if (r.done >= r.prompt_len && rows_left > 0 && take_pages(r, 1)) { dec.push_back({batch[i], 1}); --rows_left; }
  }
  for (int i = 0; i < n_batch; ++i) {
    Request& r = sv->req.at(batch[i]);
    if (r.done >= r.prompt_len || (int)pre.size() >= 32) continue;
    const int rows = std::min({sv->cfg.max_chunk, r.prompt_len - r.done, rows_left});
    if (rows > 0 && take_pages(r, rows)) { pre.push_back({batch[i], rows}); rows_left -= rows; }
  }
  rep.n_decode = (int)dec.size();
  rep.n_prefill = (int)pre.size();
  rep.n_rows = sv->cfg.max_tokens - rows_left;
  rep.n_stalled = n_batch - rep.n_decode - rep.n_prefill;

  if (rep.n_rows > 0) {
    const int B = rep.n_decode + rep.n_prefill, T = rep.n_rows;
    const int sl = sv->slot;
    sv->slot = (sl + 1) % kSlots;
    if (sv->used[sl]) LS_CHECK_HIP(hipEventSynchronize(sv->copied[sl]));
    int32_t* table = (int32_t*)sv->host_stage[sl];
    int32_t* ctx = table + (size_t)sv->cfg.max_batch * maxp;
    uint64_t* xptr = (uint64_t*)(sv->host_stage[sl] + sv->ptr_off);
    uint64_t* yptr = xptr + sv->cfg.max_tokens;
    std::vector<int32_t> chunk_len;
    int b = 0, row = 0;
    auto add = [&](const Member& m) {
      const Request& r = sv->req.at(m.id);
      for (int j = 0; j < maxp; ++j) table[(size_t)b * maxp + j] = j < (int)r.pages.size() ? r.pages[j] : 0;
      ctx[b] = r.done;
      for (int k = 0; k < m.rows; ++k, ++row) {
        xptr[row] = (uint64_t)(uintptr_t)(r.X + (size_t)(r.done + k) * sv->row_bytes);
        yptr[row] = (uint64_t)(uintptr_t)(r.Y + (size_t)(r.done + k) * sv->row_bytes);
      }
      if (ran_ids) ran_ids[b] = m.id;
      ++b;
    };
    for (const Member& m : dec) add(m);
    for (const Member& m : pre) { add(m); chunk_len.push_back(m.rows); }
    char* dv = sv->dev_stage[sl];
    LS_CHECK_HIP(hipMemcpyAsync(dv, sv->host_stage[sl], sv->stage_bytes, hipMemcpyHostToDevice, st));
    LS_CHECK_HIP(hipEventRecord(sv->copied[sl], st));
    sv->used[sl] = true;
    const uint64_t* dx = (const uint64_t*)(dv + sv->ptr_off);
    const uint64_t* dy = dx + sv->cfg.max_tokens;
    rows_copy_kernel<<<T, 128, 0, st>>>(dx, sv->xb, sv->row_bytes, 1);
    LS_CHECK_LAUNCH();
    ls_kv kv;
    kv.k_pool = sv->k_pool;
    kv.v_pool = sv->v_pool;
    kv.block_table = (const int32_t*)dv;
    kv.ctx_len = (const int32_t*)dv + (size_t)sv->cfg.max_batch * maxp;
    kv.ctx_len_host = ctx;
    kv.n_pages = sv->cfg.n_pages;
    kv.max_pages_per_req = maxp;
    LS_TRY(stage_step(sv->stage, sv->xb, rep.n_decode, chunk_len.data(), rep.n_prefill, &kv, sv->yb, workspace, st));
    rows_copy_kernel<<<T, 128, 0, st>>>(dy, sv->yb, sv->row_bytes, 0);
    LS_CHECK_LAUNCH();

    // progress and the filter of finished requests
    std::vector<int64_t> fin;
    auto advance = [&](const Member& m) {
      Request& r = sv->req.at(m.id);
      r.done += m.rows;
      if (r.done >= r.total) fin.push_back(m.id);
    };
    for (const Member& m : dec) advance(m);
    for (const Member& m : pre) advance(m);
    for (size_t i = 0; i < fin.size(); ++i) {
      Request& r = sv->req.at(fin[i]);
      for (int32_t pg : r.pages) sv->free_pages.push_back(pg);
      sv->unreserved += r.reserved;
      sv->req.erase(fin[i]);
      if (finished_ids) finished_ids[i] = fin[i];
    }
    LS_TRY(ls_batcher_finish(sv->batcher, fin.data(), (int)fin.size()));
    rep.n_finished = (int)fin.size();
  }
  rep.free_pages = (int)sv->free_pages.size();
  rep.unreserved_pages = sv->unreserved;
  if (report) *report = rep;
  return LS_OK;
}

}  // extern "C"
