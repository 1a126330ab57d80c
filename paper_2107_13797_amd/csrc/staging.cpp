// Host staging: the path between a framework's host memory and the device-resident operators.
//
// A stager owns a pool of page-locked host buffers (reused by size, least recently used ones
// released beyond a byte cap), two device staging buffers and a copy stream. Arrays move in
// chunks: while chunk c is converted on the caller's stream (import / export kernel), chunk c + 1
// is copied between pageable memory, a page-locked buffer and the device on the copy stream, so
// that the PCIe transfer, the host-side copy and the kernels overlap. All streams have the default
// priority; page-locked memory is allocated, never registered.
#include <string.h>

#include <algorithm>
#include <list>

#include "haflo_internal.hpp"

namespace {

struct PinnedBuf {
  void* p = nullptr;
  size_t bytes = 0;
  bool in_use = false;
  unsigned long long last_use = 0;
};

}  // namespace

struct haflo_stager {
  const haflo_ctx* ctx = nullptr;
  size_t chunk = 0;        // elements per chunk
  size_t pool_cap = 0;     // bytes of idle page-locked memory kept for reuse
  unsigned long long clock = 0;
  std::list<PinnedBuf> pool;  // a list: pointers to entries stay valid while others come and go
  void* d_stage[2] = {nullptr, nullptr};  // chunk * Lc words each
  hipStream_t copy = nullptr;
  hipEvent_t copied[2] = {nullptr, nullptr};    // chunk arrived in / left d_stage[s]
  hipEvent_t consumed[2] = {nullptr, nullptr};  // d_stage[s] may be overwritten
  // consumed[s] has been recorded by some call: its kernel may still be queued on the caller's stream
  // when the next call starts, so every later writer of d_stage[s] waits for the event first
  bool consumed_recorded[2] = {false, false};
  hipEvent_t entered = nullptr;  // position of the caller's stream when a transfer into device memory starts
  size_t pinned_allocs = 0, pinned_reuses = 0;

  // a free buffer of at least `bytes` (the smallest that fits), or a new one
  PinnedBuf* acquire(size_t bytes) {
    PinnedBuf* best = nullptr;
    for (PinnedBuf& b : pool)
      if (!b.in_use && b.bytes >= bytes && (!best || b.bytes < best->bytes)) best = &b;
    if (best) {
      ++pinned_reuses;
    } else {
      PinnedBuf nb;
      if (hipHostMalloc(&nb.p, bytes, hipHostMallocDefault) != hipSuccess) return nullptr;
      nb.bytes = bytes;
      pool.push_back(nb);
      best = &pool.back();
      ++pinned_allocs;
    }
    best->in_use = true;
    best->last_use = ++clock;
    return best;
  }
  void release(PinnedBuf* b) {
    b->in_use = false;
    b->last_use = ++clock;
    // keep at most pool_cap bytes idle: drop the least recently used idle buffers
    for (;;) {
      size_t idle = 0;
      std::list<PinnedBuf>::iterator lru = pool.end();
      for (std::list<PinnedBuf>::iterator it = pool.begin(); it != pool.end(); ++it) {
        if (it->in_use) continue;
        idle += it->bytes;
        if (lru == pool.end() || it->last_use < lru->last_use) lru = it;
      }
      if (idle <= pool_cap || lru == pool.end()) break;
      (void)hipHostFree(lru->p);
      pool.erase(lru);
    }
  }
};

namespace {

// `count` elements of `words` 32-bit words each from host memory to the device, chunk by chunk;
// when `import` is set each chunk is canonical ciphertexts and is converted into d_dst (internal
// elements), otherwise the words are copied as they are (plaintext residues).
int stage_in(haflo_stager* s, const uint32_t* h_src, size_t words, void* d_dst, size_t dst_stride_bytes,
             uint32_t* d_status, size_t count, bool import, hipStream_t st) {
  if (count == 0) return HAFLO_OK;
  const size_t chunk_bytes = s->chunk * words * 4;
  PinnedBuf* pin[2] = {s->acquire(chunk_bytes), s->acquire(chunk_bytes)};
  if (!pin[0] || !pin[1]) {
    if (pin[0]) s->release(pin[0]);
    if (pin[1]) s->release(pin[1]);
    return HAFLO_ENOMEM;
  }
  int rc = HAFLO_OK;
  bool used[2] = {false, false};
  size_t done = 0;
  // Nothing this call copies may overtake work already queued on the caller's stream: kernels that
  // still read the destination (a recycled block) or, for plaintexts, anything ordered before the call.
  if (hipEventRecord(s->entered, st) != hipSuccess || hipStreamWaitEvent(s->copy, s->entered, 0) != hipSuccess)
    rc = HAFLO_EHIP;
  for (int slot = 0; done < count && rc == HAFLO_OK; slot ^= 1) {
    const size_t n = std::min(s->chunk, count - done);
    // the page-locked buffer of this slot is free once the copy that used it has finished
    if (used[slot] && hipEventSynchronize(s->copied[slot]) != hipSuccess) rc = HAFLO_EHIP;
    // the staging buffer is free once the kernel that read it last has run: one of this call, or
    // one that an earlier call left queued on its stream
    if (import && s->consumed_recorded[slot] && hipStreamWaitEvent(s->copy, s->consumed[slot], 0) != hipSuccess)
      rc = HAFLO_EHIP;
    if (rc != HAFLO_OK) break;
    memcpy(pin[slot]->p, h_src + done * words, n * words * 4);
    void* dst = import ? s->d_stage[slot] : (void*)((char*)d_dst + done * dst_stride_bytes);
    if (hipMemcpyAsync(dst, pin[slot]->p, n * words * 4, hipMemcpyHostToDevice, s->copy) != hipSuccess ||
        hipEventRecord(s->copied[slot], s->copy) != hipSuccess) {
      rc = HAFLO_EHIP;
      break;
    }
    used[slot] = true;
    if (hipStreamWaitEvent(st, s->copied[slot], 0) != hipSuccess) {
      rc = HAFLO_EHIP;
      break;
    }
    if (import) {
      rc = haflo_import_cipher(s->ctx, (const uint32_t*)s->d_stage[slot], (char*)d_dst + done * dst_stride_bytes,
                               d_status, n, st);
      if (rc == HAFLO_OK) {
        if (hipEventRecord(s->consumed[slot], st) != hipSuccess) rc = HAFLO_EHIP;
        else s->consumed_recorded[slot] = true;
      }
    }
    done += n;
  }
  // the page-locked buffers go back to the pool only after their last copy has left them
  for (int slot = 0; slot < 2; ++slot) {
    if (used[slot] && hipEventSynchronize(s->copied[slot]) != hipSuccess && rc == HAFLO_OK) rc = HAFLO_EHIP;
    s->release(pin[slot]);
  }
  return rc;
}

int stage_out(haflo_stager* s, const void* d_src, size_t src_stride_bytes, size_t words, uint32_t* h_dst, size_t count,
              bool do_export, hipStream_t st) {
  if (count == 0) return HAFLO_OK;
  const size_t chunk_bytes = s->chunk * words * 4;
  PinnedBuf* pin[2] = {s->acquire(chunk_bytes), s->acquire(chunk_bytes)};
  if (!pin[0] || !pin[1]) {
    if (pin[0]) s->release(pin[0]);
    if (pin[1]) s->release(pin[1]);
    return HAFLO_ENOMEM;
  }
  int rc = HAFLO_OK;
  size_t issued = 0;
  size_t len[2] = {0, 0}, at[2] = {0, 0};
  bool busy[2] = {false, false};
  auto drain = [&](int slot) {
    if (!busy[slot]) return;
    if (hipEventSynchronize(s->copied[slot]) != hipSuccess) rc = HAFLO_EHIP;
    memcpy(h_dst + at[slot] * words, pin[slot]->p, len[slot] * words * 4);
    busy[slot] = false;
  };
  for (int slot = 0; issued < count && rc == HAFLO_OK; slot ^= 1) {
    drain(slot);  // chunk issued two rounds ago: copy it out of the page-locked buffer
    if (rc != HAFLO_OK) break;
    const size_t n = std::min(s->chunk, count - issued);
    const void* src = (const char*)d_src + issued * src_stride_bytes;
    if (do_export) {
      // the staging buffer of this slot was last read by the copy that drain() waited for, or by an
      // import kernel that an earlier call queued (on this stream or another)
      if (s->consumed_recorded[slot] && hipStreamWaitEvent(st, s->consumed[slot], 0) != hipSuccess) {
        rc = HAFLO_EHIP;
        break;
      }
      rc = haflo_export_cipher(s->ctx, src, (uint32_t*)s->d_stage[slot], n, st);
      if (rc != HAFLO_OK) break;
      src = s->d_stage[slot];
    }
    if (hipEventRecord(s->consumed[slot], st) != hipSuccess ||
        hipStreamWaitEvent(s->copy, s->consumed[slot], 0) != hipSuccess ||
        hipMemcpyAsync(pin[slot]->p, src, n * words * 4, hipMemcpyDeviceToHost, s->copy) != hipSuccess ||
        hipEventRecord(s->copied[slot], s->copy) != hipSuccess) {
      rc = HAFLO_EHIP;
      break;
    }
    s->consumed_recorded[slot] = true;
    busy[slot] = true;
    len[slot] = n;
    at[slot] = issued;
    issued += n;
  }
  // finish in issue order
  const int first = (busy[0] && busy[1] && at[1] < at[0]) ? 1 : 0;
  drain(first);
  drain(first ^ 1);
  for (int slot = 0; slot < 2; ++slot) {
    if (busy[slot]) (void)hipEventSynchronize(s->copied[slot]);  // error path: the copy must not outlive the buffer
    s->release(pin[slot]);
  }
  return rc;
}

}  // namespace

extern "C" {

int haflo_stager_create(const haflo_ctx* ctx, size_t chunk_elems, size_t pool_cap_bytes, haflo_stager** out) {
  if (!ctx || !out || chunk_elems == 0) return HAFLO_EINVAL;
  haflo_stager* s = new haflo_stager();
  s->ctx = ctx;
  s->chunk = chunk_elems;
  s->pool_cap = pool_cap_bytes;
  bool ok = hipStreamCreateWithFlags(&s->copy, hipStreamNonBlocking) == hipSuccess &&
            hipEventCreateWithFlags(&s->entered, hipEventDisableTiming) == hipSuccess;
  for (int i = 0; i < 2 && ok; ++i) {
    ok = hipMalloc(&s->d_stage[i], chunk_elems * (size_t)ctx->lc * 4) == hipSuccess &&
         hipEventCreateWithFlags(&s->copied[i], hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&s->consumed[i], hipEventDisableTiming) == hipSuccess;
  }
  if (!ok) {
    haflo_stager_destroy(s);
    return HAFLO_ENOMEM;
  }
  *out = s;
  return HAFLO_OK;
}

int haflo_stager_destroy(haflo_stager* s) {
  if (!s) return HAFLO_OK;
  // best effort: nothing useful can be done about a failing release
  if (s->copy) (void)hipStreamSynchronize(s->copy);
  for (PinnedBuf& b : s->pool) (void)hipHostFree(b.p);
  for (int i = 0; i < 2; ++i) {
    if (s->d_stage[i]) (void)hipFree(s->d_stage[i]);
    if (s->copied[i]) (void)hipEventDestroy(s->copied[i]);
    if (s->consumed[i]) (void)hipEventDestroy(s->consumed[i]);
  }
  if (s->entered) (void)hipEventDestroy(s->entered);
  if (s->copy) (void)hipStreamDestroy(s->copy);
  delete s;
  return HAFLO_OK;
}

int haflo_stager_stats(const haflo_stager* s, size_t* pinned_bytes, size_t* pinned_allocs, size_t* pinned_reuses) {
  if (!s) return HAFLO_EINVAL;
  size_t total = 0;
  for (const PinnedBuf& b : s->pool) total += b.bytes;
  if (pinned_bytes) *pinned_bytes = total;
  if (pinned_allocs) *pinned_allocs = s->pinned_allocs;
  if (pinned_reuses) *pinned_reuses = s->pinned_reuses;
  return HAFLO_OK;
}

int haflo_stage_in_cipher(haflo_stager* s, const uint32_t* h_canon, void* d_cipher, uint32_t* d_status, size_t count,
                          void* stream) {
  if (!s || (count && (!h_canon || !d_cipher))) return HAFLO_EINVAL;
  return stage_in(s, h_canon, (size_t)s->ctx->lc, d_cipher, (size_t)s->ctx->N.nl * 4, d_status, count, true,
                  (hipStream_t)stream);
}

int haflo_stage_in_plain(haflo_stager* s, const uint32_t* h_plain, uint32_t* d_plain, size_t count, void* stream) {
  if (!s || (count && (!h_plain || !d_plain))) return HAFLO_EINVAL;
  return stage_in(s, h_plain, (size_t)s->ctx->lp, d_plain, (size_t)s->ctx->lp * 4, nullptr, count, false,
                  (hipStream_t)stream);
}

int haflo_stage_out_cipher(haflo_stager* s, const void* d_cipher, uint32_t* h_canon, size_t count, void* stream) {
  if (!s || (count && (!d_cipher || !h_canon))) return HAFLO_EINVAL;
  return stage_out(s, d_cipher, (size_t)s->ctx->N.nl * 4, (size_t)s->ctx->lc, h_canon, count, true,
                   (hipStream_t)stream);
}

int haflo_stage_out_plain(haflo_stager* s, const uint32_t* d_plain, uint32_t* h_plain, size_t count, void* stream) {
  if (!s || (count && (!d_plain || !h_plain))) return HAFLO_EINVAL;
  return stage_out(s, d_plain, (size_t)s->ctx->lp * 4, (size_t)s->ctx->lp, h_plain, count, false,
                   (hipStream_t)stream);
}

}  // extern "C"
