// Managed device-resident operands: the store behind the handle-based operator calls.
//
// The paper's section 3.3 keeps operator results in GPU memory, hands the framework a small
// handle for each and accepts handles back as operands, with an allocator of its own for those
// results. Here a store sub-allocates one device arena that the caller provides: objects
// (operands that were uploaded and results of operators) are carved from its low end, the
// temporary workspace of a call from its high end, both in units of 256 bytes with free
// neighbours merged. Every object carries the number of operator calls that will still consume
// it; the call that consumes it last frees its block, or writes its result into that block
// when the operator allows aliasing. All device work of a store runs on the one stream it was
// created with, so a freed block may be handed out again at once: the launches that use it are
// ordered behind those that read the old contents.
#include <algorithm>
#include <iterator>
#include <map>
#include <vector>

#include "haflo_internal.hpp"

namespace {

constexpr size_t kAlign = 256;
inline size_t round_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Obj {
  size_t off = 0, bytes = 0, count = 0;
  int kind = 0;
  uint32_t uses = 0;  // operator calls that may still consume it; 0 = until released
  uint32_t gen = 0;
  bool live = false;
};

}  // namespace

struct haflo_store {
  const haflo_ctx* ctx = nullptr;
  char* base = nullptr;
  size_t bytes = 0;
  hipStream_t st = nullptr;
  size_t cipher_bytes = 0, plain_bytes = 0;
  std::map<size_t, size_t> free_;  // offset -> length; neighbours never touch
  std::vector<Obj> objs;
  std::vector<uint32_t> free_slots;
  size_t live_bytes = 0, peak_bytes = 0, live_objs = 0;

  size_t elem_bytes(int kind) const {
    switch (kind) {
      case HAFLO_KIND_CIPHER: return cipher_bytes;
      case HAFLO_KIND_PLAIN: return plain_bytes;
      case HAFLO_KIND_F32: case HAFLO_KIND_I32: case HAFLO_KIND_U32: return 4;
      case HAFLO_KIND_F64: case HAFLO_KIND_U64: case HAFLO_KIND_I64: return 8;
      default: return 0;
    }
  }

  // a block of `want` bytes: the smallest free block that fits, cut at its low end (objects),
  // or the highest free block that fits, cut at its high end (temporaries)
  bool carve(size_t want, bool top, size_t* off) {
    want = round_up(want ? want : 1);
    std::map<size_t, size_t>::iterator pick = free_.end();
    if (top) {
      for (std::map<size_t, size_t>::iterator it = free_.end(); it != free_.begin();) {
        --it;
        if (it->second >= want) { pick = it; break; }
      }
    } else {
      for (std::map<size_t, size_t>::iterator it = free_.begin(); it != free_.end(); ++it)
        if (it->second >= want && (pick == free_.end() || it->second < pick->second)) pick = it;
    }
    if (pick == free_.end()) return false;
    size_t o = pick->first, len = pick->second;
    free_.erase(pick);
    if (top) {
      *off = o + len - want;
      if (len > want) free_[o] = len - want;
    } else {
      *off = o;
      if (len > want) free_[o + want] = len - want;
    }
    live_bytes += want;
    peak_bytes = std::max(peak_bytes, live_bytes);
    return true;
  }
  void give_back(size_t off, size_t len) {
    len = round_up(len ? len : 1);
    live_bytes -= len;
    std::map<size_t, size_t>::iterator next = free_.lower_bound(off);
    if (next != free_.end() && off + len == next->first) {
      len += next->second;
      next = free_.erase(next);
    }
    if (next != free_.begin()) {
      std::map<size_t, size_t>::iterator prev = std::prev(next);
      if (prev->first + prev->second == off) {
        prev->second += len;
        return;
      }
    }
    free_[off] = len;
  }

  Obj* get(haflo_handle h) {
    uint32_t slot = (uint32_t)(h & 0xFFFFFFFFu), gen = (uint32_t)(h >> 32);
    if (slot == 0 || slot > objs.size()) return nullptr;
    Obj* o = &objs[slot - 1];
    return (o->live && o->gen == gen) ? o : nullptr;
  }
  const Obj* get(haflo_handle h) const { return const_cast<haflo_store*>(this)->get(h); }
  void* ptr(const Obj* o) const { return base + o->off; }

  // a new object of `count` elements at offset `off` (already carved)
  haflo_handle adopt(int kind, size_t count, size_t off, size_t nbytes, uint32_t uses) {
    uint32_t slot;
    if (!free_slots.empty()) {
      slot = free_slots.back();
      free_slots.pop_back();
    } else {
      objs.push_back(Obj());
      slot = (uint32_t)objs.size() - 1;
    }
    Obj& o = objs[slot];
    o.off = off;
    o.bytes = nbytes;
    o.count = count;
    o.kind = kind;
    o.uses = uses;
    o.gen += 1;
    o.live = true;
    ++live_objs;
    return ((haflo_handle)o.gen << 32) | (slot + 1);
  }
  int create(int kind, size_t count, uint32_t uses, haflo_handle* out) {
    size_t eb = elem_bytes(kind);
    if (eb == 0 || (count && eb > (size_t)-1 / 2 / count)) return HAFLO_EINVAL;
    size_t off;
    if (!carve(eb * count, false, &off)) return HAFLO_ENOMEM;
    *out = adopt(kind, count, off, eb * count, uses);
    return HAFLO_OK;
  }
  // forget an object; its block is freed unless `keep_block`
  void retire(Obj* o, bool keep_block) {
    if (!keep_block) give_back(o->off, o->bytes);
    o->live = false;
    --live_objs;
    free_slots.push_back((uint32_t)(o - &objs[0]));
  }
  void drop(haflo_handle h) {
    Obj* o = get(h);
    if (o) retire(o, false);
  }
  // one use of `o` is over
  void consume(Obj* o) {
    if (o->uses == 0) return;
    if (--o->uses == 0) retire(o, false);
  }

  // the operands of one call: all alive, of the expected kinds, and each with enough uses left
  // for the number of times it appears
  bool operands_ok(const haflo_handle* h, const int* kinds, int n) {
    for (int i = 0; i < n; ++i) {
      Obj* o = get(h[i]);
      if (!o || o->kind != kinds[i]) return false;
      uint32_t times = 0;
      for (int j = 0; j < n; ++j) times += (h[j] == h[i]);
      if (o->uses != 0 && o->uses < times) return false;
    }
    return true;
  }
  // `o` is at its last use and appears once among the operands: its block can take the result
  bool last_use(const Obj* o, const haflo_handle* h, int n, haflo_handle self) const {
    int times = 0;
    for (int j = 0; j < n; ++j) times += (h[j] == self);
    return o->uses == 1 && times == 1;
  }
};

namespace {

// Temporary workspace of one call, taken from the high end of the arena and returned when the
// call has been enqueued.
struct Scratch {
  haflo_store* s;
  size_t off = 0, bytes = 0;
  bool held = false;
  explicit Scratch(haflo_store* store) : s(store) {}
  bool take(size_t want) {
    if (want == (size_t)-1) return false;
    bytes = want;
    if (want == 0) return true;
    held = s->carve(want, true, &off);
    return held;
  }
  void* ptr() const { return held ? s->base + off : nullptr; }
  ~Scratch() {
    if (held) s->give_back(off, bytes);
  }
};

}  // namespace

extern "C" {

int haflo_store_create(const haflo_ctx* ctx, void* d_arena, size_t arena_bytes, void* stream, haflo_store** out) {
  if (!ctx || !d_arena || !out || ((uintptr_t)d_arena % kAlign) != 0 || arena_bytes < kAlign) return HAFLO_EINVAL;
  haflo_store* s = new haflo_store();
  s->ctx = ctx;
  s->base = (char*)d_arena;
  s->bytes = arena_bytes / kAlign * kAlign;
  s->st = (hipStream_t)stream;
  haflo_ctx_info(ctx, nullptr, nullptr, nullptr, &s->cipher_bytes, &s->plain_bytes);
  s->free_[0] = s->bytes;
  *out = s;
  return HAFLO_OK;
}

int haflo_store_destroy(haflo_store* s) {
  delete s;
  return HAFLO_OK;
}

int haflo_store_stats(const haflo_store* s, size_t* live_bytes, size_t* peak_bytes, size_t* live_objects,
                      size_t* largest_free) {
  if (!s) return HAFLO_EINVAL;
  if (live_bytes) *live_bytes = s->live_bytes;
  if (peak_bytes) *peak_bytes = s->peak_bytes;
  if (live_objects) *live_objects = s->live_objs;
  if (largest_free) {
    size_t m = 0;
    for (std::map<size_t, size_t>::const_iterator it = s->free_.begin(); it != s->free_.end(); ++it)
      m = std::max(m, it->second);
    *largest_free = m;
  }
  return HAFLO_OK;
}

int haflo_store_new(haflo_store* s, int kind, size_t count, uint32_t uses, haflo_handle* out) {
  if (!s || !out) return HAFLO_EINVAL;
  return s->create(kind, count, uses, out);
}

int haflo_store_info(const haflo_store* s, haflo_handle h, int* kind, size_t* count, void** d_ptr,
                     uint32_t* uses_left) {
  if (!s) return HAFLO_EINVAL;
  const Obj* o = s->get(h);
  if (!o) return HAFLO_EINVAL;
  if (kind) *kind = o->kind;
  if (count) *count = o->count;
  if (d_ptr) *d_ptr = s->ptr(o);
  if (uses_left) *uses_left = o->uses;
  return HAFLO_OK;
}

int haflo_store_release(haflo_store* s, haflo_handle h) {
  if (!s) return HAFLO_EINVAL;
  Obj* o = s->get(h);
  if (!o) return HAFLO_EINVAL;
  s->retire(o, false);
  return HAFLO_OK;
}

int haflo_h_upload(haflo_store* s, int kind, const void* src, int src_on_host, size_t count, uint32_t uses,
                   haflo_handle* out) {
  if (!s || !out || (!src && count)) return HAFLO_EINVAL;
  haflo_handle h;
  int rc = s->create(kind, count, uses, &h);
  if (rc != HAFLO_OK) return rc;
  const Obj* o = s->get(h);
  if (o->bytes &&
      hipMemcpyAsync(s->ptr(o), src, o->bytes, src_on_host ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice,
                     s->st) != hipSuccess) {
    s->drop(h);
    return HAFLO_EHIP;
  }
  *out = h;
  return HAFLO_OK;
}

int haflo_h_download(haflo_store* s, haflo_handle h, void* dst, int dst_on_host) {
  if (!s) return HAFLO_EINVAL;
  Obj* o = s->get(h);
  if (!o || (!dst && o->bytes)) return HAFLO_EINVAL;
  if (o->bytes) {
    if (hipMemcpyAsync(dst, s->ptr(o), o->bytes, dst_on_host ? hipMemcpyDeviceToHost : hipMemcpyDeviceToDevice,
                       s->st) != hipSuccess)
      return HAFLO_EHIP;
    if (dst_on_host && hipStreamSynchronize(s->st) != hipSuccess) return HAFLO_EHIP;
  }
  s->consume(o);
  return HAFLO_OK;
}

int haflo_h_encode(haflo_store* s, haflo_handle values, uint32_t scale_bits, uint32_t uses, haflo_handle* plain,
                   haflo_handle* status) {
  if (!s || !plain) return HAFLO_EINVAL;
  const int kinds[1] = {HAFLO_KIND_F32};
  if (!s->operands_ok(&values, kinds, 1)) return HAFLO_EINVAL;
  size_t count = s->get(values)->count;
  haflo_handle hp, hs = 0;
  int rc = s->create(HAFLO_KIND_PLAIN, count, uses, &hp);
  if (rc == HAFLO_OK && status && (rc = s->create(HAFLO_KIND_U32, count, 1, &hs)) != HAFLO_OK) s->drop(hp);
  if (rc != HAFLO_OK) return rc;
  rc = haflo_encode_f32(s->ctx, (const float*)s->ptr(s->get(values)), scale_bits, (uint32_t*)s->ptr(s->get(hp)),
                        hs ? (uint32_t*)s->ptr(s->get(hs)) : nullptr, count, s->st);
  if (rc != HAFLO_OK) {
    s->drop(hp);
    s->drop(hs);
    return rc;
  }
  s->consume(s->get(values));
  *plain = hp;
  if (status) *status = hs;
  return HAFLO_OK;
}

int haflo_h_encode_exponents(haflo_store* s, haflo_handle values, uint32_t scale_bits, uint32_t uses,
                             haflo_handle* exponents, haflo_handle* status) {
  if (!s || !exponents) return HAFLO_EINVAL;
  const int kinds[1] = {HAFLO_KIND_F32};
  if (!s->operands_ok(&values, kinds, 1)) return HAFLO_EINVAL;
  size_t count = s->get(values)->count;
  haflo_handle he, hs = 0;
  int rc = s->create(HAFLO_KIND_I32, count, uses, &he);
  if (rc == HAFLO_OK && status && (rc = s->create(HAFLO_KIND_U32, count, 1, &hs)) != HAFLO_OK) s->drop(he);
  if (rc != HAFLO_OK) return rc;
  rc = haflo_encode_exponents_f32((const float*)s->ptr(s->get(values)), scale_bits, (int32_t*)s->ptr(s->get(he)),
                                  hs ? (uint32_t*)s->ptr(s->get(hs)) : nullptr, count, s->st);
  if (rc != HAFLO_OK) {
    s->drop(he);
    s->drop(hs);
    return rc;
  }
  s->consume(s->get(values));
  *exponents = he;
  if (status) *status = hs;
  return HAFLO_OK;
}

int haflo_h_decode(haflo_store* s, haflo_handle plain, uint32_t scale_bits, uint32_t uses, haflo_handle* values,
                   haflo_handle* status) {
  if (!s || !values) return HAFLO_EINVAL;
  const int kinds[1] = {HAFLO_KIND_PLAIN};
  if (!s->operands_ok(&plain, kinds, 1)) return HAFLO_EINVAL;
  size_t count = s->get(plain)->count;
  haflo_handle hv, hs = 0;
  int rc = s->create(HAFLO_KIND_F64, count, uses, &hv);
  if (rc == HAFLO_OK && status && (rc = s->create(HAFLO_KIND_U32, count, 1, &hs)) != HAFLO_OK) s->drop(hv);
  if (rc != HAFLO_OK) return rc;
  rc = haflo_decode(s->ctx, (const uint32_t*)s->ptr(s->get(plain)), scale_bits, nullptr, (double*)s->ptr(s->get(hv)),
                    hs ? (uint32_t*)s->ptr(s->get(hs)) : nullptr, count, s->st);
  if (rc != HAFLO_OK) {
    s->drop(hv);
    s->drop(hs);
    return rc;
  }
  s->consume(s->get(plain));
  *values = hv;
  if (status) *status = hs;
  return HAFLO_OK;
}

int haflo_h_encrypt(haflo_store* s, haflo_handle plain, haflo_handle r, uint32_t uses, haflo_handle* cipher) {
  if (!s || !cipher) return HAFLO_EINVAL;
  const haflo_handle in[2] = {plain, r};
  const int kinds[2] = {HAFLO_KIND_PLAIN, HAFLO_KIND_PLAIN};
  if (!s->operands_ok(in, kinds, 2)) return HAFLO_EINVAL;
  size_t count = s->get(plain)->count;
  if (s->get(r)->count != count) return HAFLO_EINVAL;
  haflo_handle hc;
  int rc = s->create(HAFLO_KIND_CIPHER, count, uses, &hc);
  if (rc != HAFLO_OK) return rc;
  Scratch ws(s);
  if (!ws.take(haflo_workspace_bytes(s->ctx, HAFLO_OP_ENCRYPT, count, 0))) {
    s->drop(hc);
    return HAFLO_ENOMEM;
  }
  rc = haflo_encrypt(s->ctx, (const uint32_t*)s->ptr(s->get(plain)), (const uint32_t*)s->ptr(s->get(r)),
                     s->ptr(s->get(hc)), count, ws.ptr(), ws.bytes, s->st);
  if (rc != HAFLO_OK) {
    s->drop(hc);
    return rc;
  }
  s->consume(s->get(plain));
  s->consume(s->get(r));
  *cipher = hc;
  return HAFLO_OK;
}

int haflo_h_decrypt(haflo_store* s, haflo_handle cipher, uint32_t uses, haflo_handle* plain) {
  if (!s || !plain) return HAFLO_EINVAL;
  const int kinds[1] = {HAFLO_KIND_CIPHER};
  if (!s->operands_ok(&cipher, kinds, 1)) return HAFLO_EINVAL;
  size_t count = s->get(cipher)->count;
  const size_t want = haflo_workspace_bytes(s->ctx, HAFLO_OP_DECRYPT, count, 0);
  if (want == (size_t)-1) return HAFLO_ENOPRIV;  // a public-only context has no decryption workspace
  haflo_handle hp;
  int rc = s->create(HAFLO_KIND_PLAIN, count, uses, &hp);
  if (rc != HAFLO_OK) return rc;
  Scratch ws(s);
  if (!ws.take(want)) {
    s->drop(hp);
    return HAFLO_ENOMEM;
  }
  rc = haflo_decrypt(s->ctx, s->ptr(s->get(cipher)), (uint32_t*)s->ptr(s->get(hp)), count, ws.ptr(), ws.bytes, s->st);
  if (rc != HAFLO_OK) {
    s->drop(hp);
    return rc;
  }
  s->consume(s->get(cipher));
  *plain = hp;
  return HAFLO_OK;
}

int haflo_h_add(haflo_store* s, haflo_handle a, haflo_handle b, uint32_t uses, haflo_handle* out) {
  if (!s || !out) return HAFLO_EINVAL;
  const haflo_handle in[2] = {a, b};
  const int kinds[2] = {HAFLO_KIND_CIPHER, HAFLO_KIND_CIPHER};
  if (!s->operands_ok(in, kinds, 2)) return HAFLO_EINVAL;
  Obj* oa = s->get(a);
  Obj* ob = s->get(b);
  size_t count = oa->count;
  if (ob->count != count) return HAFLO_EINVAL;
  // the result takes over the block of an operand that nobody reads afterwards
  Obj* reuse = s->last_use(oa, in, 2, a) ? oa : (s->last_use(ob, in, 2, b) ? ob : nullptr);
  size_t off, nbytes = s->cipher_bytes * count;
  if (reuse) {
    off = reuse->off;
  } else if (!s->carve(nbytes, false, &off)) {
    return HAFLO_ENOMEM;
  }
  int rc = haflo_add(s->ctx, s->ptr(oa), s->ptr(ob), s->base + off, count, s->st);
  if (rc != HAFLO_OK) {
    if (!reuse) s->give_back(off, nbytes);
    return rc;
  }
  if (reuse) s->retire(reuse, true);
  if (oa != reuse) s->consume(oa);
  if (ob != reuse) s->consume(ob);  // a == b: the same object gives up two uses
  *out = s->adopt(HAFLO_KIND_CIPHER, count, off, nbytes, uses);
  return HAFLO_OK;
}

int haflo_h_scalar_mul(haflo_store* s, haflo_handle cipher, int64_t k, uint32_t uses, haflo_handle* out) {
  if (!s || !out) return HAFLO_EINVAL;
  const int kinds[1] = {HAFLO_KIND_CIPHER};
  if (!s->operands_ok(&cipher, kinds, 1)) return HAFLO_EINVAL;
  Obj* oc = s->get(cipher);
  size_t count = oc->count, nbytes = s->cipher_bytes * count, off;
  bool reuse = s->last_use(oc, &cipher, 1, cipher);
  if (reuse) {
    off = oc->off;
  } else if (!s->carve(nbytes, false, &off)) {
    return HAFLO_ENOMEM;
  }
  int rc = HAFLO_ENOMEM;
  {
    Scratch ws(s);
    if (ws.take(haflo_workspace_bytes(s->ctx, HAFLO_OP_SCALAR_MUL, count, 0)))
      rc = haflo_scalar_mul_i64_bcast(s->ctx, s->ptr(oc), k, s->base + off, count, ws.ptr(), ws.bytes, s->st);
  }
  if (rc != HAFLO_OK) {
    if (!reuse) s->give_back(off, nbytes);
    return rc;
  }
  if (reuse) s->retire(oc, true);
  else s->consume(oc);
  *out = s->adopt(HAFLO_KIND_CIPHER, count, off, nbytes, uses);
  return HAFLO_OK;
}

int haflo_h_scalar_mul_each(haflo_store* s, haflo_handle cipher, haflo_handle scalars, uint32_t uses,
                            haflo_handle* out) {
  if (!s || !out) return HAFLO_EINVAL;
  const haflo_handle in[2] = {cipher, scalars};
  const int kinds[2] = {HAFLO_KIND_CIPHER, HAFLO_KIND_U64};
  if (!s->operands_ok(in, kinds, 2)) return HAFLO_EINVAL;
  Obj* oc = s->get(cipher);
  Obj* ok = s->get(scalars);
  size_t count = oc->count, nbytes = s->cipher_bytes * count, off;
  if (ok->count != count) return HAFLO_EINVAL;
  bool reuse = s->last_use(oc, in, 2, cipher);
  if (reuse) {
    off = oc->off;
  } else if (!s->carve(nbytes, false, &off)) {
    return HAFLO_ENOMEM;
  }
  int rc = HAFLO_ENOMEM;
  {
    Scratch ws(s);
    if (ws.take(haflo_workspace_bytes(s->ctx, HAFLO_OP_SCALAR_MUL, count, 0)))
      rc = haflo_scalar_mul_u64(s->ctx, s->ptr(oc), (const uint64_t*)s->ptr(ok), s->base + off, count, ws.ptr(),
                                ws.bytes, s->st);
  }
  if (rc != HAFLO_OK) {
    if (!reuse) s->give_back(off, nbytes);
    return rc;
  }
  if (reuse) s->retire(oc, true);
  else s->consume(oc);
  s->consume(ok);
  *out = s->adopt(HAFLO_KIND_CIPHER, count, off, nbytes, uses);
  return HAFLO_OK;
}

int haflo_h_matvec(haflo_store* s, int orientation, haflo_handle cipher, haflo_handle exponents, size_t rows,
                   size_t cols, uint32_t uses, haflo_handle* out) {
  if (!s || !out || (orientation != 0 && orientation != 1)) return HAFLO_EINVAL;
  const haflo_handle in[2] = {cipher, exponents};
  const int kinds[2] = {HAFLO_KIND_CIPHER, HAFLO_KIND_I32};
  if (!s->operands_ok(in, kinds, 2)) return HAFLO_EINVAL;
  size_t n_in = orientation == 0 ? rows : cols, n_out = orientation == 0 ? cols : rows;
  if (s->get(cipher)->count != n_in || (cols && rows > (size_t)-1 / cols) || s->get(exponents)->count != rows * cols)
    return HAFLO_EINVAL;
  haflo_handle ho;
  int rc = s->create(HAFLO_KIND_CIPHER, n_out, uses, &ho);
  if (rc != HAFLO_OK) return rc;
  Scratch ws(s);
  if (!ws.take(haflo_workspace_bytes(s->ctx, orientation == 0 ? HAFLO_OP_MATVEC_XT_D : HAFLO_OP_MATVEC_X_W, rows,
                                     cols))) {
    s->drop(ho);
    return HAFLO_ENOMEM;
  }
  rc = haflo_cipher_matvec(s->ctx, orientation, s->ptr(s->get(cipher)), (const int32_t*)s->ptr(s->get(exponents)), rows,
                           cols, s->ptr(s->get(ho)), ws.ptr(), ws.bytes, s->st);
  if (rc != HAFLO_OK) {
    s->drop(ho);
    return rc;
  }
  s->consume(s->get(cipher));
  s->consume(s->get(exponents));
  *out = ho;
  return HAFLO_OK;
}

int haflo_h_sum(haflo_store* s, haflo_handle cipher, uint32_t uses, haflo_handle* out) {
  if (!s || !out) return HAFLO_EINVAL;
  const int kinds[1] = {HAFLO_KIND_CIPHER};
  if (!s->operands_ok(&cipher, kinds, 1)) return HAFLO_EINVAL;
  size_t count = s->get(cipher)->count;
  haflo_handle ho;
  int rc = s->create(HAFLO_KIND_CIPHER, 1, uses, &ho);
  if (rc != HAFLO_OK) return rc;
  Scratch ws(s);
  if (!ws.take(haflo_workspace_bytes(s->ctx, HAFLO_OP_MATVEC_XT_D, count, 1))) {
    s->drop(ho);
    return HAFLO_ENOMEM;
  }
  rc = haflo_cipher_sum(s->ctx, s->ptr(s->get(cipher)), count, s->ptr(s->get(ho)), ws.ptr(), ws.bytes, s->st);
  if (rc != HAFLO_OK) {
    s->drop(ho);
    return rc;
  }
  s->consume(s->get(cipher));
  *out = ho;
  return HAFLO_OK;
}

}  // extern "C"
