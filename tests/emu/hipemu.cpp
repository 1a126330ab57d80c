// Fiber scheduler behind the CPU stand-in for the HIP runtime (tests only).
#include <hip/hip_runtime.h>
#include <sys/mman.h>
#include <ucontext.h>
#include <unistd.h>

#include <execinfo.h>
#include <signal.h>

#include <map>
#include <vector>

namespace hipemu {

namespace {
constexpr int kWave = 64;
constexpr size_t kStack = 256 * 1024;

struct Lane {
  LaneState st;
  ucontext_t ctx;
  bool done = false;
  int wave = 0, lane = 0;
  uint64_t ops = 0;  // cross-lane operations issued so far
  char* stack = nullptr;
};
struct WaveSlots {
  uint32_t val[2][kWave];
  uint64_t op[2][kWave];
};

std::vector<Lane> lanes;
std::vector<WaveSlots> waves;
Lane* cur = nullptr;
ucontext_t sched;
const std::function<void()>* body = nullptr;
int live = 0;
int bar_arrived = 0;
uint64_t bar_gen = 0;

void die(const char* msg) {
  fprintf(stderr, "hipemu: %s\n", msg);
  fflush(stderr);
  abort();
}

void yield() { swapcontext(&cur->ctx, &sched); }

void trampoline() {
  (*body)();
  cur->done = true;
  --live;
}

// publish v for this wave-wide operation, switch away, and return the table of
// the values all 64 lanes published for the same operation
const uint32_t* exchange(uint32_t v) {
  Lane* me = cur;
  WaveSlots& w = waves[me->wave];
  int par = (int)(me->ops & 1);
  uint64_t id = me->ops++;
  w.val[par][me->lane] = v;
  w.op[par][me->lane] = id;
  yield();
  int nl = (int)lanes.size();
  for (int l = 0; l < kWave; ++l) {
    int gl = me->wave * kWave + l;
    if (gl >= nl) die("wave not fully populated");
    if (w.op[par][l] != id) die("divergent cross-lane operation inside a wave (or a lane exited early)");
  }
  return w.val[par];
}
}  // namespace

LaneState* current() { return &cur->st; }

uint32_t bpermute(int byte_addr, uint32_t v) {
  const uint32_t* t = exchange(v);
  return t[((unsigned)byte_addr >> 2) & (kWave - 1)];
}

uint32_t dpp(uint32_t old, uint32_t src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl) {
  int lane = cur->lane;
  const uint32_t* t = exchange(src);
  int row = lane & ~15, pos = lane & 15;
  // lanes outside the enabled rows and banks keep `old`
  if (!((row_mask >> (lane >> 4)) & 1) || !((bank_mask >> (pos >> 2)) & 1)) return old;
  int from = -1;
  if (ctrl >= 0x101 && ctrl <= 0x10f) {  // row_shl:n - lane i reads lane i+n
    int s = pos + (ctrl - 0x100);
    if (s < 16) from = row + s;
  } else if (ctrl >= 0x111 && ctrl <= 0x11f) {  // row_shr:n - lane i reads lane i-n
    int s = pos - (ctrl - 0x110);
    if (s >= 0) from = row + s;
  } else if (ctrl == 0x130) {  // wave_shl:1 - lane i reads lane i+1 of the wavefront
    if (lane + 1 < kWave) from = lane + 1;
  } else if (ctrl == 0x138) {  // wave_shr:1 - lane i reads lane i-1 of the wavefront
    if (lane >= 1) from = lane - 1;
  } else if (ctrl >= 0x150 && ctrl <= 0x15f) {  // row_newbcast:n - every lane of a row reads its lane n
    from = row + (ctrl - 0x150);
  } else if (ctrl >= 0 && ctrl <= 0xff) {  // quad_perm
    from = (lane & ~3) + ((ctrl >> (2 * (lane & 3))) & 3);
  } else {
    die("unsupported DPP control");
  }
  if (from < 0) return bound_ctrl ? 0u : old;
  return t[from];
}

uint32_t readlane(uint32_t v, int src_lane) {
  const uint32_t* t = exchange(v);
  return t[src_lane & (kWave - 1)];
}

uint64_t ballot(bool p) {
  const uint32_t* t = exchange(p ? 1u : 0u);
  uint64_t m = 0;
  for (int l = 0; l < kWave; ++l)
    if (t[l]) m |= 1ull << l;
  return m;
}

void barrier() {
  uint64_t gen = bar_gen;
  ++bar_arrived;
  if (bar_arrived == live) {
    bar_arrived = 0;
    ++bar_gen;
    return;
  }
  while (bar_gen == gen) yield();
}

void launch(dim3 grid, dim3 block, const std::function<void()>& fn) {
  if (block.y != 1 || block.z != 1 || grid.y != 1 || grid.z != 1) die("only 1-D launches are emulated");
  if (block.x == 0 || block.x % kWave) die("block size must be a multiple of 64");
  if (cur) die("nested launch");
  size_t nthreads = block.x;
  if (lanes.size() != nthreads) {
    for (Lane& l : lanes) free(l.stack);
    lanes.assign(nthreads, Lane());
    for (Lane& l : lanes) l.stack = (char*)malloc(kStack);
  }
  waves.assign(nthreads / kWave, WaveSlots());
  body = &fn;
  for (unsigned b = 0; b < grid.x; ++b) {
    for (size_t t = 0; t < nthreads; ++t) {
      Lane& l = lanes[t];
      l.st.tid = dim3((unsigned)t);
      l.st.bid = dim3(b);
      l.st.bdim = block;
      l.st.gdim = grid;
      l.done = false;
      l.ops = 0;
      l.wave = (int)(t / kWave);
      l.lane = (int)(t % kWave);
      getcontext(&l.ctx);
      l.ctx.uc_stack.ss_sp = l.stack;
      l.ctx.uc_stack.ss_size = kStack;
      l.ctx.uc_link = &sched;
      makecontext(&l.ctx, trampoline, 0);
    }
    for (WaveSlots& w : waves) memset(&w, 0xff, sizeof(w));
    live = (int)nthreads;
    bar_arrived = 0;
    while (live > 0) {
      for (size_t t = 0; t < nthreads; ++t) {
        if (lanes[t].done) continue;
        cur = &lanes[t];
        swapcontext(&sched, &lanes[t].ctx);
      }
    }
    cur = nullptr;
  }
  body = nullptr;
}

// device memory: the buffer ends right at an inaccessible page
namespace {
std::map<void*, std::pair<void*, size_t>> allocs;
std::map<void*, size_t> alloc_bytes;

// an out-of-bounds access: say which lane did it and which buffer it ran off
void on_fault(int, siginfo_t* si, void*) {
  char* addr = (char*)si->si_addr;
  fprintf(stderr, "hipemu: memory fault at %p", (void*)addr);
  if (cur) fprintf(stderr, " in block %u thread %u", cur->st.bid.x, cur->st.tid.x);
  for (auto& kv : allocs) {
    char* base = (char*)kv.second.first;
    if (addr >= base && addr < base + kv.second.second)
      fprintf(stderr, ": %ld bytes past the start of a %zu-byte buffer", (long)(addr - (char*)kv.first),
              alloc_bytes[kv.first]);
  }
  fprintf(stderr, "\n");
  void* frames[32];
  int nf = backtrace(frames, 32);
  backtrace_symbols_fd(frames, nf, 2);
  _exit(139);
}
void install_handler() {
  static bool done = false;
  if (done) return;
  done = true;
  static char altstack[1 << 16];
  stack_t ss;
  ss.ss_sp = altstack;
  ss.ss_size = sizeof(altstack);
  ss.ss_flags = 0;
  sigaltstack(&ss, nullptr);
  struct sigaction sa;
  memset(&sa, 0, sizeof(sa));
  sa.sa_sigaction = on_fault;
  sa.sa_flags = SA_SIGINFO | SA_ONSTACK;
  sigaction(SIGSEGV, &sa, nullptr);
}
}
void* dev_alloc(size_t bytes) {
  size_t page = (size_t)sysconf(_SC_PAGESIZE);
  size_t want = (bytes + 15) & ~(size_t)15;
  if (want == 0) want = 16;
  size_t body_pages = (want + page - 1) / page;
  size_t total = (body_pages + 1) * page;
  char* base = (char*)mmap(nullptr, total, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS, -1, 0);
  if (base == MAP_FAILED) return nullptr;
  mprotect(base + body_pages * page, page, PROT_NONE);
  char* p = base + body_pages * page - want;
  memset(base, 0xCD, body_pages * page);
  allocs[p] = std::make_pair((void*)base, total);
  alloc_bytes[p] = bytes;
  install_handler();
  return p;
}
void dev_free(void* p) {
  auto it = allocs.find(p);
  if (it == allocs.end()) return;
  munmap(it->second.first, it->second.second);
  alloc_bytes.erase(p);
  allocs.erase(it);
}

}  // namespace hipemu

// test harness entry points: guarded "device" buffers for the Python side
extern "C" {
void* hipemu_alloc(size_t bytes) { return hipemu::dev_alloc(bytes); }
void hipemu_free(void* p) { hipemu::dev_free(p); }
}
