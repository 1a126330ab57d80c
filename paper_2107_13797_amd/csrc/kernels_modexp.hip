// Exponentiation-bound operators: encryption, decryption through p^2 and q^2,
// ciphertext-by-scalar multiplication. Kernels and their C entry points.
#include <mutex>

#include "kernels_common.hpp"

using namespace haflo;
using namespace haflo::dev;

// Scratch of the entry point that allocates nothing (haflo_decrypt_static): every GPU the library runs on
// holds its own copy of this array, at its own address, until the process ends. In host code the name is
// only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[HAFLO_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once resolved

int decrypt_launches(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_plain, size_t count, void* d_workspace,
                     hipStream_t st);

constexpr int kModexpBlocksPerCu = 4;  // resident blocks assumed when sizing window-table workspace

// Decryption stage A: internal ciphertext -> canonical residue mod n^2 in
// 29-bit limbs (workspace), ready to be split in halves.
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_dec_unmont(ModRef M, const u32* __restrict__ in,
                                                              u32* __restrict__ canon29, size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  u32 one[LPT];
  zero_limbs<LPT>(one);
  if (g.k == 0) one[0] = 1u;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 x[LPT];
    if (active) load_limbs<LPT, T>(x, in + item * (size_t)NL, g);
    else zero_limbs<LPT>(x);
    montmul<LPT, T>(x, x, one, mod.n, mod.n0inv, g);
    canonicalise<LPT, T>(x, mod.n, g);
    if (active) store_limbs<LPT, T>(canon29 + item * (size_t)NL, x, g);
  }
}

// m_s = L_s(y) * h_s mod s for y = c^(s-1) mod s^2 (canonical, 2*NL limbs of
// which only the low NL matter): L_s(y) = (y - 1)/s is an exact quotient below
// s < 2^(29 NL), so it equals (y - 1) * s^-1 modulo 2^(29 NL). With `quotient` set,
// ylow already holds L_s(y) (NL canonical limbs).
template <int LPT, int T>
__device__ __forceinline__ void crt_branch(u32 (&ms)[LPT], const u32* ylow, bool active, int quotient,
                                           const ModRegs<LPT>& mod, const u32* sinv, const u32* hsR, const Grp<T>& g) {
  u32 x[LPT], t[LPT];
  if (active) load_limbs<LPT, T>(x, ylow, g);
  else zero_limbs<LPT>(x);
  if (!quotient) {  // uniform over the launch
    s32 d[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) d[j] = (s32)x[j];
    if (g.k == 0) d[0] -= 1;
    resolve<LPT, T>(d, g);  // modulo 2^(29 NL): a borrow out of the top is dropped
#pragma unroll
    for (int j = 0; j < LPT; ++j) x[j] = (u32)d[j];
    load_limbs<LPT, T>(t, sinv, g);
    mullo<LPT, T>(x, x, t, g);
  }
  load_limbs<LPT, T>(t, hsR, g);
  montmul<LPT, T>(ms, x, t, mod.n, mod.n0inv, g);
  canonicalise<LPT, T>(ms, mod.n, g);
}

// Decryption stage C: both branches, then the Chinese remainder
// m = m_p + p * ((m_q - m_p) * p^-1 mod q), written as Lp 32-bit words.
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_dec_crt(ModRef MP, ModRef MQ, const u32* __restrict__ pinv2,
                                                           const u32* __restrict__ qinv2, const u32* __restrict__ hpR,
                                                           const u32* __restrict__ hqR, const u32* __restrict__ pinvqR,
                                                           const u32* __restrict__ yp, const u32* __restrict__ yq,
                                                           int quotients, u32* __restrict__ plain, int lp,
                                                           size_t count) {
  constexpr int NL = LPT * T;
  __shared__ u32 stage[kBlockThreads * LPT * 2];
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mp, mq;
  load_mod<LPT, T>(mp, MP, g);
  load_mod<LPT, T>(mq, MQ, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 a[LPT], b[LPT], t[LPT], u[LPT];
    const size_t ystride = quotients ? NL : 2 * NL;
    crt_branch<LPT, T>(a, yp + item * ystride, active, quotients, mp, pinv2, hpR, g);  // m_p
    crt_branch<LPT, T>(b, yq + item * ystride, active, quotients, mq, qinv2, hqR, g);  // m_q
    // (m_q - m_p) mod q; m_p < p < 2q so one conditional subtraction reduces it
#pragma unroll
    for (int j = 0; j < LPT; ++j) t[j] = a[j];
    canonicalise<LPT, T>(t, mq.n, g);
    sub_mod<LPT, T>(u, b, t, mq.n, g);
    load_limbs<LPT, T>(t, pinvqR, g);
    montmul<LPT, T>(u, u, t, mq.n, mq.n0inv, g);
    canonicalise<LPT, T>(u, mq.n, g);
    // p * u as a 2*NL-limb product: low half, then high half
    u32 lo[LPT], hi[LPT];
    mulwide<LPT, T>(lo, hi, mp.n, u, g);
#pragma unroll
    for (int j = 0; j < LPT; ++j) lo[j] += a[j];
    int carry = resolve<LPT, T>(lo, g);
    if (g.k == 0) hi[0] += (u32)carry;
    resolve<LPT, T>(hi, g);
    u32* mine = stage + bt.gib * (2 * NL);
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      mine[g.k * LPT + j] = lo[j];
      mine[NL + g.k * LPT + j] = hi[j];
    }
    __syncthreads();
    if (active)
      for (int w = g.k; w < lp; w += T) plain[item * (size_t)lp + w] = word_from_limbs(mine, 2 * NL, w);
    __syncthreads();
  }
}

// Key owner's encryption, recombination: from y_p = r^n mod p^2 and y_q = r^n mod q^2
// (canonical) to r^n mod n^2 = y_p + p^2 ((y_q - y_p) (p^2)^-1 mod q^2), written as the
// 2*NL limbs of a residue modulo n^2 (low half, high half).
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_enc_crt(ModRef MP2, ModRef MQ2, const u32* __restrict__ p2invR,
                                                           const u32* __restrict__ yp, const u32* __restrict__ yq,
                                                           u32* __restrict__ rn, size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mp, mq;
  load_mod<LPT, T>(mp, MP2, g);
  load_mod<LPT, T>(mq, MQ2, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 a[LPT], b[LPT], t[LPT], u[LPT];
    if (active) {
      load_limbs<LPT, T>(a, yp + item * (size_t)NL, g);
      load_limbs<LPT, T>(b, yq + item * (size_t)NL, g);
    } else {
      zero_limbs<LPT>(a);
      zero_limbs<LPT>(b);
    }
    // y_p < p^2 < 2 q^2: one conditional subtraction reduces it modulo q^2
#pragma unroll
    for (int j = 0; j < LPT; ++j) t[j] = a[j];
    canonicalise<LPT, T>(t, mq.n, g);
    sub_mod<LPT, T>(u, b, t, mq.n, g);
    load_limbs<LPT, T>(t, p2invR, g);
    montmul<LPT, T>(u, u, t, mq.n, mq.n0inv, g);
    canonicalise<LPT, T>(u, mq.n, g);
    u32 lo[LPT], hi[LPT];
    mulwide<LPT, T>(lo, hi, mp.n, u, g);
#pragma unroll
    for (int j = 0; j < LPT; ++j) lo[j] += a[j];
    int carry = resolve<LPT, T>(lo, g);
    if (g.k == 0) hi[0] += (u32)carry;
    resolve<LPT, T>(hi, g);
    if (active) {
      store_limbs<LPT, T>(rn + item * (size_t)(2 * NL), lo, g);
      store_limbs<LPT, T>(rn + item * (size_t)(2 * NL) + NL, hi, g);
    }
  }
}

// A batch that leaves most of the chip idle is latency-bound. Up to two chains per SIMD, each gets a
// wavefront to itself (a few limbs per lane: the shortest steps); beyond that, while twice the lanes still
// are at most two wavefronts per SIMD, its integers are spread over twice the lanes (9 limbs each), which
// shortens every product of the chain at 1.2 times the instructions. `jobs`: independent halves of one launch.
// `nine`: take 9 limbs per lane (twice the lanes per integer) also for a batch that fills the chip.
int engine_geo(const haflo_ctx* ctx, size_t count, const ModHost& m, int jobs = 1, bool nine = false) {
  // up to two chains per SIMD (measured: 2048 encryptions at a 1024-bit key 4.4 ms against 5.2 ms at nine limbs
  // per lane, 1024 decryptions 0.91 against 1.37 ms; three per SIMD no longer gain)
  if (haflo_has_wave_geometry(m) && count * (size_t)jobs <= (size_t)ctx->num_cu * 4 * 2) return kGeoWave;
  if (m.lpt == 18 && m.t < 16 && (nine || count * (size_t)jobs * (size_t)m.t <= (size_t)ctx->num_cu * 256)) return kGeoWide;
  return kGeoPlain;
}
LaunchShape modexp_shape(const haflo_ctx* ctx, size_t count, const ModHost& m, int jobs = 1, bool nine = false) {
  const int geo = engine_geo(ctx, count, m, jobs, nine);
  LaunchShape s;
  if (geo == kGeoWave) {
    s.blocks = (int)(count ? count : 1);
    s.threads = 64;
    s.gpb = 1;
  } else {
    s = launch_shape(ctx, count, geo == kGeoWide ? 2 * m.t : m.t, kModexpBlocksPerCu);
  }
  s.geo = geo;
  return s;
}

EngineIO engine_io(const ModHost& m) {
  EngineIO io = {};
  const ModRef r = m.ref();
  io.constant[kConstR1] = r.r1;
  io.constant[kConstR2] = r.r2;
  io.constant[kConstR3] = r.r3;
  io.constant[kConstOne] = r.one;
  io.constant[kConstExtra] = nullptr;
  return io;
}

bool to_inline(ProgInline& pi, const std::vector<uint32_t>& prog) {
  if (prog.size() > (size_t)kInlineProgMax) return false;
  pi.len = (int)prog.size();
  for (size_t i = 0; i < prog.size(); ++i) pi.ins[i] = prog[i];
  return true;
}

template <class Prog>
int launch_engine(const ModHost& m, const LaunchShape& sh, hipStream_t st, const Prog& prog, const EngineIO& io,
                  size_t count) {
#define CALL(LPT, T) HAFLO_LAUNCH((k_engine<LPT, T, Prog>), sh, st, m.ref(), prog, io, count)
  if (sh.geo == kGeoWave) { HAFLO_DISPATCH_GEOMETRY_WAVE(m, CALL); }
  else if (sh.geo == kGeoWide) { HAFLO_DISPATCH_GEOMETRY_WIDE(m, CALL); }
  else { HAFLO_DISPATCH_GEOMETRY(m, CALL); }
#undef CALL
  return hip_status(hipGetLastError());
}

// One element is one sequential chain, so a batch that does not fill its last pass over the resident
// lane groups would still pay for it in full. Such a batch is cut in two launches: the full passes, and
// the remainder in single-wavefront blocks that spread over all SIMDs (and over twice the lanes per
// integer when it is small), which runs the fewer wavefronts per SIMD correspondingly faster.
struct BatchSplit {
  size_t full;       // elements of the full passes (0: one launch of `shape` for everything)
  LaunchShape shape; // of the full passes, or of the only launch
  LaunchShape tail;  // of the remainder
};
BatchSplit split_batch(const haflo_ctx* ctx, size_t count, const ModHost& m) {
  BatchSplit b;
  b.shape = modexp_shape(ctx, count, m);
  b.full = 0;
  b.tail = b.shape;
  const size_t slots = b.shape.slots();
  if (b.shape.geo != kGeoPlain || count <= slots || count % slots == 0) return b;
  b.full = count / slots * slots;
  const size_t rest = count - b.full;
  b.tail.geo = engine_geo(ctx, rest, m);
  const int t = b.tail.geo == kGeoWave ? 64 : (b.tail.geo == kGeoWide ? 2 * m.t : m.t);
  b.tail.threads = 64;
  b.tail.gpb = 64 / t;
  b.tail.blocks = (int)((rest + b.tail.gpb - 1) / b.tail.gpb);
  return b;
}

// `io` with the constants of the pair arithmetic modulo ms^2 in place of those of the plain engine
EngineIO pair_io(const ModHost& ms, EngineIO io) {
  for (int i = 0; i < kNumConst; ++i) io.constant[i] = ms.d_pairs + (size_t)i * 2 * ms.nl;
  io.out_mode = kOutInteger;
  return io;
}

// Two jobs of the pair engine in one launch (moduli p and q, 9 limbs per lane)
int launch_engine_pairs2(const ModHost& mh, const LaunchShape& sh, hipStream_t st, const EngineJob& j0,
                         const EngineJob& j1, unsigned split, size_t count) {
#define CALL(T) HAFLO_LAUNCH((k_engine_pairs2<9, T>), sh, st, j0, j1, split, count)
  if (sh.geo == kGeoWave) {
    // one pair per wavefront: 36 lanes with 2 limbs of each half
    if (mh.nl != 72) return HAFLO_EINVAL;
    HAFLO_LAUNCH((k_engine_pairs2<2, 36>), sh, st, j0, j1, split, count);
    return hip_status(hipGetLastError());
  }
  if (mh.lpt == 9 && mh.t == 1) {
    CALL(1);
    return hip_status(hipGetLastError());
  }
  if (mh.lpt != 18) return HAFLO_EINVAL;
  switch (mh.t) {
    case 1: CALL(2); break;
    case 2: CALL(4); break;
    case 4: CALL(8); break;
    case 8: CALL(16); break;
    default: return HAFLO_EINVAL;
  }
#undef CALL
  return hip_status(hipGetLastError());
}

// The pair engine (residues modulo n^2 as pairs modulo n) for the elements of full passes: `mh` is n at half
// the limbs of n^2, spread over as many lanes per element as n^2 itself takes (9 limbs per lane).
template <class Prog>
int launch_engine_pairs(const ModHost& mh, const LaunchShape& sh, hipStream_t st, const Prog& prog,
                        const EngineIO& io, size_t count) {
#define CALL(T) HAFLO_LAUNCH((k_engine_pairs<9, T, Prog>), sh, st, mh.ref(), prog, io, count)
  if (sh.geo == kGeoWave) {
    // one pair per wavefront: 36 lanes of 2 limbs or 48 lanes of 3 limbs for each half
    if (mh.nl == 72) HAFLO_LAUNCH((k_engine_pairs<2, 36, Prog>), sh, st, mh.ref(), prog, io, count);
    else if (mh.nl == 144) HAFLO_LAUNCH((k_engine_pairs<3, 48, Prog>), sh, st, mh.ref(), prog, io, count);
    else return HAFLO_EINVAL;
    return hip_status(hipGetLastError());
  }
  if (mh.lpt != 18) return HAFLO_EINVAL;
  switch (mh.t) {
    case 1: CALL(2); break;
    case 2: CALL(4); break;
    case 4: CALL(8); break;
    case 8: CALL(16); break;
    default: return HAFLO_EINVAL;
  }
#undef CALL
  return hip_status(hipGetLastError());
}

template <class Prog>
int launch_engine_batch(const haflo_ctx* ctx, const ModHost& m, hipStream_t st, const Prog& prog, EngineIO io,
                        size_t count) {
  const BatchSplit b = split_batch(ctx, count, m);
  if (b.full == 0) return launch_engine(m, b.shape, st, prog, io, count);
  int rc = launch_engine(m, b.shape, st, prog, io, b.full);
  if (rc != HAFLO_OK) return rc;
  io.first = b.full;  // the table slots are free again once the first launch has finished (stream order)
  return launch_engine(m, b.tail, st, prog, io, count - b.full);
}

// A power of stored ciphertexts (`prog` begins with ENG_LOAD_L 0 and leaves the power in Montgomery form):
// the full passes of a batch that fills the chip run the same program on pairs modulo n, with the element
// taken into the pair form first and out of it at the end; what is left over runs as it is.
int launch_power_batch(const haflo_ctx* ctx, hipStream_t st, const ProgInline& pi, const std::vector<uint32_t>& prog,
                       EngineIO io, size_t count) {
  const ModHost& m = ctx->N;
  const BatchSplit b = split_batch(ctx, count, m);
  std::vector<uint32_t> pp;
  pp.push_back(eng_ins(ENG_LOAD_L, 1));
  pp.push_back(eng_ins(ENG_MUL_C, kConstR5));
  pp.push_back(eng_ins(ENG_STORE_T, 0));
  pp.push_back(eng_ins(ENG_LOAD_L, 0));
  pp.push_back(eng_ins(ENG_MUL_C, kConstR4));
  pp.push_back(eng_ins(ENG_ADD_T, 0));
  pp.insert(pp.end(), prog.begin() + 1, prog.end());
  pp.push_back(eng_ins(ENG_MUL_C, kConstR3));
  ProgInline ppi;
  if (b.shape.geo != kGeoPlain || prog.empty() || prog[0] != eng_ins(ENG_LOAD_L, 0) || !to_inline(ppi, pp))
    return launch_engine_batch(ctx, m, st, pi, io, count);
  const size_t full = b.full ? b.full : count;
  int rc = launch_engine_pairs(ctx->Nh, b.shape, st, ppi, pair_io(ctx->Nh, io), full);
  if (rc != HAFLO_OK || full == count) return rc;
  io.first = full;
  if (b.tail.geo == kGeoPlain) return launch_engine_pairs(ctx->Nh, b.tail, st, ppi, pair_io(ctx->Nh, io), count - full);
  return launch_engine(m, b.tail, st, pi, io, count - full);
}

}  // namespace

namespace haflo {
// Resolves the device address of the static scratch array on the current device (once per device) and
// keeps it. Called when a context is created, with the context's device current.
int static_scratch_init() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return HAFLO_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return HAFLO_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev]) return HAFLO_OK;
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return HAFLO_EHIP;
  g_scratch_ptr[dev] = ptr;
  return HAFLO_OK;
}

// table slots: one set per resident lane group
size_t ws_encrypt(const haflo_ctx* ctx, size_t count) {
  if (!ctx->has_priv)
    return modexp_shape(ctx, count, ctx->N).slots() * (size_t)ctx->prog_enc.table_entries * ctx->N.nl * 4;
  // key owner: [y_p, y_q: count*P2.nl each][r^n: count*N.nl; before it is written, the first
  // stage's results: count*P.nl for each prime][tables of whichever stage runs, both halves of the
  // grid; for the last stage one table slot of N.nl limbs per lane group]
  size_t tl1 = (size_t)std::max(ctx->prog_enc_p.table_entries, ctx->prog_enc_q.table_entries);
  size_t tl2 = (size_t)std::max(ctx->prog_lift_p.table_entries, ctx->prog_lift_q.table_entries);
  size_t low = 2 * modexp_shape(ctx, count, ctx->P, 2, ctx->P.t <= 2).slots() * tl1 * ctx->P.nl;
  size_t lift = 2 * modexp_shape(ctx, count, ctx->P2, 2).slots() * tl2 * ctx->P2.nl;
  size_t last = modexp_shape(ctx, count, ctx->N).slots() * (size_t)ctx->N.nl;
  return (2 * count * (size_t)ctx->P2.nl + count * (size_t)ctx->N.nl + std::max(std::max(low, lift), last)) * 4;
}
// one table slot per resident lane group
size_t ws_encrypt_obf(const haflo_ctx* ctx, size_t count) {
  return launch_shape(ctx, count, haflo_wide_lanes(ctx->N), 8).slots() * (size_t)ctx->N.nl * 4;
}
// sized for the per-element variant (16 entries); the broadcast variant never needs more
size_t ws_scalar_mul(const haflo_ctx* ctx, size_t count) {
  return modexp_shape(ctx, count, ctx->N).slots() * (size_t)16 * ctx->N.nl * 4;
}
// layout: [canon29: count*N.nl][yp: count*P2.nl][yq: count*Q2.nl][tables]
size_t ws_decrypt(const haflo_ctx* ctx, size_t count) {
  if (!ctx->has_priv) return 0;
  size_t tl = (size_t)std::max(ctx->prog_dec_p.table_entries, ctx->prog_dec_q.table_entries);
  return (count * (size_t)ctx->N.nl + 2 * count * (size_t)ctx->P2.nl +
          2 * modexp_shape(ctx, count, ctx->P2, 2).slots() * tl * ctx->P2.nl) * 4;
}

// tables[i][d] = c_i^d, d < entries, for `count` internal ciphertexts (used by the matvec)
int power_tables(const haflo_ctx* ctx, const uint32_t* d_c, uint32_t* d_tables, int entries, size_t count,
                 hipStream_t st) {
  const ModHost& m = ctx->N;
  std::vector<uint32_t> prog;
  prog.push_back(eng_ins(ENG_LOAD_L, 0));
  append_power_table(prog, entries);
  ProgInline pi;
  if (!to_inline(pi, prog)) return HAFLO_EINVAL;
  EngineIO io = engine_io(m);
  io.in_limbs = d_c;
  io.in_limbs_stride = m.nl;
  io.tables = d_tables;
  io.table_entries = entries;
  io.table_per_item = 1;
  // 9 limbs per lane: the 18-limb form of the engine spills registers
  LaunchShape sh = launch_shape(ctx, count, haflo_wide_lanes(m), 8);
  sh.geo = m.lpt == 18 && m.t < 16 ? kGeoWide : kGeoPlain;
  return launch_engine(m, sh, st, pi, io, count);
}
}  // namespace haflo

extern "C" {

int haflo_encrypt(const haflo_ctx* ctx, const uint32_t* d_plain, const uint32_t* d_r, void* d_cipher, size_t count,
                  void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || (count && (!d_plain || !d_r || !d_cipher))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_encrypt(ctx, count)) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  hipStream_t st = (hipStream_t)stream;
  if (!ctx->has_priv) {
    // public key: r^n with the full exponent modulo n^2
    EngineIO io = engine_io(m);
    io.constant[kConstExtra] = ctx->d_k1;
    io.in_words[0] = d_plain;
    io.in_words[1] = d_r;
    io.in_nwords = ctx->lp;
    io.out = (u32*)d_cipher;
    io.tables = (u32*)d_workspace;
    io.table_entries = ctx->prog_enc.table_entries;
    ProgPtr prog = {ctx->prog_enc.d_ins, (int)ctx->prog_enc.host.size()};
    const BatchSplit b = split_batch(ctx, count, m);
    // one integer per wavefront: from 2048-bit keys on the pair arithmetic pays there too (half the steps of a
    // product, each with two accumulator windows: 4 % off the chain at 2048 bits, 11 % at 4096)
    const bool wave_pairs = b.shape.geo == kGeoWave && (ctx->Nh.nl == 72 || ctx->Nh.nl == 144);
    if (b.shape.geo != kGeoPlain && !wave_pairs) return launch_engine(m, b.shape, st, prog, io, count);
    // a batch that fills the chip: the pair arithmetic modulo n (5/8 of the limb products of a product,
    // 0.57 of those of a squaring) for the full passes, the engine above for what is left over
    EngineIO pio = pair_io(ctx->Nh, io);
    pio.table_entries = ctx->prog_enc_pairs.table_entries;
    ProgPtr pprog = {ctx->prog_enc_pairs.d_ins, (int)ctx->prog_enc_pairs.host.size()};
    const size_t full = b.full ? b.full : count;
    int rc = launch_engine_pairs(ctx->Nh, b.shape, st, pprog, pio, full);
    if (rc != HAFLO_OK || full == count) return rc;
    // what is left over: on pairs as well while it still is a batch of many wavefronts, else the engine above
    // in the geometry of a small batch
    if (b.tail.geo == kGeoPlain) {
      pio.first = full;
      return launch_engine_pairs(ctx->Nh, b.tail, st, pprog, pio, count - full);
    }
    io.first = full;
    return launch_engine(m, b.tail, st, prog, io, count - full);
  }
  // key owner: r^n modulo p^2 and q^2, each as (r^(n mod (s-1)) mod s)^s mod s^2 (a half-length
  // exponent on the quarter-size modulus, then a half-length exponent on the half-size one),
  // Chinese remainder, then the (1 + m n) factor and the Montgomery form modulo n^2.
  // Bit-identical to the public path: the residue r^n mod n^2 is unique.
  const ModHost& h = ctx->P2;
  const ModHost& l = ctx->P;
  u32* yp = (u32*)d_workspace;
  u32* yq = yp + count * (size_t)h.nl;
  u32* rn = yq + count * (size_t)h.nl;
  u32* tables = rn + count * (size_t)m.nl;
  u32* y0p = rn;  // the first stage's results live where r^n goes later
  u32* y0q = y0p + count * (size_t)l.nl;
  for (int stage = 0; stage < 2; ++stage) {
    const ModHost& geo = stage ? h : l;
    const DevProg* progs[2] = {stage ? &ctx->prog_lift_p : &ctx->prog_enc_p, stage ? &ctx->prog_lift_q : &ctx->prog_enc_q};
    const int tl = std::max(progs[0]->table_entries, progs[1]->table_entries);
    // the first stage (plain residues modulo the primes) runs faster on 9 limbs per lane at any batch size up
    // to 2048-bit keys (measured: 18.9 -> 15.6 ms per 65536 there, 112 -> 114.5 ms at 4096 bits)
    LaunchShape sh = modexp_shape(ctx, count, geo, 2, stage == 0 && geo.t <= 2);
    EngineJob job[2];
    for (int side = 0; side < 2; ++side) {
      const ModHost& ms = stage ? (side ? ctx->Q2 : ctx->P2) : (side ? ctx->Q : ctx->P);
      job[side].M = ms.ref();
      job[side].P = ProgPtr{progs[side]->d_ins, (int)progs[side]->host.size()};
      job[side].io = engine_io(ms);
      if (stage == 0) {
        job[side].io.in_words[1] = d_r;
        job[side].io.in_nwords = ctx->lp;
        job[side].io.out = side ? y0q : y0p;
      } else {
        job[side].io.in_limbs = side ? y0q : y0p;
        job[side].io.in_limbs_stride = l.nl;
        job[side].io.in_limbs_valid = l.nl;
        job[side].io.out = side ? yq : yp;
      }
      job[side].io.tables = tables + (side ? sh.slots() * (size_t)tl * ms.nl : 0);
      job[side].io.table_entries = tl;
    }
    const unsigned split = (unsigned)sh.blocks;
    sh.blocks *= 2;
    if (stage == 1 && (sh.geo == kGeoPlain || (sh.geo == kGeoWave && ctx->P.nl == 72))) {
      // a batch that fills the chip (or, at a 4096-bit key, one integer per wavefront): the second stage on pairs
      // modulo the primes (same result, the canonical integer modulo the prime's square, from about 0.6 of the
      // limb products)
      for (int side = 0; side < 2; ++side) {
        const ModHost& ms = side ? ctx->Q : ctx->P;
        const DevProg& dp = side ? ctx->prog_lift_pairs_q : ctx->prog_lift_pairs_p;
        job[side].M = ms.ref();
        job[side].P = ProgPtr{dp.d_ins, (int)dp.host.size()};
        job[side].io = pair_io(ms, job[side].io);
      }
      int rc = launch_engine_pairs2(ctx->P, sh, st, job[0], job[1], split, count);
      if (rc != HAFLO_OK) return rc;
      continue;
    }
#define CALL(LPT, T) HAFLO_LAUNCH((k_engine_pair<LPT, T>), sh, st, job[0], job[1], split, count)
    if (sh.geo == kGeoWave) { HAFLO_DISPATCH_GEOMETRY_WAVE(geo, CALL); }
    else if (sh.geo == kGeoWide) { HAFLO_DISPATCH_GEOMETRY_WIDE(geo, CALL); }
    else { HAFLO_DISPATCH_GEOMETRY(geo, CALL); }
#undef CALL
  }
  {
    const LaunchShape sh = launch_shape(ctx, count, h.t, 8);
#define CALL(LPT, T)                                                                                  \
  HAFLO_LAUNCH((k_enc_crt<LPT, T>), sh, st, ctx->P2.ref(), ctx->Q2.ref(), (const u32*)ctx->d_p2inv,   \
               (const u32*)yp, (const u32*)yq, rn, count)
    HAFLO_DISPATCH_GEOMETRY(h, CALL);
#undef CALL
  }
  // acc = m -> (m n) R + R = (1 + m n) R -> times r^n (plain) -> times R^2: Montgomery form of E(m)
  std::vector<uint32_t> prog;
  prog.push_back(eng_ins(ENG_LOAD_L, 0));
  prog.push_back(eng_ins(ENG_STORE_T, 0));
  prog.push_back(eng_ins(ENG_LOAD_W, 0));
  prog.push_back(eng_ins(ENG_MUL_C, kConstExtra));
  prog.push_back(eng_ins(ENG_ADD_C, kConstR1));
  prog.push_back(eng_ins(ENG_MUL_T, 0));
  prog.push_back(eng_ins(ENG_MUL_C, kConstR2));
  ProgInline pi;
  if (!to_inline(pi, prog)) return HAFLO_EINVAL;
  EngineIO io = engine_io(m);
  io.constant[kConstExtra] = ctx->d_k1;
  io.in_words[0] = d_plain;
  io.in_nwords = ctx->lp;
  io.in_limbs = rn;
  io.in_limbs_stride = m.nl;
  io.out = (u32*)d_cipher;
  io.tables = tables;
  io.table_entries = 1;
  // three products per element: a batch that fills the chip takes 9 limbs per lane in one launch (the 18-limb
  // form of the engine spills registers), smaller ones the geometries of small batches
  if (m.lpt == 18 && m.t < 16 && engine_geo(ctx, count, m) == kGeoPlain) {
    LaunchShape sh = launch_shape(ctx, count, 2 * m.t, kModexpBlocksPerCu);
    sh.geo = kGeoWide;
    return launch_engine(m, sh, st, pi, io, count);
  }
  return launch_engine_batch(ctx, m, st, pi, io, count);
}

int haflo_encrypt_with_obfuscator(const haflo_ctx* ctx, const uint32_t* d_plain, const void* d_obfuscator,
                                  void* d_cipher, size_t count, void* d_workspace, size_t workspace_bytes,
                                  void* stream) {
  if (!ctx || (count && (!d_plain || !d_obfuscator || !d_cipher))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_encrypt_obf(ctx, count)) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  // table[0] = r^n (Montgomery form); acc = m -> (m n) R + R = (1 + m n) R -> times table[0]
  std::vector<uint32_t> prog;
  prog.push_back(eng_ins(ENG_LOAD_L, 0));
  prog.push_back(eng_ins(ENG_STORE_T, 0));
  prog.push_back(eng_ins(ENG_LOAD_W, 0));
  prog.push_back(eng_ins(ENG_MUL_C, kConstExtra));
  prog.push_back(eng_ins(ENG_ADD_C, kConstR1));
  prog.push_back(eng_ins(ENG_MUL_T, 0));
  ProgInline pi;
  if (!to_inline(pi, prog)) return HAFLO_EINVAL;
  EngineIO io = engine_io(m);
  io.constant[kConstExtra] = ctx->d_k1;
  io.in_words[0] = d_plain;
  io.in_nwords = ctx->lp;
  io.in_limbs = (const u32*)d_obfuscator;
  io.in_limbs_stride = m.nl;
  io.out = (u32*)d_cipher;
  io.tables = (u32*)d_workspace;
  io.table_entries = 1;
  // 9 limbs per lane: the 18-limb form of the engine spills registers
  LaunchShape sh = launch_shape(ctx, count, haflo_wide_lanes(m), 8);
  sh.geo = m.lpt == 18 && m.t < 16 ? kGeoWide : kGeoPlain;
  return launch_engine(m, sh, (hipStream_t)stream, pi, io, count);
}

int haflo_scalar_mul_u64(const haflo_ctx* ctx, const void* d_c, const uint64_t* d_k, void* d_out, size_t count,
                         void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || (count && (!d_c || !d_k || !d_out))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_scalar_mul(ctx, count)) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  // fixed 4-bit windows over the table c^0..c^15: every window multiplies (by 1 for a zero
  // digit), so the instruction stream is the same for every element
  std::vector<uint32_t> prog;
  prog.push_back(eng_ins(ENG_LOAD_L, 0));
  append_power_table(prog, 16);
  prog.push_back(eng_ins(ENG_LOAD_TD, 60));
  for (int wi = 14; wi >= 0; --wi) {
    for (int s = 0; s < 4; ++s) prog.push_back(eng_ins(ENG_SQ));
    prog.push_back(eng_ins(ENG_MUL_TD, (uint32_t)(4 * wi)));
  }
  ProgInline pi;
  if (!to_inline(pi, prog)) return HAFLO_EINVAL;
  EngineIO io = engine_io(m);
  io.in_limbs = (const u32*)d_c;
  io.in_limbs_stride = m.nl;
  io.k64 = (const unsigned long long*)d_k;
  io.out = (u32*)d_out;
  io.tables = (u32*)d_workspace;
  io.table_entries = 16;
  return launch_power_batch(ctx, (hipStream_t)stream, pi, prog, io, count);
}

int haflo_scalar_mul_i64_bcast(const haflo_ctx* ctx, const void* d_c, int64_t k, void* d_out, size_t count,
                               void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || (count && (!d_c || !d_out))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_scalar_mul(ctx, count)) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  hipStream_t st = (hipStream_t)stream;
  const u32* src = (const u32*)d_c;
  uint64_t mag = k < 0 ? 0ull - (uint64_t)k : (uint64_t)k;
  if (k < 0) {
    // a negative scalar is a power of the inverse: invert into d_out first
    int rc = invert_batch(ctx, src, (u32*)d_out, count, st);
    if (rc != HAFLO_OK) return rc;
    src = (const u32*)d_out;
  }
  const HostSched plan = make_schedule(Big(mag), 4);
  std::vector<uint32_t> prog;
  prog.push_back(eng_ins(ENG_LOAD_L, 0));
  append_modexp(prog, plan);
  ProgInline pi;
  if (!to_inline(pi, prog)) return HAFLO_EINVAL;
  EngineIO io = engine_io(m);
  io.in_limbs = src;
  io.in_limbs_stride = m.nl;
  io.out = (u32*)d_out;
  io.tables = (u32*)d_workspace;
  io.table_entries = plan.table_len + 1;
  return launch_power_batch(ctx, st, pi, prog, io, count);
}

int haflo_decrypt(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_plain, size_t count, void* d_workspace,
                  size_t workspace_bytes, void* stream) {
  if (!ctx || (count && (!d_cipher || !d_plain))) return HAFLO_EINVAL;
  if (!ctx->has_priv) return HAFLO_ENOPRIV;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_decrypt(ctx, count)) return HAFLO_EINVAL;
  return decrypt_launches(ctx, d_cipher, d_plain, count, d_workspace, (hipStream_t)stream);
}

int haflo_decrypt_static(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_plain, size_t count, void* stream) {
  if (!ctx || (count && (!d_cipher || !d_plain))) return HAFLO_EINVAL;
  if (!ctx->has_priv) return HAFLO_ENOPRIV;
  if (count == 0) return HAFLO_OK;
  if (ws_decrypt(ctx, count) > (size_t)HAFLO_STATIC_SCRATCH_BYTES) return HAFLO_ETOOBIG;
  if (ctx->device < 0 || ctx->device >= kMaxDevices) return HAFLO_EINVAL;
  void* ptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    ptr = g_scratch_ptr[ctx->device];
  }
  if (!ptr) return HAFLO_EHIP;  // the context was created on a device whose array could not be resolved
  // every temporary of the decryption (canonical residues, both branch results, window tables) is
  // written before it is read, so nothing of an earlier call's contents has to be cleared
  return decrypt_launches(ctx, d_cipher, d_plain, count, ptr, (hipStream_t)stream);
}

}  // extern "C"

namespace {
int decrypt_launches(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_plain, size_t count, void* d_workspace,
                     hipStream_t st) {
  int pairs = 0;  // the branch results are the quotients L_s on P.nl limbs, not residues modulo s^2
  u32* canon29 = (u32*)d_workspace;
  u32* yp = canon29 + count * (size_t)ctx->N.nl;
  u32* yq = yp + count * (size_t)ctx->P2.nl;
  u32* tables = yq + count * (size_t)ctx->Q2.nl;
  const int dp_table_entries = std::max(ctx->prog_dec_p.table_entries, ctx->prog_dec_q.table_entries);
  {
    const ModHost& m = ctx->N;
    const LaunchShape sh = launch_shape(ctx, count, m.t, 8);
#define CALL(LPT, T) HAFLO_LAUNCH((k_dec_unmont<LPT, T>), sh, st, m.ref(), (const u32*)d_cipher, canon29, count)
    HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  }
  {
    // both prime-power branches in one launch: the first half of the grid works modulo p^2,
    // the second half modulo q^2, each half with its own table slots
    const ModHost& m = ctx->P2;
    LaunchShape sh = modexp_shape(ctx, count, m, 2);
    EngineJob job[2];
    for (int side = 0; side < 2; ++side) {
      const ModHost& ms = side ? ctx->Q2 : ctx->P2;
      const DevProg& dp = side ? ctx->prog_dec_q : ctx->prog_dec_p;
      job[side].M = ms.ref();
      job[side].P = ProgPtr{dp.d_ins, (int)dp.host.size()};
      job[side].io = engine_io(ms);
      job[side].io.in_limbs = canon29;
      job[side].io.in_limbs_stride = 2 * ms.nl;
      job[side].io.out = side ? yq : yp;
      job[side].io.tables = tables + (side ? sh.slots() * (size_t)dp_table_entries * ms.nl : 0);
      job[side].io.table_entries = dp_table_entries;
    }
    const unsigned split = (unsigned)sh.blocks;
    sh.blocks *= 2;
    if (sh.geo == kGeoPlain || (sh.geo == kGeoWave && ctx->P.nl == 72)) {
      // a batch that fills the chip (or, at a 4096-bit key, one integer per wavefront): both branches on pairs
      // modulo the primes; what comes out is the second half of the pair 1 + s L, the quotient L_s itself
      for (int side = 0; side < 2; ++side) {
        const ModHost& ms = side ? ctx->Q : ctx->P;
        const DevProg& dp = side ? ctx->prog_dec_pairs_q : ctx->prog_dec_pairs_p;
        job[side].M = ms.ref();
        job[side].P = ProgPtr{dp.d_ins, (int)dp.host.size()};
        job[side].io = pair_io(ms, job[side].io);
        job[side].io.in_limbs_stride = ctx->N.nl;
        job[side].io.out_mode = kOutSecond;
      }
      pairs = 1;
      int rc = launch_engine_pairs2(ctx->P, sh, st, job[0], job[1], split, count);
      if (rc != HAFLO_OK) return rc;
    } else {
#define CALL(LPT, T) HAFLO_LAUNCH((k_engine_pair<LPT, T>), sh, st, job[0], job[1], split, count)
      if (sh.geo == kGeoWave) { HAFLO_DISPATCH_GEOMETRY_WAVE(m, CALL); }
      else if (sh.geo == kGeoWide) { HAFLO_DISPATCH_GEOMETRY_WIDE(m, CALL); }
      else { HAFLO_DISPATCH_GEOMETRY(m, CALL); }
#undef CALL
    }
  }
  {
    const ModHost& m = ctx->P;
    const LaunchShape sh = launch_shape(ctx, count, m.t, 8);
#define CALL(LPT, T)                                                                                            \
  HAFLO_LAUNCH((k_dec_crt<LPT, T>), sh, st, ctx->P.ref(), ctx->Q.ref(), ctx->d_pinv, ctx->d_qinv, ctx->d_hp,    \
               ctx->d_hq, ctx->d_pinvq, (const u32*)yp, (const u32*)yq, pairs, d_plain, ctx->lp, count)
    HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  }
  return hip_status(hipGetLastError());
}
}  // namespace
