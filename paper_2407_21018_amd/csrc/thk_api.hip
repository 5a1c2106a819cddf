// C ABI of libthk: argument checks, workspace carving, launch sizing.
// Everything here is host code; no entry point allocates or synchronises.
#include <math.h>
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <mutex>

#include "thk_internal.h"

using namespace thk;

namespace thk {
namespace {
thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

std::atomic<const EnvSwitches *> g_env{nullptr};
std::mutex g_env_mu;

long env_long_raw(const char *name, long unset) {
  const char *e = getenv(name);
  return (e == nullptr || *e == 0) ? unset : atol(e);
}

// A fresh, immutable snapshot of the switches; earlier snapshots stay valid for threads that
// still hold them (reloading is a test hook: the few bytes per reload are never freed).
const EnvSwitches *read_env() {
  EnvSwitches *s = new EnvSwitches();
  const char *path = getenv("THK_PRUNE_PATH");
  s->prune_path = (path != nullptr) ? path[0] : 0;
  s->group_mib = env_long_raw("THK_PRUNE_GROUP_MIB", 0);
  s->block_rows = env_long_raw("THK_PRUNE_BLOCK_ROWS", 0);
  s->hold_rows = env_long_raw("THK_PRUNE_HOLD_ROWS", 0);
  s->max_blocks = env_long_raw("THK_PRUNE_MAX_BLOCKS", -1);
  s->spin_limit = env_long_raw("THK_PRUNE_SPIN_LIMIT", -1);
  const char *ns = getenv("THK_PRUNE_STAGGER_NS");
  s->stagger_set = ns != nullptr;
  s->stagger_ns = ns != nullptr ? atof(ns) : -1.0;
  const char *mf = getenv("THK_DECODE_MFMA");
  s->decode_mfma_off = mf != nullptr && mf[0] == '0';
  const char *pl = getenv("THK_PRUNE_LAUNCH");
  s->prune_launch = pl != nullptr ? pl[0] : 0;
  s->prologue_delay_us = env_long_raw("THK_PRUNE_PROLOGUE_DELAY_US", 0);
  const char *mk = getenv("THK_DECODE_MERGE");
  s->decode_merge = mk != nullptr ? mk[0] : 0;
  const char *vc = getenv("THK_VALUE_COMPACT");
  s->value_compact = vc != nullptr ? vc[0] : 0;
  return s;
}
}  // namespace

const EnvSwitches &env_switches() {
  const EnvSwitches *s = g_env.load(std::memory_order_acquire);
  if (s == nullptr) {
    std::lock_guard<std::mutex> lock(g_env_mu);
    s = g_env.load(std::memory_order_relaxed);
    if (s == nullptr) {
      s = read_env();
      g_env.store(s, std::memory_order_release);
    }
  }
  return *s;
}

hipError_t launch_main_kernel(const void *fn, dim3 grid, dim3 block, void **args, size_t lds, hipStream_t st) {
  if (g_prof_start == nullptr || g_prof_stop == nullptr) return hipLaunchKernel(fn, grid, block, args, lds, st);
  const hipEvent_t e0 = g_prof_start, e1 = g_prof_stop;
  g_prof_start = g_prof_stop = nullptr;
  return hipExtLaunchKernel(fn, grid, block, args, lds, st, e0, e1, 0);
}
}  // namespace thk

namespace {

thread_local hipError_t g_last_hip = hipSuccess;   // the launch error behind the last THK_ERR_HIP
inline bool failed(hipError_t e) {
  if (e != hipSuccess) g_last_hip = e;
  return e != hipSuccess;
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// Compute units of the current device, looked up once per device: 256 on the MI355X the launch
// heuristics are fitted to, fewer on a partitioned one; 256 where no device answers (the planning
// functions are also called by hosts without a GPU).  Only the rule that decides whether a unit's
// row blocks can all be resident at once -- a matter of safety of the one-pass prune, whose
// blocks wait for each other -- uses it; the tuning constants stay those of the 256-unit chip.
int device_cus() {
  constexpr int kMaxDev = 64;
  static std::atomic<int> cache[kMaxDev];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) {
    (void)hipGetLastError();
    return kCUs;
  }
  int n = cache[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
      (void)hipGetLastError();
      n = kCUs;
    }
    cache[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}
inline int elem_bytes(int dtype) { return dtype == THK_BF16 ? 2 : 4; }
inline int64_t units_of(const thk_shape *s) { return (int64_t)s->L * s->B * s->N_kv; }
inline int ld_of(const thk_shape *s) { return s->ld_keep ? s->ld_keep : s->T; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
// rows of the prunable segment that get compacted, and rows between units of K_pruned / V
inline int64_t keep_rows(const thk_shape *s) { return s->S - s->S_recent; }
inline int64_t cache_rows(const thk_shape *s, int64_t used) { return s->S_cap ? s->S_cap : used; }

constexpr int kMaxSplit = 4096;
constexpr int64_t kMaxGrid = 2147483647LL;

// Shape checks common to all entry points.
thk_status check_shape(const thk_shape *s, bool need_obs) {
  if (s == nullptr) return THK_ERR_NULL;
  if (s->L < 1 || s->B < 1 || s->N_q < 1 || s->N_kv < 1 || s->D < 1 || s->S < 1) return THK_ERR_SHAPE;
  if (s->N_q % s->N_kv != 0) return THK_ERR_SHAPE;
  if (s->T < 1 || s->T > s->D) return THK_ERR_SHAPE;
  // rows of K_pruned hold T kept channels and at most D elements in all (the compaction's gather
  // table and the decode kernels' staging are sized for rows of up to D elements)
  if (s->ld_keep != 0 && (s->ld_keep < s->T || s->ld_keep > s->D)) return THK_ERR_SHAPE;
  if (need_obs && (s->S_obs < 1 || (int64_t)s->S_obs > s->S)) return THK_ERR_SHAPE;
  if (s->n_split < 0 || s->n_split > kMaxSplit) return THK_ERR_SHAPE;
  if (s->S_recent < 0 || (int64_t)s->S_recent >= s->S) return THK_ERR_SHAPE;
  if (s->S_cap < 0) return THK_ERR_SHAPE;
  if (s->dtype != THK_F32 && s->dtype != THK_BF16) return THK_ERR_UNSUPPORTED;
  if (s->D != kD) return THK_ERR_UNSUPPORTED;
  if (s->S > (int64_t)1 << 40 || units_of(s) > kMaxGrid) return THK_ERR_SHAPE;
  return THK_OK;
}

// Split of the S axis for the column reduction: `rows` rows per piece.
struct Split { int n; int64_t rows; };

Split score_split(const thk_shape *s, int64_t units) {
  int n = s->n_split;
  if (n == 0) {
    // aim at ~8 blocks per compute unit over the call, pieces of >= 256 rows
    n = (int)ceil_div((int64_t)kCUs * 8, units);
    const int64_t cap = ceil_div(s->S, 256);
    if (n > cap) n = (int)cap;
    if (n > kMaxSplit) n = kMaxSplit;
    if (n < 1) n = 1;
  }
  int64_t rows = ceil_div(s->S, n);
  rows = ceil_div(rows, 16) * 16;
  return {n, rows};
}

int group_width(int G) { return G <= 2 ? G : 4; }   // head slots per block of the general decode kernel

// Query heads that share a block of the decode kernel the shape takes.
int decode_heads_per_block(const thk_shape *s) {
  DecodeArgs a = {};
  a.T = s->T; a.ldk = ld_of(s); a.N_q = s->N_q; a.N_kv = s->N_kv; a.dtype = s->dtype;
  return decode_mq_serves(a) ? decode_mq_heads(a) : group_width(s->N_q / s->N_kv);
}

// Head groups (blocks per split) of a call, and the bytes of its split records rounded up to
// the 8-byte boundary where the flag words (one per group and split) start.
int64_t decode_groups(const thk_shape *s) {
  return units_of(s) * ceil_div(s->N_q / s->N_kv, decode_heads_per_block(s));
}
size_t decode_records_bytes(const thk_shape *s, int n_split) {
  const size_t b = (size_t)s->L * s->B * s->N_q * n_split * (kD + 2) * sizeof(float);
  return (b + 7) & ~(size_t)7;
}

// A 64-bit number, never 0, different for every call of the process and spread over the whole
// range (what an earlier call or other data left in a workspace will not look like it).
unsigned long long next_nonce() {
  static std::atomic<unsigned long long> counter{
      (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count() * 0x9e3779b97f4a7c15ull};
  unsigned long long z = counter.fetch_add(0x9e3779b97f4a7c15ull, std::memory_order_relaxed);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  z = z ^ (z >> 31);
  return z != 0 ? z : 1;
}

// The split records of a call are merged inside the launch (by the block that finishes last for
// a head group) where that saves more than it costs -- see decode_merge_in_launch below.
bool decode_merge_in_launch(const thk_shape *s, int n_split);

Split decode_split(const thk_shape *s) {
  int n = s->n_split;
  const int G = s->N_q / s->N_kv;
  const int64_t wgs = units_of(s) * ceil_div(G, decode_heads_per_block(s));
  if (n == 0) {
    // About one resident set of blocks over the call (4 per compute unit, 3 where a block
    // serves eight heads), a power of two pieces per unit.  A piece has at least 256 rows, or
    // 128 while the launch stays within one block per compute unit; more than 64 pieces (the
    // merge grows with n) only where even that leaves compute units idle.  Short sequences
    // take one block per unit: below these lengths the second launch (the merge) costs more
    // than the split saves.  Big calls still get two pieces per unit so that the last blocks
    // to finish are short.
    const int hpb = decode_heads_per_block(s);
    const int per_cu = hpb == 8 ? 3 : 4;
    const int64_t one_block_rows = (hpb >= 4 ? 320 : 768) * 2 / elem_bytes(s->dtype);   // bf16 rows; half as many fp32 rows
    n = 1;
    while (s->S > one_block_rows && n < 128) {
      const int64_t blocks = (int64_t)n * 2 * wgs;
      if (blocks > (int64_t)kCUs * per_cu || (n >= 64 && blocks > kCUs)) break;
      if (ceil_div(s->S, (int64_t)n * 2) < (blocks <= kCUs ? 128 : 256)) break;
      n *= 2;
    }
    if (n == 1 && s->S >= 2048) n = 2;
  }
  int64_t rows = ceil_div(s->S, n);
  rows = ceil_div(rows, 64) * 64;
  if (s->n_split == 0) n = (int)ceil_div(s->S, rows);   // drop empty pieces
  return {n, rows};
}

// Small calls merge their split records inside the launch: the block that finishes last for a
// head group does it, and the second launch goes away (fp32, 8 heads x 2048 rows: 11.8 -> 9.3 us;
// one sequence of 32 heads x 1024 bf16 rows: 11.1 -> 9.4 us).  The hand-off costs three memory
// round trips at the end of the kernel, a second launch about as much, so the gain fades as the
// launch grows (nothing left at 1024 blocks; a launch that fills the chip four blocks deep --
// 128 units x 8 pieces of 512 rows -- runs 1 us SLOWER: 38.4 -> 39.5 us) and a block that
// serves four or eight heads needs two or four rounds of loads for its merge (+1.1 .. 1.6 us).
// Hence: at most 16 pieces, at most two heads per block, at most two blocks per compute unit.
// THK_DECODE_MERGE = kernel | fused overrides (fused only within the 16 pieces).
bool decode_merge_in_launch(const thk_shape *s, int n_split) {
  if (n_split < 2 || n_split > kDecodeFuseMaxSplit) return false;
  const char sw = env_switches().decode_merge;
  if (sw == 'k') return false;
  if (sw == 'f') return true;
  return decode_heads_per_block(s) <= 2 && decode_groups(s) * n_split <= 2 * (int64_t)kCUs;
}

// Units per group in the staged form of thk_prune (three launches per group).
// Small groups would let the compaction re-read K from the memory-side cache,
// but measured launch overheads outweigh that; the default keeps groups large.
int64_t prune_group_units(const thk_shape *s) {
  size_t budget = (size_t)1024 << 20;
  if (env_switches().group_mib > 0) budget = (size_t)env_switches().group_mib << 20;
  const size_t per_unit = (size_t)s->S * kD * elem_bytes(s->dtype);
  int64_t g = (int64_t)(budget / per_unit);
  if (g < 1) g = 1;
  const int64_t U = units_of(s);
  return g > U ? U : g;
}

// ---- one-launch prune: eligibility and blocking -------------------------------
struct FusedPlan;
bool value_compact_in_bursts(const thk_shape *s, const FusedPlan &fp);

struct FusedPlan { bool ok; int NB; int64_t RB; int hold; };

// The one-launch forms of thk_prune.  Blocks take 512 bf16 / 256 fp32 rows each (measured best on
// MI355X; fewer for small calls) and the blocks of a unit wait for each other; a unit may have
// as many as are resident at once (768 bf16 / 512 fp32; above 64 their sums travel in two
// levels), longer sequences go through the staged path instead.
FusedPlan fused_plan(const thk_shape *s) {
  FusedPlan p{false, 0, 0, 0};
  const EnvSwitches &env = env_switches();
  const char path = env.prune_path;
  if (path == 's') return p;   // "staged": the three-kernel path
  if (s->S_cap != 0 && s->S_cap < keep_rows(s)) return p;
  int64_t rb = env.block_rows;
  if (rb <= 0) {
    // the default block size: 128 KB of rows, the most a block can hold on chip (512 bf16 rows,
    // 256 fp32 rows); small calls take the smallest held size (down to 128 rows) that keeps the
    // launch within two blocks per compute unit, i.e. within one round of resident blocks:
    // a launch that spills into a second round pays the whole load -> list -> store chain twice
    // (32 units of 4096 bf16 rows: 23 us with 512 blocks of 256 rows, 36 us with 1024 of 128)
    const int64_t rb_max = env.hold_rows > 0 ? env.hold_rows : (s->dtype == THK_BF16 ? 512 : 256);
    auto blocks = [&](int64_t r) { return units_of(s) * ceil_div(s->S, r); };
    rb = rb_max;
    while (rb > 128 && (blocks(rb / 2) <= (int64_t)kCUs * 2 || blocks(rb / 2) == blocks(rb))) rb /= 2;
  }
  if (rb < 32) rb = 32;
  rb = ceil_div(rb, 32) * 32;
  // blocks of 128, 256 or 512 rows (fp32: 128 or 256) keep their rows on chip between the
  // column sums and the compaction; other sizes, or THK_PRUNE_PATH=reread, read them twice
  const bool reread = path == 'r';
  if (!reread && (rb == 128 || rb == 256 || (rb == 512 && s->dtype == THK_BF16))) p.hold = (int)(rb / 128);
  const int64_t nb = ceil_div(s->S, rb);
  // the blocks of a unit wait for each other, so all of them must be resident at once; 256 where
  // the rows are read twice (the second read wants the unit's rows still in the memory-side cache)
  // (LDS decides: 2 KB + four tiles + 7 KB per block, i.e. three bf16 blocks or two fp32 blocks
  // per compute unit)
  const long fit = p.hold == 0 ? 256L : (s->dtype == THK_BF16 ? 3L : 2L) * std::min(device_cus(), kCUs);
  const bool forced = path == 'f' || path == 'r';   // regardless of the env limit
  if (nb > (forced || env.max_blocks < 0 ? fit : std::min(fit, env.max_blocks))) return p;
  p.RB = rb;
  p.NB = (int)nb;
  p.ok = units_of(s) * p.NB <= kMaxGrid;
  return p;
}

// Calls whose rows are held on chip and whose blocks make at most two rounds of resident blocks
// (three for units of more than 64 blocks) run as ONE launch (thk_prune_solo.hip): the two extra
// launches of the other form and the gaps around them are 7-30 % of such a call (fp32, 8 units
// x 2048 rows: 17.8 -> 12.8 us; 128 units x 4096 bf16 rows: 58.1 -> 51.8 us; 8 units x 131072
// rows: 97 -> 88-90 us).  From about four rounds on the single launch is no better (4 x 128
// units x 4096 rows: 161 against 161 us) and then worse (32 x 128 units: 1151-1282 against
// 1141-1154 us; 1280 units x 16384 rows: 1379-1497 against 1287-1306 us), so longer launches keep
// the three-launch form.  THK_PRUNE_LAUNCH = solo | classic overrides.
bool prune_single_launch(const thk_shape *s, const FusedPlan &fp) {
  if (!fp.ok || fp.hold == 0) return false;
  if (units_of(s) * ((int64_t)fp.NB + 1) > kMaxGrid) return false;
  const char sw = env_switches().prune_launch;
  if (sw == 'c') return false;
  if (sw == 's') return true;
  const int64_t resident = (int64_t)kCUs * (s->dtype == THK_BF16 ? 3 : 2);
  return units_of(s) * fp.NB <= (fp.NB > 64 ? 3 : 2) * resident;
}

// thk_prune_value compacts V through the one-pass prune kernels (index list given) where a call
// is long enough for the grouping of stores to pay: rows held on chip and at least 16 rounds of
// resident blocks.  Measured against the plain compaction kernel, whole thk_prune_value calls:
// units of 4096 bf16 rows +5 % at 2.7 rounds, +1 % at 5, -2 % at 11, -2.5 % at 16, -4.4 % at 32,
// -5 % at 43; units of 32768 rows +2 % at 5, +1 % at 11, -1.6 % at 21.
// THK_VALUE_COMPACT = flat | burst overrides (burst only where the rows can be held).
bool value_compact_in_bursts(const thk_shape *s, const FusedPlan &fp) {
  if (!fp.ok || fp.hold == 0) return false;
  const char sw = env_switches().value_compact;
  if (sw == 'f') return false;
  if (sw == 'b') return true;
  const int64_t resident = (int64_t)kCUs * (s->dtype == THK_BF16 ? 3 : 2);
  return units_of(s) * (int64_t)fp.NB >= 16 * resident;
}

// Split of the S axis for the value score: pieces are whole 128-row chunks of at least 512
// rows (fp32: 128), enough of them for one resident set of blocks (two per compute unit: 74 KB of LDS
// each; more pieces only add merge work -- one layer of config 2: 65 us with 8 pieces per
// unit, 54-55 us with 2-4), and few enough that the merge kernel's weight table (at most 256
// pieces) fits.
Split value_split(const thk_shape *s) {
  const int G = s->N_q / s->N_kv;
  const int QT = value_attn_qt(G, s->S_obs);
  const int nqt = (G * s->S_obs + 31) / 32;
  const int64_t blocks1 = units_of(s) * ceil_div(nqt, QT);
  int n = s->n_split;
  if (n == 0) {
    n = (int)ceil_div((int64_t)kCUs * 2, blocks1);
    // fp32: pieces down to one 128-row chunk (a block is one to four wavefronts bound by the
    // fp32 matrix rate: 8 units x 2048 rows 110 -> 47 us, 64 x 1024 rows 112 -> 48 us); bf16
    // blocks take four chunks side by side and lose 10-15 % with smaller pieces
    const int64_t cap = ceil_div(s->S, s->dtype == THK_F32 ? 128 : 512);
    if (n > cap) n = (int)cap;
    if (n < 1) n = 1;
  }
  if (n > 256) n = 256;
  int64_t rows = ceil_div(s->S, n);
  rows = ceil_div(rows, 128) * 128;
  n = (int)ceil_div(s->S, rows);   // drop empty pieces
  return {n, rows};
}

size_t score_ws_bytes(const thk_shape *s, int64_t units) {
  return (size_t)units * score_split(s, units).n * kD * sizeof(double);
}

}  // namespace

extern "C" {

int32_t thk_version(void) { return 200; }

void thk_reload_env(void) {
  std::lock_guard<std::mutex> lock(g_env_mu);
  g_env.store(read_env(), std::memory_order_release);
}

void thk_profile_next(void *ev_start, void *ev_stop) {
  g_prof_start = (ev_start != nullptr && ev_stop != nullptr) ? (hipEvent_t)ev_start : nullptr;
  g_prof_stop = (ev_start != nullptr && ev_stop != nullptr) ? (hipEvent_t)ev_stop : nullptr;
}

thk_status thk_bench_stream(int32_t mode, const void *src, void *dst, int64_t n_blocks, int32_t w, void *stream) {
  if (mode < THK_STREAM_READ || mode > THK_STREAM_WRITE) return THK_ERR_SHAPE;
  if (n_blocks < 1 || n_blocks > 2147483647LL || w < 0 || w > 32) return THK_ERR_SHAPE;
  if (mode != THK_STREAM_READ && w < 1) return THK_ERR_SHAPE;
  if (mode != THK_STREAM_WRITE && src == nullptr) return THK_ERR_NULL;
  if (mode != THK_STREAM_READ && dst == nullptr) return THK_ERR_NULL;
  if (!aligned16(src) || !aligned16(dst)) return THK_ERR_ALIGN;
  clear_stale_hip_error();
  return failed(launch_bench_stream(mode, src, dst, n_blocks, w, (hipStream_t)stream)) ? THK_ERR_HIP : THK_OK;
}

const char *thk_last_hip_error(void) { return hipGetErrorString(g_last_hip); }

const char *thk_status_string(thk_status st) {
  switch (st) {
    case THK_OK: return "ok";
    case THK_ERR_NULL: return "null pointer";
    case THK_ERR_SHAPE: return "invalid shape";
    case THK_ERR_UNSUPPORTED: return "unsupported configuration";
    case THK_ERR_ALIGN: return "pointer not 16-byte aligned";
    case THK_ERR_WORKSPACE: return "workspace missing or too small";
    case THK_ERR_HIP: return "HIP launch failed";
    case THK_ERR_SCRATCH: return "the call needs more scratch than the library's static buffer holds";
  }
  return "unknown status";
}

int32_t thk_keep_count(int32_t D, double lambda) {
  if (D < 1 || !(lambda >= 0.0) || !(lambda < 1.0)) return -1;
  return (int32_t)floor((1.0 - lambda) * (double)D + 1e-9);
}

int32_t thk_default_split(const thk_shape *s, int32_t op) {
  if (check_shape(s, false) != THK_OK) return 0;
  thk_shape t = *s;
  t.n_split = 0;
  if (op == THK_OP_DECODE) return decode_split(&t).n;
  if (op == THK_OP_SCORE) return score_split(&t, units_of(&t)).n;
  if (op == THK_OP_PRUNE) return score_split(&t, prune_group_units(&t)).n;
  if (op == THK_OP_SCORE_VALUE || op == THK_OP_PRUNE_VALUE) return (t.S_obs >= 1 && t.S_obs <= t.S) ? value_split(&t).n : 0;
  return 0;
}

int32_t thk_prune_is_fused(const thk_shape *s) {
  if (check_shape(s, true) != THK_OK) return 0;
  const FusedPlan fp = fused_plan(s);
  return !fp.ok ? 0 : fp.hold != 0 ? 2 : 1;
}

int32_t thk_prune_launches(const thk_shape *s) {
  if (check_shape(s, true) != THK_OK) return 0;
  const FusedPlan fp = fused_plan(s);
  if (!fp.ok) return 3 * (int32_t)ceil_div(units_of(s), prune_group_units(s));
  return prune_single_launch(s, fp) ? 1 : 3;
}

int32_t thk_decode_on_matrix_cores(const thk_shape *s, int32_t T_v, int32_t ld_v) {
  if (check_shape(s, false) != THK_OK) return 0;
  if (T_v < 0 || T_v > kD || (T_v > 0 && (ld_v < T_v || ld_v > kD))) return 0;
  DecodeArgs a = {};
  a.T = s->T; a.ldk = ld_of(s); a.N_q = s->N_q; a.N_kv = s->N_kv; a.dtype = s->dtype;
  a.T_v = T_v; a.ld_v = T_v > 0 ? ld_v : 0;
  return decode_mq_serves(a) ? 1 : 0;
}

size_t thk_workspace_bytes(const thk_shape *s, int32_t op) {
  if (check_shape(s, false) != THK_OK) return 0;
  switch (op) {
    case THK_OP_SCORE:
      return score_ws_bytes(s, units_of(s));
    case THK_OP_DECODE: {
      const Split sp = decode_split(s);
      if (sp.n == 1) return 16;
      return decode_records_bytes(s, sp.n) + (size_t)decode_groups(s) * sp.n * sizeof(unsigned long long);
    }
    case THK_OP_SCORE_VALUE:
      if (s->S_obs < 1 || (int64_t)s->S_obs > s->S) return 0;
      return value_part_bytes(units_of(s), s->N_q / s->N_kv, s->S_obs, value_split(s).n);
    case THK_OP_PRUNE_VALUE: {
      if (s->S_obs < 1 || (int64_t)s->S_obs > s->S) return 0;
      size_t a = value_part_bytes(units_of(s), s->N_q / s->N_kv, s->S_obs, value_split(s).n);
      const FusedPlan fp = fused_plan(s);
      if (value_compact_in_bursts(s, fp)) a = std::max(a, prune_fused_ws_bytes(units_of(s), fp.NB));
      return ((a + 15) & ~(size_t)15) + (size_t)units_of(s) * kD * sizeof(float);
    }
    case THK_OP_PRUNE: {
      // a score array for the whole call + the larger of the two paths' scratch
      const FusedPlan fp = fused_plan(s);
      size_t a = score_ws_bytes(s, prune_group_units(s));
      if (fp.ok) {
        const size_t b = std::max(prune_fused_ws_bytes(units_of(s), fp.NB), prune_solo_ws_bytes(units_of(s), fp.NB));
        if (b > a) a = b;
      }
      return ((a + 15) & ~(size_t)15) + (size_t)units_of(s) * kD * sizeof(float);
    }
  }
  return 0;
}

static thk_status score_common(const thk_shape *s, int mode, const void *q_obs, const void *k,
                               float *score, void *ws, size_t ws_bytes, void *stream) {
  thk_status st = check_shape(s, mode == 0);
  if (st != THK_OK) return st;
  if (k == nullptr || score == nullptr || (mode == 0 && q_obs == nullptr)) return THK_ERR_NULL;
  if (!aligned16(k) || !aligned16(score) || (mode == 0 && !aligned16(q_obs))) return THK_ERR_ALIGN;
  const int64_t U = units_of(s);
  const Split sp = score_split(s, U);
  if (U * sp.n > kMaxGrid) return THK_ERR_SHAPE;
  if (ws == nullptr || !aligned16(ws) || ws_bytes < score_ws_bytes(s, U)) return THK_ERR_WORKSPACE;
  hipStream_t hs = (hipStream_t)stream;
  if (failed(launch_colsum(s->dtype, k, (double *)ws, U, s->S, sp.n, sp.rows, mode == 1 ? 1 : 2, hs)))
    return THK_ERR_HIP;
  if (failed(launch_finalize(s->dtype, mode, (const double *)ws, q_obs, score, nullptr, U, s->N_q / s->N_kv,
                      s->S_obs, sp.n, s->T, hs)))
    return THK_ERR_HIP;
  return THK_OK;
}

thk_status thk_score(const thk_shape *s, const void *q_obs, const void *k, float *score, void *ws,
                     size_t ws_bytes, void *stream) {
  return score_common(s, 0, q_obs, k, score, ws, ws_bytes, stream);
}

thk_status thk_score_magnitude(const thk_shape *s, const void *k, int32_t p, float *score,
                               void *ws, size_t ws_bytes, void *stream) {
  if (p != 1 && p != 2) return s == nullptr ? THK_ERR_NULL : THK_ERR_SHAPE;
  return score_common(s, p == 1 ? 1 : 2, nullptr, k, score, ws, ws_bytes, stream);
}

thk_status thk_select_topk(const thk_shape *s, const float *score, int16_t *idx, void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  if (score == nullptr || idx == nullptr) return THK_ERR_NULL;
  if (!aligned16(score) || !aligned16(idx)) return THK_ERR_ALIGN;
  if (failed(launch_select(score, idx, units_of(s), s->T, (hipStream_t)stream))) return THK_ERR_HIP;
  return THK_OK;
}

thk_status thk_compact_keys(const thk_shape *s, const void *k, const int16_t *idx, void *k_pruned,
                            void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  if (k == nullptr || idx == nullptr || k_pruned == nullptr) return THK_ERR_NULL;
  if (!aligned16(k) || !aligned16(idx) || !aligned16(k_pruned)) return THK_ERR_ALIGN;
  if (units_of(s) * ceil_div(s->S, 512) > kMaxGrid) return THK_ERR_SHAPE;
  if (s->S_cap != 0 && s->S_cap < keep_rows(s)) return THK_ERR_SHAPE;
  if (failed(launch_compact(s->dtype, k, s->S, 0, idx, k_pruned, cache_rows(s, keep_rows(s)), 0, units_of(s),
                            keep_rows(s), s->T, ld_of(s), (hipStream_t)stream)))
    return THK_ERR_HIP;
  return THK_OK;
}

thk_status thk_compact_rows(const thk_shape *s, const void *src, int64_t src_unit_rows, int64_t src_row0,
                            const int16_t *idx, void *k_pruned, int64_t dst_row0, int64_t n_rows,
                            void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  if (src == nullptr || idx == nullptr || k_pruned == nullptr) return THK_ERR_NULL;
  const int64_t dst_unit_rows = cache_rows(s, s->S);
  if (n_rows < 0 || src_row0 < 0 || dst_row0 < 0 || src_row0 + n_rows > src_unit_rows ||
      dst_row0 + n_rows > dst_unit_rows)
    return THK_ERR_SHAPE;
  if (!aligned16(src) || !aligned16(idx) || !aligned16(k_pruned)) return THK_ERR_ALIGN;
  if (units_of(s) * ceil_div(n_rows > 0 ? n_rows : 1, 512) > kMaxGrid) return THK_ERR_SHAPE;
  if (failed(launch_compact(s->dtype, src, src_unit_rows, src_row0, idx, k_pruned, dst_unit_rows, dst_row0,
                     units_of(s), n_rows, s->T, ld_of(s), (hipStream_t)stream)))
    return THK_ERR_HIP;
  return THK_OK;
}

thk_status thk_copy_rows(const thk_shape *s, const void *src, int64_t src_unit_rows, int64_t src_row0,
                         void *dst, int64_t dst_unit_rows, int64_t dst_row0, int64_t n_rows,
                         void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  if (src == nullptr || dst == nullptr) return THK_ERR_NULL;
  if (n_rows < 0 || src_row0 < 0 || dst_row0 < 0 || src_row0 + n_rows > src_unit_rows ||
      dst_row0 + n_rows > dst_unit_rows)
    return THK_ERR_SHAPE;
  if (src == dst && (dst_unit_rows != src_unit_rows || dst_row0 > src_row0)) return THK_ERR_SHAPE;
  if (!aligned16(src) || !aligned16(dst)) return THK_ERR_ALIGN;
  if (failed(launch_copy_rows(s->dtype, src, src_unit_rows, src_row0, dst, dst_unit_rows, dst_row0, units_of(s),
                       n_rows, (hipStream_t)stream)))
    return THK_ERR_HIP;
  return THK_OK;
}

thk_status thk_cache_append(const thk_shape *s, const void *k_new, const void *v_new, void *k_tail,
                            void *v, int32_t s_tail, int32_t s_tail_cap, void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  if (k_new == nullptr || v_new == nullptr || k_tail == nullptr || v == nullptr) return THK_ERR_NULL;
  if (s_tail < 0 || s_tail >= s_tail_cap) return THK_ERR_SHAPE;
  if (s->S + s_tail >= cache_rows(s, s->S)) return THK_ERR_SHAPE;   // the value cache is full
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_tail) || !aligned16(v)) return THK_ERR_ALIGN;
  if (failed(launch_tail_append(s->dtype, k_new, v_new, k_tail, v, units_of(s), s_tail_cap, s_tail,
                         cache_rows(s, s->S), s->S + s_tail, (hipStream_t)stream)))
    return THK_ERR_HIP;
  return THK_OK;
}

thk_status thk_tail_flush(const thk_shape *s, const int16_t *idx, void *k_pruned, void *k_tail, void *v,
                          void *v_tail, int32_t s_tail, int32_t s_tail_cap, int32_t n_flush,
                          void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  if (idx == nullptr || k_pruned == nullptr || k_tail == nullptr) return THK_ERR_NULL;
  if ((v == nullptr) != (v_tail == nullptr)) return THK_ERR_NULL;
  if (s_tail < 0 || s_tail > s_tail_cap || n_flush < 0 || n_flush > s_tail) return THK_ERR_SHAPE;
  const int64_t unit_rows = cache_rows(s, s->S);
  if (s->S + n_flush > unit_rows) return THK_ERR_SHAPE;   // no room left in the pruned cache
  if (!aligned16(idx) || !aligned16(k_pruned) || !aligned16(k_tail) ||
      (v != nullptr && (!aligned16(v) || !aligned16(v_tail))))
    return THK_ERR_ALIGN;
  hipStream_t hs = (hipStream_t)stream;
  const int64_t U = units_of(s);
  if (failed(launch_compact(s->dtype, k_tail, s_tail_cap, 0, idx, k_pruned, unit_rows, s->S, U, n_flush, s->T,
                     ld_of(s), hs)))
    return THK_ERR_HIP;
  if (failed(launch_copy_rows(s->dtype, k_tail, s_tail_cap, n_flush, k_tail, s_tail_cap, 0, U, s_tail - n_flush,
                       hs)))
    return THK_ERR_HIP;
  if (v != nullptr) {
    if (failed(launch_copy_rows(s->dtype, v_tail, s_tail_cap, 0, v, unit_rows, s->S, U, n_flush, hs)))
      return THK_ERR_HIP;
    if (failed(launch_copy_rows(s->dtype, v_tail, s_tail_cap, n_flush, v_tail, s_tail_cap, 0, U, s_tail - n_flush,
                         hs)))
      return THK_ERR_HIP;
  }
  return THK_OK;
}

thk_status thk_prune(const thk_shape *s, const void *q_obs, const void *k, float *score,
                     int16_t *idx, void *k_pruned, void *ws, size_t ws_bytes, void *stream) {
  thk_status st = check_shape(s, true);
  if (st != THK_OK) return st;
  if (q_obs == nullptr || k == nullptr || idx == nullptr || k_pruned == nullptr) return THK_ERR_NULL;
  if (!aligned16(q_obs) || !aligned16(k) || !aligned16(idx) || !aligned16(k_pruned) ||
      (score != nullptr && !aligned16(score)))
    return THK_ERR_ALIGN;
  if (ws == nullptr || !aligned16(ws) || ws_bytes < thk_workspace_bytes(s, THK_OP_PRUNE)) return THK_ERR_WORKSPACE;
  const int64_t U = units_of(s);
  const int G = s->N_q / s->N_kv;
  hipStream_t hs = (hipStream_t)stream;
  const size_t score_off = thk_workspace_bytes(s, THK_OP_PRUNE) - (size_t)U * kD * sizeof(float);
  float *sc = score != nullptr ? score : (float *)((char *)ws + score_off);
  const FusedPlan fp = fused_plan(s);
  if (fp.ok) {
    const int spin = env_switches().spin_limit >= 0 ? (int)env_switches().spin_limit : 4096;
    if (prune_single_launch(s, fp)) {
      if (failed(launch_prune_solo(s->dtype, q_obs, k, sc, idx, k_pruned, ws, U, s->S, keep_rows(s),
                                   cache_rows(s, keep_rows(s)), G, s->S_obs, s->T, ld_of(s), fp.NB, fp.RB, fp.hold,
                                   spin, hs)))
        return THK_ERR_HIP;
      return THK_OK;
    }
    if (failed(launch_prune_fused(s->dtype, q_obs, k, sc, idx, k_pruned, ws, U, s->S, keep_rows(s),
                                  cache_rows(s, keep_rows(s)), G, s->S_obs, s->T, ld_of(s), fp.NB, fp.RB, fp.hold,
                                  spin < 0 ? 0 : spin, 0, hs)))
      return THK_ERR_HIP;
    return THK_OK;
  }
  // staged path: score -> select -> compact per group of units
  if (s->S_cap != 0 && s->S_cap < keep_rows(s)) return THK_ERR_SHAPE;
  const int64_t kp_rows = cache_rows(s, keep_rows(s));
  const int64_t gu = prune_group_units(s);
  const Split sp = score_split(s, gu);
  if (gu * sp.n > kMaxGrid || gu * ceil_div(s->S, 512) > kMaxGrid) return THK_ERR_SHAPE;
  double *partial = (double *)ws;
  const int eb = elem_bytes(s->dtype);
  const int ld = ld_of(s);
  for (int64_t u0 = 0; u0 < U; u0 += gu) {
    const int64_t nu = (U - u0 < gu) ? U - u0 : gu;
    const char *kg = (const char *)k + (size_t)u0 * s->S * kD * eb;
    if (failed(launch_colsum(s->dtype, kg, partial, nu, s->S, sp.n, sp.rows, 2, hs))) return THK_ERR_HIP;
    // unit u reads query heads u * G .. u * G + G - 1, so a group starting at u0 starts u0 * G heads in
    const char *qg = (const char *)q_obs + (size_t)u0 * G * s->S_obs * kD * eb;
    if (failed(launch_finalize(s->dtype, 0, partial, qg, sc + (size_t)u0 * kD, idx + (size_t)u0 * s->T, nu, G,
                        s->S_obs, sp.n, s->T, hs)))
      return THK_ERR_HIP;
    const hipError_t ce = launch_compact(s->dtype, kg, s->S, 0, idx + (size_t)u0 * s->T,
                                         (char *)k_pruned + (size_t)u0 * kp_rows * ld * eb, kp_rows, 0, nu,
                                         keep_rows(s), s->T, ld, hs);
    if (failed(ce)) return THK_ERR_HIP;
  }
  return THK_OK;
}

thk_status thk_score_value(const thk_shape *s, const void *q_obs, const void *k, const void *v,
                           int32_t causal, float *score_v, void *ws, size_t ws_bytes, void *stream) {
  thk_status st = check_shape(s, true);
  if (st != THK_OK) return st;
  if (q_obs == nullptr || k == nullptr || v == nullptr || score_v == nullptr) return THK_ERR_NULL;
  if (!aligned16(q_obs) || !aligned16(k) || !aligned16(v) || !aligned16(score_v)) return THK_ERR_ALIGN;
  if (causal != 0 && causal != 1) return THK_ERR_SHAPE;
  const int G = s->N_q / s->N_kv;
  if ((int64_t)G * s->S_obs > 32 * 1024) return THK_ERR_SHAPE;
  const Split sp = value_split(s);
  const int QT = value_attn_qt(G, s->S_obs);
  // (the launch rounds the pieces up to a multiple of 8 where a unit has several query blocks)
  const int64_t grid = (units_of(s) * sp.n + 7) * ceil_div((G * s->S_obs + 31) / 32, QT);
  if (grid > kMaxGrid) return THK_ERR_SHAPE;
  if (ws == nullptr || !aligned16(ws) || ws_bytes < thk_workspace_bytes(s, THK_OP_SCORE_VALUE))
    return THK_ERR_WORKSPACE;
  if (failed(launch_value_score(s->dtype, q_obs, k, v, (float *)ws, score_v, units_of(s), s->S, G, s->S_obs, causal,
                         sp.n, sp.rows, (hipStream_t)stream)))
    return THK_ERR_HIP;
  return THK_OK;
}

thk_status thk_prune_value(const thk_shape *s, const void *q_obs, const void *k, const void *v,
                           int32_t causal, float *score_v, int16_t *idx_v, void *v_pruned, void *ws,
                           size_t ws_bytes, void *stream) {
  thk_status st = check_shape(s, true);
  if (st != THK_OK) return st;
  if (idx_v == nullptr || v_pruned == nullptr) return THK_ERR_NULL;
  if (!aligned16(idx_v) || !aligned16(v_pruned) || (score_v != nullptr && !aligned16(score_v)))
    return THK_ERR_ALIGN;
  const size_t need = thk_workspace_bytes(s, THK_OP_PRUNE_VALUE);
  if (ws == nullptr || !aligned16(ws) || ws_bytes < need) return THK_ERR_WORKSPACE;
  // the score array sits behind the value score's own scratch unless the caller wants it
  float *sc = score_v != nullptr ? score_v : (float *)((char *)ws + need - (size_t)units_of(s) * kD * sizeof(float));
  st = thk_score_value(s, q_obs, k, v, causal, sc, ws, thk_workspace_bytes(s, THK_OP_SCORE_VALUE), stream);
  if (st != THK_OK) return st;
  st = thk_select_topk(s, sc, idx_v, stream);
  if (st != THK_OK) return st;
  // Long calls compact through the one-pass prune kernels with the list given: their hand-off
  // makes the blocks of a unit store together, and the memory takes a unit's rows in one burst
  // better than the same rows interleaved with other units' loads (32 layers of 128 units x
  // 4096 rows: 1225 -> 1100 us).  The value score's scratch is free again by then.
  const FusedPlan fp = fused_plan(s);
  if (value_compact_in_bursts(s, fp)) {
    const int spin = env_switches().spin_limit >= 0 ? (int)env_switches().spin_limit : 4096;
    if (failed(launch_prune_fused(s->dtype, v, v, nullptr, idx_v, v_pruned, ws, units_of(s), s->S, keep_rows(s),
                                  cache_rows(s, keep_rows(s)), 1, 0, s->T, ld_of(s), fp.NB, fp.RB, fp.hold, spin, 1,
                                  (hipStream_t)stream)))
      return THK_ERR_HIP;
    return THK_OK;
  }
  return thk_compact_keys(s, v, idx_v, v_pruned, stream);
}

static thk_status decode_common(const thk_shape *s, const void *q, const void *k_pruned,
                                const int16_t *idx, const void *v, const int16_t *idx_v, int32_t T_v,
                                int32_t ld_v, const void *k_tail, const void *v_tail, int32_t s_tail,
                                int32_t s_tail_cap, void *out, void *ws, size_t ws_bytes, void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  if (q == nullptr || k_pruned == nullptr || idx == nullptr || v == nullptr || out == nullptr) return THK_ERR_NULL;
  if (s_tail < 0 || s_tail_cap < 0 || s_tail > s_tail_cap) return THK_ERR_SHAPE;
  if (s_tail > 0 && k_tail == nullptr) return THK_ERR_NULL;
  const bool pruned_v = T_v > 0;
  if (pruned_v) {
    if (idx_v == nullptr || (s_tail > 0 && v_tail == nullptr)) return THK_ERR_NULL;
    if (T_v > s->D || ld_v < T_v || ld_v > s->D) return THK_ERR_SHAPE;
    if (ld_v % 4 != 0) return THK_ERR_UNSUPPORTED;
    if (!aligned16(idx_v)) return THK_ERR_ALIGN;
  }
  const bool unified_v = s_tail > 0 && v_tail == nullptr;   // tail values follow row S in v
  const int64_t unit_rows = cache_rows(s, s->S);
  if (unit_rows < s->S + (unified_v ? s_tail : 0)) return THK_ERR_SHAPE;
  if (!aligned16(q) || !aligned16(k_pruned) || !aligned16(idx) || !aligned16(v) || !aligned16(out) ||
      (s_tail > 0 && (!aligned16(k_tail) || (v_tail != nullptr && !aligned16(v_tail)))))
    return THK_ERR_ALIGN;
  const Split sp = decode_split(s);
  const int G = s->N_q / s->N_kv;
  if (units_of(s) * ceil_div(G, decode_heads_per_block(s)) * sp.n > kMaxGrid) return THK_ERR_SHAPE;
  if (sp.n > 1 && (ws == nullptr || !aligned16(ws) || ws_bytes < thk_workspace_bytes(s, THK_OP_DECODE)))
    return THK_ERR_WORKSPACE;
  DecodeArgs a;
  a.q = q; a.kp = k_pruned; a.v = v; a.kt = k_tail; a.vt = v_tail; a.idx = idx; a.out = out;
  a.ws = (float *)ws;
  a.S = s->S; a.rows_per_split = sp.rows;
  a.T = s->T; a.ldk = ld_of(s); a.N_q = s->N_q; a.N_kv = s->N_kv;
  a.s_tail = s_tail; a.s_tail_cap = s_tail_cap; a.n_split = sp.n; a.dtype = s->dtype;
  a.units = units_of(s);
  a.unit_rows = unit_rows;
  a.unified_v = unified_v ? 1 : 0;
  a.scale_log2_d = 1.4426950408889634 / sqrt((double)s->D);
  a.scale_log2 = (float)a.scale_log2_d;
  a.idx_v = idx_v; a.T_v = pruned_v ? T_v : 0; a.ld_v = pruned_v ? ld_v : 0;
  // up to kDecodeFuseMaxSplit pieces per unit are merged inside the launch by the block that
  // finishes last; more pieces go to the merge kernel
  a.arrive = nullptr;
  a.nonce = 0;
  if (decode_merge_in_launch(s, sp.n)) {
    a.arrive = (unsigned long long *)((char *)ws + decode_records_bytes(s, sp.n));
    a.nonce = next_nonce();
  }
  if (failed(launch_decode(a, (hipStream_t)stream))) return THK_ERR_HIP;
  return THK_OK;
}

thk_status thk_decode_attn(const thk_shape *s, const void *q, const void *k_pruned,
                           const int16_t *idx, const void *v, const void *k_tail,
                           const void *v_tail, int32_t s_tail, int32_t s_tail_cap, void *out,
                           void *ws, size_t ws_bytes, void *stream) {
  return decode_common(s, q, k_pruned, idx, v, nullptr, 0, 0, k_tail, v_tail, s_tail, s_tail_cap, out, ws,
                       ws_bytes, stream);
}

thk_status thk_decode_attn_kv(const thk_shape *s, const void *q, const void *k_pruned,
                              const int16_t *idx, const void *v_pruned, const int16_t *idx_v,
                              int32_t T_v, int32_t ld_v, const void *k_tail, const void *v_tail,
                              int32_t s_tail, int32_t s_tail_cap, void *out, void *ws,
                              size_t ws_bytes, void *stream) {
  if (T_v < 1) return s == nullptr ? THK_ERR_NULL : THK_ERR_SHAPE;
  return decode_common(s, q, k_pruned, idx, v_pruned, idx_v, T_v, ld_v, k_tail, v_tail, s_tail, s_tail_cap, out,
                       ws, ws_bytes, stream);
}

// ---- the entry point that allocates nothing ---------------------------------------------
// Split partials of thk_decode_attn_static live in this file-scope device array instead of a
// caller workspace.  Every GPU the library runs on holds its own copy, at its own address,
// until the process ends.  In host code the array's NAME is only a stand-in for the symbol:
// the memory is reached through the per-device address hipGetSymbolAddress returns, looked up
// once per device on the entry point's first call there, and nowhere through the name.
static __device__ __align__(256) unsigned char scratch[THK_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mu;

// Device address of `scratch` on the current device (set-up on first use, no allocation).
thk_status static_scratch(void **out) {
  int dev = -1;
  if (failed(hipGetDevice(&dev))) return THK_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return THK_ERR_UNSUPPORTED;
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (p == nullptr) {
      if (failed(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) || p == nullptr) return THK_ERR_HIP;
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return THK_OK;
}
}  // namespace

thk_status thk_decode_attn_static(const thk_shape *s, const void *q, const void *k_pruned,
                                  const int16_t *idx, const void *v, const void *k_tail,
                                  const void *v_tail, int32_t s_tail, int32_t s_tail_cap, void *out,
                                  void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  // the size check comes before anything touches the device
  const size_t need = thk_workspace_bytes(s, THK_OP_DECODE);
  if (need > (size_t)THK_STATIC_SCRATCH_BYTES) return THK_ERR_SCRATCH;
  void *ws = nullptr;
  st = static_scratch(&ws);
  if (st != THK_OK) return st;
  return decode_common(s, q, k_pruned, idx, v, nullptr, 0, 0, k_tail, v_tail, s_tail, s_tail_cap, out, ws,
                       (size_t)THK_STATIC_SCRATCH_BYTES, stream);
}

thk_status thk_tail_append(const thk_shape *s, const void *k_new, const void *v_new, void *k_tail,
                           void *v_tail, int32_t s_tail, int32_t s_tail_cap, void *stream) {
  thk_status st = check_shape(s, false);
  if (st != THK_OK) return st;
  if (k_new == nullptr || v_new == nullptr || k_tail == nullptr || v_tail == nullptr) return THK_ERR_NULL;
  if (s_tail < 0 || s_tail >= s_tail_cap) return THK_ERR_SHAPE;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_tail) || !aligned16(v_tail)) return THK_ERR_ALIGN;
  if (failed(launch_tail_append(s->dtype, k_new, v_new, k_tail, v_tail, units_of(s), s_tail_cap, s_tail, s_tail_cap,
                         s_tail, (hipStream_t)stream)))
    return THK_ERR_HIP;
  return THK_OK;
}

}  // extern "C"
