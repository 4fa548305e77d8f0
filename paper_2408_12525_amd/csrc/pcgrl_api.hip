// Host side of the C ABI declared in include/pcgrl.h: argument checks, device state, launches.
#include "../../include/pcgrl.h"

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>

#include "pcgrl_kernels.hip.h"

using namespace pcgrl;

struct pcgrl_ctx {
  pcgrl_config cfg;
  int device;
  int S, G, P, K, M, C;
  int B_pad, nwaves;
  int epw;  // distinct levels per wavefront (a divisor of G)
  size_t word_bytes;
  size_t lds_bytes;  // per wavefront
  int split_roll;    // pcgrl_rollout with observations does the same, with its own shape:
  int roll_m, roll_o, roll_groups, roll_turns;
  size_t roll_lds_wave;
  int split;         // pcgrl_step with an observation uses the metrics | observation kernel, with
  int split_m, split_o, split_groups;  // this many levels per metrics / observation wavefront and workgroups
  size_t split_lds_wave;  // LDS bytes of one observation wavefront there
  size_t obs_bytes;  // bytes of one level's observation in the chosen format
  size_t obs_stride; // bytes from one level's observation to the next (obs_bytes, or the configured pitch)
  int store_step, store_roll;  // how a step / a rollout launch stores observations (kStore*)
  int store_step_auto;         // store_step follows the buffers the caller hands in (below)
  const uint8_t* recent_obs[32];  // observation pointers of the last 32 pcgrl_step calls
  unsigned recent_n;
  KArgs base;  // device pointers and configuration, copied into every launch
  void* d_planes;
  void* d_frozen;
  void* d_env;
  void* d_metrics;
  void* d_targets;
  void* d_bad;
  void* d_exact;         // partial results of pcgrl_exact_diameter, [1 << exact_parts_log2][batch] ints (NULL for one part)
  int exact_parts_log2;  // a level's sources are shared out over this many workgroups there
};

namespace {

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    ok = hipSetDevice(dev) == hipSuccess;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

int tiles_of(int problem) { return problem == PCGRL_BINARY ? 2 : problem == PCGRL_MAZE ? 4 : problem == PCGRL_DUNGEON ? 7 : 0; }
int planes_of(int problem) { return problem == PCGRL_BINARY ? 1 : problem == PCGRL_MAZE ? 2 : 3; }
int metrics_of(int problem) { return (problem == PCGRL_DUNGEON ? 3 : 2) + tiles_of(problem); }

int check_config(const pcgrl_config* c) {
  if (tiles_of(c->problem) == 0) return PCGRL_E_CONFIG;
  if (c->batch < 1 || c->batch > (1 << 24)) return PCGRL_E_CONFIG;
  if (c->max_h < 1 || c->max_h > 64 || c->max_w < 1 || c->max_w > 64) return PCGRL_E_CONFIG;
  if (c->min_h < 1 || c->min_h > c->max_h || c->min_w < 1 || c->min_w > c->max_w) return PCGRL_E_CONFIG;
  if (c->obs_w < 1 || c->obs_w > 63) return PCGRL_E_CONFIG;
  if (c->pad_mode != PCGRL_PAD_BORDER && c->pad_mode != PCGRL_PAD_WALL) return PCGRL_E_CONFIG;
  if (c->pos_mode != PCGRL_POS_SCAN && c->pos_mode != PCGRL_POS_RANDOM) return PCGRL_E_CONFIG;
  if (c->n_frozen < 0 || c->n_frozen > 8 || c->n_frozen > c->min_h * c->min_w) return PCGRL_E_CONFIG;
  if (c->max_steps < 1 || c->max_changes < 0) return PCGRL_E_CONFIG;
  if (c->regions_mode != PCGRL_REGIONS_INCREMENTAL && c->regions_mode != PCGRL_REGIONS_RECOUNT) return PCGRL_E_CONFIG;
  if (c->levels_per_wave < 0 || c->levels_per_wave > 4) return PCGRL_E_CONFIG;
  if (c->obs_store_mode < 0 || c->obs_store_mode > 3) return PCGRL_E_CONFIG;
  if (c->split_step < 0 || c->split_step > 2) return PCGRL_E_CONFIG;
  if (c->split_obs_levels < 0 || c->split_obs_levels > 4) return PCGRL_E_CONFIG;
  if (c->rollout_turns != 0 && c->rollout_turns != 1 && c->rollout_turns != 2 && c->rollout_turns != 4) return PCGRL_E_CONFIG;
  if (c->obs_format != PCGRL_OBS_ONEHOT_U8 && c->obs_format != PCGRL_OBS_PACKED) return PCGRL_E_CONFIG;
  if (c->obs_pitch < PCGRL_OBS_PITCH_LINES || (c->obs_pitch > 0 && (c->obs_pitch & 15) != 0)) return PCGRL_E_CONFIG;
  for (int j = 0; j < 8; ++j)
    if (c->pinpoint_tile[j] < -1 || c->pinpoint_tile[j] >= tiles_of(c->problem)) return PCGRL_E_CONFIG;
  for (int i = 0; i < metrics_of(c->problem); ++i)
    if (((c->ctrl_mask >> i) & 1u) && (c->ctrl_lo[i] < 0 || c->ctrl_hi[i] < c->ctrl_lo[i] || c->ctrl_hi[i] > 65535))
      return PCGRL_E_CONFIG;
  for (int k = 1; k < tiles_of(c->problem) - 1; ++k)
    if (c->init_cdf[k] < c->init_cdf[k - 1]) return PCGRL_E_CONFIG;
  return PCGRL_OK;
}

template <template <int, int> class Launcher, typename... A>
int dispatch(int S, int problem, A&&... args) {
#define PCGRL_CASE(SS, PP) \
  if (S == SS && problem == PP) return Launcher<SS, PP>::run(static_cast<A&&>(args)...);
  PCGRL_CASE(16, kBinary) PCGRL_CASE(16, kMaze) PCGRL_CASE(16, kDungeon)
  PCGRL_CASE(32, kBinary) PCGRL_CASE(32, kMaze) PCGRL_CASE(32, kDungeon)
  PCGRL_CASE(64, kBinary) PCGRL_CASE(64, kMaze) PCGRL_CASE(64, kDungeon)
#undef PCGRL_CASE
  return PCGRL_E_CONFIG;
}

// The step kernel takes what it needs first as leading scalar arguments (see the kernel).
inline uint32_t step_shape(const KArgs& a) {
  return (uint32_t)a.B | ((uint32_t)(a.envs_per_wave_log2 & 0xff) << 25) |
         ((uint32_t)((a.envs_per_wave_log2 >> 8) & 0xff) << 27) | ((uint32_t)(a.use_frozen & 3) << 29);
}
#define PCGRL_STEP_ARGS(a) (a).planes, (a).frozen, (a).env, (a).metrics, (a).targets, (a).actions, step_shape(a), (a).plane_stride, (a)
// (single steps come in three builds: windows of up to 32 cells with and without the code that looks
// pinpoint cells up, and wider windows, with it)
template <int S, int PROBLEM> struct LaunchStep {
  static int run(const pcgrl_ctx* ctx, const KArgs& a, hipStream_t st) {
    if (a.obs_w > 32)
      hipLaunchKernelGGL((step_kernel<S, PROBLEM, kModeStep, true, true>), dim3(ctx->nwaves), dim3(64), ctx->lds_bytes, st,
                         PCGRL_STEP_ARGS(a));
    else if (a.use_frozen)
      hipLaunchKernelGGL((step_kernel<S, PROBLEM, kModeStep, true, false>), dim3(ctx->nwaves), dim3(64), ctx->lds_bytes, st,
                         PCGRL_STEP_ARGS(a));
    else
      hipLaunchKernelGGL((step_kernel<S, PROBLEM, kModeStep, false, false>), dim3(ctx->nwaves), dim3(64), ctx->lds_bytes, st,
                         PCGRL_STEP_ARGS(a));
    return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
  }
};
template <int S, int PROBLEM> struct LaunchSplit {  // a metrics wavefront and its observation wavefronts per workgroup
  static int run(const pcgrl_ctx* ctx, const KArgs& a, hipStream_t st) {
    const int obs_waves = ctx->split_m / ctx->split_o;
    const dim3 grid(ctx->split_groups), block(64 * (1 + obs_waves));
    if (a.obs_w > 32)
      hipLaunchKernelGGL((step_kernel<S, PROBLEM, kModeSplit, true, true>), grid, block, obs_waves * ctx->split_lds_wave, st,
                         PCGRL_STEP_ARGS(a));
    else if (a.use_frozen)
      hipLaunchKernelGGL((step_kernel<S, PROBLEM, kModeSplit, true, false>), grid, block, obs_waves * ctx->split_lds_wave, st,
                         PCGRL_STEP_ARGS(a));
    else
      hipLaunchKernelGGL((step_kernel<S, PROBLEM, kModeSplit, false, false>), grid, block, obs_waves * ctx->split_lds_wave, st,
                         PCGRL_STEP_ARGS(a));
    return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
  }
};
template <int S, int PROBLEM> struct LaunchRolloutSplit {
  static int run(const pcgrl_ctx* ctx, const KArgs& a, hipStream_t st) {
    const int obs_waves = (ctx->roll_m / ctx->roll_o) << ((a.envs_per_wave_log2 >> 16) & 0xff);
    hipLaunchKernelGGL((rollout_kernel<S, PROBLEM, kModeRolloutSplit>), dim3(ctx->roll_groups),
                       dim3(64 * (1 + obs_waves)), obs_waves * ctx->roll_lds_wave, st, a);
    return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
  }
};
template <int S, int PROBLEM> struct LaunchRollout {
  static int run(const pcgrl_ctx* ctx, const KArgs& a, hipStream_t st) {
    hipLaunchKernelGGL((rollout_kernel<S, PROBLEM, kModeRollout>), dim3(ctx->nwaves), dim3(64), ctx->lds_bytes, st, a);
    return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
  }
};
template <int S, int PROBLEM> struct LaunchInit {
  static int run(const pcgrl_ctx* ctx, const KArgs& a, hipStream_t st) {
    hipLaunchKernelGGL((init_kernel<S, PROBLEM>), dim3(ctx->nwaves), dim3(64), ctx->lds_bytes, st, a);
    return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
  }
};

template <int S, int PROBLEM> struct LaunchExact {
  static int run(const pcgrl_ctx* ctx, const KArgs& a, int32_t* out, int parts_log2, hipStream_t st) {
    hipLaunchKernelGGL((exact_diameter_kernel<S, PROBLEM>), dim3((unsigned)ctx->nwaves << parts_log2), dim3(64),
                       ctx->lds_bytes, st, a, out, parts_log2);
    return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
  }
};

// Exact diameters into `out`, the sources of every level shared out over 1 << parts_log2
// workgroups whose partial results go through `partial` ([parts][batch] ints, unused for one part).
int exact_diameter_with(pcgrl_ctx* ctx, int32_t* out, int32_t* partial, int parts_log2, hipStream_t st) {
  if (parts_log2 == 0) return dispatch<LaunchExact>(ctx->S, ctx->cfg.problem, ctx, ctx->base, out, 0, st);
  int rc = dispatch<LaunchExact>(ctx->S, ctx->cfg.problem, ctx, ctx->base, partial, parts_log2, st);
  if (rc != PCGRL_OK) return rc;
  const int B = ctx->cfg.batch;
  hipLaunchKernelGGL(max_over_parts_kernel, dim3((B + 255) / 256), dim3(256), 0, st, partial, out, B, 1 << parts_log2);
  return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
}

// Partial results of pcgrl_exact_diameter_static, for callers that must not allocate: one array per
// GPU the library runs on, held until the process ends.  The name is a host-side stand-in, not a
// device address; host code uses only the address hipGetSymbolAddress gives for the current device.
constexpr size_t kStaticScratchInts = (size_t)1 << 18;  // 1 MiB
__device__ __align__(256) int32_t scratch[kStaticScratchInts];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, once asked for

// The device address of `scratch` on `device`, which must be the current device.
int static_scratch(int device, int32_t** out) {
  if (device < 0 || device >= kMaxDevices) return PCGRL_E_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PCGRL_E_HIP;
    g_scratch_ptr[device] = static_cast<int32_t*>(ptr);
  }
  *out = g_scratch_ptr[device];
  return PCGRL_OK;
}

// ---- launch shapes.  Results never depend on them; every row below is a measurement on MI355X
// (per-step launches replayed from a HIP graph, rollouts of 100 steps; the figures are in the
// design notes).  A rule table is read top down and the first row whose conditions all hold
// decides; ranges are inclusive.
constexpr int64_t kMax = INT64_MAX;
constexpr int64_t kMB = (int64_t)1 << 20;
struct SplitRule {
  int S;                            // size class (16 / 32 / 64 rows), 0 = any
  int64_t batch_lo, batch_hi;       // environments
  int64_t obs_lo, obs_hi;           // bytes of one level's observation
  int64_t step_lo, step_hi;         // bytes of one step's observations, whole batch
  int problem;                      // -1 = any
  int split;                        // 1: a metrics wavefront and observation wavefronts per workgroup
};
// pcgrl_step.  Two wavefronts per level group shorten the dependent chain of a launch at the price
// of loading the level twice.
const SplitRule kStepSplit[] = {
    {16, 1, 8192, 0, kMax, 0, kMax, -1, 1},           // -10...-25 % per step at batches of 512...8192
    {16, 8193, kMax, 3072, kMax, 256 * kMB + 1, 448 * kMB, -1, 0},  // stored through the cache: +17 %
    {16, 8193, kMax, 1536, kMax, 0, kMax, -1, 1},     // maze16 -13 % at 12 288, -2...-4 % from 32 768; binary16 -3 % at 262 144
    {32, 1, 4096, 0, kMax, 0, kMax, -1, 1},           // dungeon32 -16 % at 256, -7 % at 4096
    {32, 4097, 16384, 8192, kMax, 0, kMax, -1, 1},    // 63-cell window (12 KB a level): -7 % at 16 384
    {64, 1, 4096, 0, kMax, 0, kMax, -1, 1},           // maze64 -12 % at 256, -4 % at 4096; none from 8192 on
    {0, 1, kMax, 0, kMax, 0, kMax, -1, 0},
};
// pcgrl_rollout (each wavefront keeps its own copy of the level for all the steps).
const SplitRule kRolloutSplit[] = {
    {16, 1, 2048, 0, kMax, 0, kMax, -1, 1},           // -35 % per step at 64 and 1024
    {16, 2049, 12288, 0, 4095, 0, kMax, -1, 1},       // binary16 +39 % steps/s at 4096, +22 % at 8192
    {16, 12289, kMax, 1536, 4095, 0, kMax, -1, 1},    // binary16 -5...-9 % per step from 16 384 to 131 072
    {16, 2049, 4096, 4096, kMax, 0, kMax, -1, 1},     // maze16 -20 % at 4096
    {16, 16384, kMax, 4096, kMax, 0, kMax, -1, 1},    // maze16 -2...-3 % (at 8192: +6 %, hence the gap)
    {32, 1, 4096, 0, kMax, 0, kMax, -1, 1},           // -43 % at 256, -24 % at 4096
    {32, 4097, kMax, 0, kMax, 0, kMax, PCGRL_BINARY, 1},  // +10 % steps/s at 16 384 (dungeon: +-2 %)
    {64, 1, 8192, 0, kMax, 0, kMax, -1, 1},           // -6 %
    {0, 1, kMax, 0, kMax, 0, kMax, -1, 0},
};
template <size_t N>
int first_match(const SplitRule (&table)[N], int S, int64_t batch, int64_t obs, int64_t step_bytes, int problem) {
  for (const SplitRule& r : table)
    if ((r.S == 0 || r.S == S) && batch >= r.batch_lo && batch <= r.batch_hi && obs >= r.obs_lo && obs <= r.obs_hi &&
        step_bytes >= r.step_lo && step_bytes <= r.step_hi && (r.problem < 0 || r.problem == problem))
      return r.split;
  return 0;
}
// As many levels per wavefront (a power of two up to G) as still leave `min_groups` wavefronts.
int levels_per_wave_for(int G, int batch, int min_groups) {
  int n = G;
  while (n > 1 && (batch + n - 1) / n < min_groups) n /= 2;
  return n;
}

// Into how many parts (a power of two, at most one per row) pcgrl_exact_diameter splits the
// sources of a level: enough for about four thousand wavefronts.
int exact_parts_for(int nwaves, int S) {
  int lg = 0;
  while ((1 << (lg + 1)) <= S && ((long long)nwaves << (lg + 1)) <= 4096) ++lg;
  return lg;
}

int launch_init(pcgrl_ctx* ctx, int flags, uint64_t seed, uint8_t* obs, hipStream_t st) {
  KArgs a = ctx->base;
  a.flags = flags;
  a.seed = seed;
  a.obs = obs;
  return dispatch<LaunchInit>(ctx->S, ctx->cfg.problem, ctx, a, st);
}

// How a pcgrl_step launch stores its observations when the configuration leaves the choice open.
// What matters is whether the bytes stay in the 256 MB memory-side cache: a caller that rewrites
// one buffer every step (a policy in the loop) keeps it there, and write-through stores are the
// fastest way in; a caller that gives every step a slot of its own (a learner keeping the
// rollout) sends every byte to HBM, where write-through stores are the slowest kind (measured,
// 64x64 maze at a batch of 8192, 28 slots of 39 MB: 22.9 us per step against 19.5 with ordinary
// and 17.6 with non-temporal stores; 17.1 with one buffer and write-through stores).  The library
// sees only pointers, so it remembers those of the last 32 calls and takes the bytes of the
// distinct buffers among them as the working set.  Tuning only: results do not depend on it.
int step_store_kind(pcgrl_ctx* ctx, const uint8_t* obs) {
  ctx->recent_obs[ctx->recent_n++ & 31u] = obs;
  const unsigned filled = ctx->recent_n < 32u ? ctx->recent_n : 32u;
  unsigned distinct = 0;
  for (unsigned i = 0; i < filled; ++i) {
    bool seen = false;
    for (unsigned j = 0; j < i; ++j) seen = seen || ctx->recent_obs[j] == ctx->recent_obs[i];
    distinct += seen ? 0u : 1u;
  }
  const size_t step_bytes = (size_t)ctx->cfg.batch * ctx->obs_stride;
  if (distinct <= 1) return ctx->store_step;
  if ((size_t)distinct * step_bytes <= ((size_t)256 << 20)) return kStoreThrough;
  // (where one step alone writes several times what the L2s hold, and in large pieces, ordinary
  // stores are ahead: 32x32 levels with a 63-cell window, 195 MB a step, 41 against 48 us)
  return (step_bytes >= ((size_t)128 << 20) && ctx->obs_bytes >= 3072) ? kStoreCached : kStoreStream;
}

}  // namespace

extern "C" {

const char* pcgrl_strerror(int code) {
  switch (code) {
    case PCGRL_OK: return "ok";
    case PCGRL_E_NULL: return "a required pointer is NULL";
    case PCGRL_E_CONFIG: return "configuration field out of range";
    case PCGRL_E_HIP: return "HIP runtime call failed";
    case PCGRL_E_NOMEM: return "device allocation failed";
    case PCGRL_E_DEVICE: return "no such device, or not a gfx950 device";
    case PCGRL_E_SCRATCH: return "the call needs more partial results than the library's static scratch array holds";
    default: return "unknown error code";
  }
}

int pcgrl_config_default(int32_t problem, pcgrl_config* cfg) {
  if (!cfg) return PCGRL_E_NULL;
  const int K = tiles_of(problem);
  if (K == 0) return PCGRL_E_CONFIG;
  std::memset(cfg, 0, sizeof(*cfg));
  cfg->problem = problem;
  cfg->batch = 1;
  cfg->max_h = cfg->max_w = cfg->min_h = cfg->min_w = 16;
  cfg->obs_w = 31;
  cfg->pad_mode = PCGRL_PAD_BORDER;
  cfg->pos_mode = PCGRL_POS_SCAN;
  cfg->max_steps = 1000;
  cfg->autoreset = 1;
  cfg->regions_mode = PCGRL_REGIONS_INCREMENTAL;
  for (int j = 0; j < 8; ++j) cfg->pinpoint_tile[j] = -1;
  for (int k = 0; k < K; ++k)
    cfg->init_cdf[k] = k == K - 1 ? 0xFFFFFFFFu : (uint32_t)(((uint64_t)(k + 1) << 32) / (uint64_t)K);
  const int BIG = 64 * 64;  // no path is this long: "as long as possible"
  const int base = problem == PCGRL_DUNGEON ? 3 : 2;
  const int M = metrics_of(problem);
  for (int i = 0; i < M; ++i) {
    cfg->target_lo[i] = 0;
    cfg->target_hi[i] = BIG;
  }
  cfg->weights[0] = 5.0f;  // regions: exactly one
  cfg->target_lo[0] = cfg->target_hi[0] = 1;
  cfg->weights[1] = 2.0f;  // path / diameter: maximise
  cfg->target_lo[1] = cfg->target_hi[1] = BIG;
  if (problem == PCGRL_MAZE) {
    for (int t = 2; t <= 3; ++t) {  // one player, one door
      cfg->weights[base + t] = 3.0f;
      cfg->target_lo[base + t] = cfg->target_hi[base + t] = 1;
    }
  } else if (problem == PCGRL_DUNGEON) {
    cfg->weights[2] = 2.0f;  // nearest enemy at least 4 away
    cfg->target_lo[2] = 4;
    cfg->target_hi[2] = BIG;
    for (int t = 2; t <= 4; ++t) {  // one player, key, door
      cfg->weights[base + t] = 3.0f;
      cfg->target_lo[base + t] = cfg->target_hi[base + t] = 1;
    }
    cfg->weights[base + 5] = 3.0f;  // two to five enemies
    cfg->target_lo[base + 5] = 2;
    cfg->target_hi[base + 5] = 5;
  }
  return PCGRL_OK;
}

int pcgrl_create(pcgrl_ctx** out, const pcgrl_config* cfg, int device) {
  if (!out || !cfg) return PCGRL_E_NULL;
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc != PCGRL_OK) return rc;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return PCGRL_E_DEVICE;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return PCGRL_E_DEVICE;
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return PCGRL_E_DEVICE;
  DeviceGuard guard(device);
  if (!guard.ok) return PCGRL_E_DEVICE;

  pcgrl_ctx* ctx = new (std::nothrow) pcgrl_ctx();
  if (!ctx) return PCGRL_E_NOMEM;
  ctx->cfg = *cfg;
  ctx->device = device;
  const int side = cfg->max_h > cfg->max_w ? cfg->max_h : cfg->max_w;
  ctx->S = side <= 16 ? 16 : side <= 32 ? 32 : 64;
  ctx->G = 64 / ctx->S;
  ctx->K = tiles_of(cfg->problem);
  ctx->P = planes_of(cfg->problem);
  ctx->M = metrics_of(cfg->problem);
  ctx->C = ctx->K + (cfg->pad_mode == PCGRL_PAD_BORDER ? 1 : 0) + (cfg->obs_frozen_channel ? 1 : 0);
  // Levels per wavefront: all G groups when the batch alone fills the machine; fewer (the spare
  // groups then hold copies that share the observation work) when that is what it takes to have
  // about two wavefronts on each of the 1024 SIMDs (measured optimum).
  ctx->epw = levels_per_wave_for(ctx->G, cfg->batch, 2048);
  if (cfg->levels_per_wave > 0) {  // explicit choice, rounded down to what the size class allows
    ctx->epw = 1;
    while (ctx->epw * 2 <= cfg->levels_per_wave && ctx->epw * 2 <= ctx->G) ctx->epw *= 2;
  }
  ctx->nwaves = (cfg->batch + ctx->epw - 1) / ctx->epw;
  ctx->B_pad = (cfg->batch + ctx->G - 1) / ctx->G * ctx->G;
  ctx->word_bytes = ctx->S == 64 ? 8 : 4;
  const size_t E1 = (size_t)ctx->C * cfg->obs_w * cfg->obs_w;  // one-hot cells of one observation
  const size_t E = cfg->obs_format == PCGRL_OBS_PACKED ? (E1 + 7) / 8 : E1;  // its bytes
  ctx->obs_bytes = E;
  // Distance between the observations of consecutive levels: dense, a pitch given in bytes, or
  // the next multiple of a 128-byte cache line (the bytes in between are written as zeros).
  ctx->obs_stride = cfg->obs_pitch == PCGRL_OBS_PITCH_LINES ? (E + 127) / 128 * 128
                    : cfg->obs_pitch > 0 ? (size_t)cfg->obs_pitch : E;
  if (ctx->obs_stride < E) {
    delete ctx;
    return PCGRL_E_CONFIG;
  }
  // (the staging stream holds one bit per output byte, or per output bit when packed)
  const size_t stride_bits = cfg->obs_format == PCGRL_OBS_PACKED ? ctx->obs_stride * 8 : ctx->obs_stride;
  // (rounded up to whole 16-byte pieces: the kernels clear it 16 bytes per lane at a time)
  auto lds_for = [&](int levels) {
    return (((8 * 15 + (size_t)levels * (stride_bits + 8) + 31) / 32 + 6) * 4 + 15) / 16 * 16;
  };
  ctx->lds_bytes = lds_for(ctx->epw);
  if (ctx->lds_bytes > 64 * 1024) {
    delete ctx;
    return PCGRL_E_CONFIG;
  }
  // One wavefront per level group, or a metrics wavefront and observation wavefronts: by table.
  const size_t obs_batch_bytes = ctx->obs_stride * (size_t)cfg->batch;
  ctx->split = first_match(kStepSplit, ctx->S, cfg->batch, (int64_t)E, (int64_t)obs_batch_bytes, cfg->problem);
  ctx->split_roll = first_match(kRolloutSplit, ctx->S, cfg->batch, (int64_t)E, (int64_t)obs_batch_bytes, cfg->problem);
  const bool obs_heavy = E >= 4096;
  if (cfg->split_step == PCGRL_SPLIT_OFF) ctx->split = ctx->split_roll = 0;
  if (cfg->split_step == PCGRL_SPLIT_ON) ctx->split = ctx->split_roll = 1;
  // Shape of the split step: one metrics wavefront carries as many levels as the explicit choice
  // (or the automatic one above) says, and the observation can be shared out over several
  // wavefronts of split_o levels each (measured: within 3 % of one observation wavefront, which
  // stays the default).
  // With two wavefronts per workgroup, fewer and fuller workgroups do better than the rule above
  // gives (measured on 16x16 levels, batches of 512 to 8192: about a thousand workgroups where
  // the observation is the larger half of the work, about five hundred where it is not; with a
  // large observation two levels per wavefront, whose two copies halve the channels a lane
  // writes, stay ahead of four up to 2048 workgroups).
  ctx->split_m = ctx->epw;
  if (cfg->levels_per_wave <= 0) {
    const bool large_obs = E >= 3072;
    ctx->split_m = levels_per_wave_for(ctx->G, cfg->batch, large_obs ? 1024 : 512);
    if (large_obs && ctx->split_m == 4 && (cfg->batch + 1) / 2 <= 2048) ctx->split_m = 2;
  }
  ctx->split_o = ctx->split_m;
  if (cfg->split_obs_levels > 0) {
    ctx->split_o = 1;
    while (ctx->split_o * 2 <= cfg->split_obs_levels && ctx->split_o * 2 <= ctx->split_m) ctx->split_o *= 2;
  }
  ctx->split_groups = (cfg->batch + ctx->split_m - 1) / ctx->split_m;
  ctx->split_lds_wave = lds_for(ctx->split_o);
  // The split rollout is bound by instruction issue sooner than a single step is by its chain:
  // it packs as many levels into a wavefront as leave about a thousand workgroups (measured).
  ctx->roll_m = levels_per_wave_for(ctx->G, cfg->batch, 1024);
  // Observation wavefronts of a split rollout: one for all the levels of the metrics wavefront
  // where the observation is small, two (or one per level) where it is the larger half of the
  // work (measured on 16x16 levels: maze16 at 4096, 2.8 against 3.2 us per step; binary16 at
  // 16 384, 6.4 against 7.6 the other way round).
  ctx->roll_o = ctx->roll_m;
  if (ctx->S == 16 && obs_heavy && ctx->roll_m >= 2) ctx->roll_o = ctx->roll_m / 2;
  if (cfg->levels_per_wave > 0) ctx->roll_m = ctx->roll_o = ctx->split_m;
  if (cfg->split_obs_levels > 0) ctx->roll_o = ctx->split_o < ctx->roll_m ? ctx->split_o : ctx->roll_m;
  ctx->roll_groups = (cfg->batch + ctx->roll_m - 1) / ctx->roll_m;
  ctx->roll_lds_wave = lds_for(ctx->roll_o);
  if (ctx->roll_lds_wave * (ctx->roll_m / ctx->roll_o) > 64 * 1024) ctx->split_roll = 0;
  // A small batch leaves most SIMDs idle while every wavefront runs one long dependent chain per
  // step.  The observation wavefronts then take the steps in turn: each follows the level through
  // all the edits (a few dozen instructions a step) and builds the observation of every n-th step
  // only.  As many turns (1, 2, 4) as keep the launch at two wavefronts per SIMD (2048 in all;
  // three where the observation is the longer half of the work) and a workgroup at four
  // observation wavefronts.  Measured, us per step with 1 / 2 / 4 turns: 16x16 maze at a batch of
  // 64 1.46 / 0.95 / 0.92, at 512 1.59 / 1.09 / 1.26, at 1024 1.80 / 1.47 / 2.31, at 2048 2.29 /
  // 2.95 / 2.97; 64x64 maze at 64 1.42 / 1.26 / 1.24; 32x32 dungeon at 512 1.58 / 1.50 / 1.47, at
  // 1024 1.55 / 1.61 / 2.66; 16x16 binary at 64 1.21 / 1.18 / 1.16 (its metrics wavefront is the
  // longer one).
  {
    const int per_step = ctx->roll_m / ctx->roll_o;
    auto fits = [&](int turns) {
      return per_step * turns <= 4 && ctx->roll_lds_wave * per_step * turns <= 64 * 1024;
    };
    const long long most_waves = obs_heavy ? 3072 : 2048;
    ctx->roll_turns = 1;
    if (cfg->rollout_turns > 0) {
      while (ctx->roll_turns * 2 <= cfg->rollout_turns && fits(ctx->roll_turns * 2)) ctx->roll_turns *= 2;
    } else {
      while (fits(ctx->roll_turns * 2) && (long long)ctx->roll_groups * (1 + per_step * ctx->roll_turns * 2) <= most_waves)
        ctx->roll_turns *= 2;
    }
  }

  ctx->exact_parts_log2 = exact_parts_for(ctx->nwaves, ctx->S);
  const size_t rows = (size_t)ctx->B_pad * ctx->S;
  struct { void** p; size_t n; } allocs[] = {
      // (the binary problem keeps one more plane: the component of the first walkable cell)
      {&ctx->d_planes, rows * ctx->word_bytes * (ctx->P + (cfg->problem == PCGRL_BINARY ? 1 : 0))},
      {&ctx->d_frozen, rows * ctx->word_bytes},
      {&ctx->d_env, (size_t)ctx->B_pad * sizeof(EnvRec)},
      {&ctx->d_metrics, (size_t)ctx->B_pad * kMaxMetrics * sizeof(int32_t)},
      // (one more row in front of the target ranges holds the reward weights: a step reads both
      // through the one pointer it has at hand when it issues its loads)
      {&ctx->d_targets, ((size_t)ctx->B_pad + 1) * kMaxMetrics * sizeof(uint32_t)},
      {&ctx->d_bad, sizeof(unsigned long long)},
      {&ctx->d_exact, ctx->exact_parts_log2 ? ((size_t)cfg->batch << ctx->exact_parts_log2) * sizeof(int32_t) : 0},
  };
  for (auto& al : allocs) *al.p = nullptr;
  for (auto& al : allocs) {
    if (al.n == 0) continue;
    if (hipMalloc(al.p, al.n) != hipSuccess || hipMemset(*al.p, 0, al.n) != hipSuccess) {
      for (auto& f : allocs)
        if (*f.p) (void)hipFree(*f.p);
      delete ctx;
      return PCGRL_E_NOMEM;
    }
  }

  KArgs& a = ctx->base;
  std::memset(&a, 0, sizeof(a));
  a.planes = ctx->d_planes;
  a.frozen = ctx->d_frozen;
  a.env = static_cast<EnvRec*>(ctx->d_env);
  a.metrics = static_cast<int32_t*>(ctx->d_metrics);
  a.targets = static_cast<uint32_t*>(ctx->d_targets) + kMaxMetrics;
  a.bad_actions = static_cast<unsigned long long*>(ctx->d_bad);
  if (hipMemcpy(ctx->d_targets, cfg->weights, kMaxMetrics * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) {
    for (auto& f : allocs)
      if (*f.p) (void)hipFree(*f.p);
    delete ctx;
    return PCGRL_E_HIP;
  }
  a.B = cfg->batch;
  a.plane_stride = (int32_t)rows;
  a.max_h = cfg->max_h;
  a.max_w = cfg->max_w;
  a.min_h = cfg->min_h;
  a.min_w = cfg->min_w;
  a.obs_w = cfg->obs_w;
  a.pad_mode = cfg->pad_mode;
  a.pos_mode = cfg->pos_mode;
  a.n_frozen = cfg->n_frozen;
  a.max_steps = cfg->max_steps;
  a.max_changes = cfg->max_changes;
  a.autoreset = cfg->autoreset;
  a.regions_mode = cfg->regions_mode;
  a.env_obs_bytes = (int32_t)ctx->obs_stride;
  a.obs_packed = cfg->obs_format == PCGRL_OBS_PACKED ? 1 : 0;
  a.obs_frozen_channel = cfg->obs_frozen_channel ? 1 : 0;
  a.envs_per_wave_log2 = ctx->epw == 4 ? 2 : ctx->epw == 2 ? 1 : 0;
  a.use_frozen = cfg->n_frozen > 0 ? (cfg->obs_frozen_channel ? 3 : 1) : 0;
  // How the observation is stored (measured on MI355X).  A launch per step ends with the L2
  // write-back of whatever its stores left dirty, after the last wavefront: stores that write
  // through as they are issued overlap that traffic with the rest of the step (13 % of the step
  // at 20 MB of observations per step, a few percent at 200 MB); from about 256 MB per step on,
  // ordinary stores, which the 256 MB last-level cache absorbs, are ahead where one level's
  // observation is large (4.8 KB: 65 against 81 us at 315 MB), non-temporal ones where it is small
  // (1.9 KB: 79 against 86 us at 315 MB, 103 against 135 at 409 MB), and far beyond the cache
  // non-temporal stores in any case.  A rollout launch has no such tail per step, and what counts
  // is the whole ring of observation slots it writes: while that fits the last-level cache, ordinary
  // stores (equal to or up to 6 % ahead of the others at every batch tried); beyond it, ordinary
  // stores for large observations (maze16, a slot per step: 4.4 against 4.9 us per step; maze64
  // 11.0 against 11.8) and for 16-row levels (binary16 at 65 536: 2.1e9 against 2.0e9 steps/s once
  // neighbouring level groups share an L2, which is what a rollout with ordinary stores does),
  // non-temporal ones for the small observations of 32-row levels (dungeon32 9.5 against 10.4).
  // Decided per pcgrl_rollout call, which knows the number of slots.
  {
    const size_t obs_step_bytes = (size_t)cfg->batch * E;
    const size_t MB = (size_t)1 << 20;
    ctx->store_step = obs_step_bytes <= 256 * MB ? kStoreThrough
                      : (obs_step_bytes <= 448 * MB && E >= 3072) ? kStoreCached : kStoreStream;
    ctx->store_roll = -1;  // by ring size, see pcgrl_rollout
    const int forced = cfg->obs_store_mode == PCGRL_OBS_STORE_CACHED ? kStoreCached
                       : cfg->obs_store_mode == PCGRL_OBS_STORE_STREAM ? kStoreStream
                       : cfg->obs_store_mode == PCGRL_OBS_STORE_THROUGH ? kStoreThrough : -1;
    if (forced >= 0) ctx->store_step = ctx->store_roll = forced;
    ctx->store_step_auto = forced < 0;
    a.stream_obs = ctx->store_step;
  }
  for (int k = 0; k < 8; ++k) a.cdf[k] = cfg->init_cdf[k];
  for (int i = 0; i < kMaxMetrics; ++i) {
    a.target_lo[i] = cfg->target_lo[i];
    a.target_hi[i] = cfg->target_hi[i];
    a.ctrl_lo[i] = cfg->ctrl_lo[i];
    a.ctrl_hi[i] = cfg->ctrl_hi[i];
  }
  for (int j = 0; j < 8; ++j) a.pinpoint_tile[j] = cfg->pinpoint_tile[j];
  a.ctrl_mask = cfg->ctrl_mask & ((1u << ctx->M) - 1u);

  rc = launch_init(ctx, kInitGenerate | kInitMetrics | kInitTargets, 0, nullptr, nullptr);
  if (rc == PCGRL_OK && hipDeviceSynchronize() != hipSuccess) rc = PCGRL_E_HIP;
  if (rc != PCGRL_OK) {
    pcgrl_destroy(ctx);
    return rc;
  }
  *out = ctx;
  return PCGRL_OK;
}

int pcgrl_destroy(pcgrl_ctx* ctx) {
  if (!ctx) return PCGRL_OK;
  DeviceGuard guard(ctx->device);  // (freed in any case)
  int rc = guard.ok && hipDeviceSynchronize() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
  void* bufs[] = {ctx->d_planes, ctx->d_frozen, ctx->d_env, ctx->d_metrics, ctx->d_targets, ctx->d_bad, ctx->d_exact};
  for (void* b : bufs)
    if (b && hipFree(b) != hipSuccess) rc = PCGRL_E_HIP;
  delete ctx;
  return rc;
}

int pcgrl_reset(pcgrl_ctx* ctx, uint64_t seed, uint8_t* obs, void* stream) {
  if (!ctx) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  ctx->base.seed = seed;
  return launch_init(ctx, kInitGenerate | kInitMetrics | kInitTargets | kInitObs, seed, obs,
                     static_cast<hipStream_t>(stream));
}

int pcgrl_step(pcgrl_ctx* ctx, const int32_t* actions, uint8_t* obs, float* reward, uint8_t* done,
               void* stream) {
  if (!ctx || !actions) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  KArgs a = ctx->base;
  a.actions = actions;
  a.obs = obs;
  a.reward = reward;
  a.done = done;
  if (obs && ctx->store_step_auto) a.stream_obs = step_store_kind(ctx, obs);
  if (obs && ctx->split) {
    auto lg2 = [](int v) { return v == 4 ? 2 : v == 2 ? 1 : 0; };
    a.envs_per_wave_log2 = lg2(ctx->split_m) | (lg2(ctx->split_o) << 8);
    a.obs_lds_words = (int32_t)(ctx->split_lds_wave / 4);
    return dispatch<LaunchSplit>(ctx->S, ctx->cfg.problem, ctx, a, static_cast<hipStream_t>(stream));
  }
  return dispatch<LaunchStep>(ctx->S, ctx->cfg.problem, ctx, a, static_cast<hipStream_t>(stream));
}

int pcgrl_rollout(pcgrl_ctx* ctx, const int32_t* actions, int32_t n_steps, uint8_t* obs,
                  int32_t obs_slots, float* reward, uint8_t* done, void* stream) {
  if (!ctx || !actions) return PCGRL_E_NULL;
  if (n_steps < 1 || n_steps > (1 << 20)) return PCGRL_E_CONFIG;
  if (obs && (obs_slots < 1 || obs_slots > n_steps)) return PCGRL_E_CONFIG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  KArgs a = ctx->base;
  a.actions = actions;
  a.obs = obs;
  a.reward = reward;
  a.done = done;
  a.rollout_steps = n_steps;
  a.obs_slots = obs ? obs_slots : 1;
  if (ctx->store_roll >= 0) {
    a.stream_obs = ctx->store_roll;
  } else {
    const size_t step_bytes = (size_t)ctx->cfg.batch * ctx->obs_stride;
    const size_t ring = (size_t)a.obs_slots * step_bytes;
    a.stream_obs = (ring <= ((size_t)448 << 20) || ctx->obs_bytes >= 3072 || ctx->S == 16) ? kStoreCached : kStoreStream;
    // With whole cache lines per level no line is written twice, and non-temporal stores are ahead
    // once a step writes 32 MB or more (64x64 maze 8.5 against 8.8 us per step, 32x32 levels with
    // the 63-cell window 37.5 against 40.4, 16x16 maze at a batch of 65 536 60 against 67; at a
    // batch of 4096, 20 MB a step, 4.0 against 3.9).
    if (ring > ((size_t)448 << 20) && (ctx->obs_stride & 127) == 0 && step_bytes >= ((size_t)32 << 20))
      a.stream_obs = kStoreStream;
  }
  // (consecutive level groups on one die: only where neighbouring observations share cache lines)
  a.by_die = (a.stream_obs == kStoreCached && (ctx->obs_stride & 127) != 0) ? 1 : 0;
  if (obs && ctx->split_roll) {
    auto lg2 = [](int v) { return v == 4 ? 2 : v == 2 ? 1 : 0; };
    // Wavefronts that take turns are not ordered among each other: a slot that is written more than
    // once in this rollout must be written by the same wavefront every time, i.e. the number of
    // turns has to divide the number of slots.
    int turns = ctx->roll_turns;
    while (turns > 1 && a.obs_slots != n_steps && a.obs_slots % turns != 0) turns /= 2;
    a.envs_per_wave_log2 = lg2(ctx->roll_m) | (lg2(ctx->roll_o) << 8) | (lg2(turns) << 16);
    a.obs_lds_words = (int32_t)(ctx->roll_lds_wave / 4);
    return dispatch<LaunchRolloutSplit>(ctx->S, ctx->cfg.problem, ctx, a, static_cast<hipStream_t>(stream));
  }
  return dispatch<LaunchRollout>(ctx->S, ctx->cfg.problem, ctx, a, static_cast<hipStream_t>(stream));
}

int pcgrl_metrics(pcgrl_ctx* ctx, int32_t* out, void* stream) {
  if (!ctx || !out) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  const int n = ctx->cfg.batch * ctx->M;
  hipLaunchKernelGGL(copy_metrics_kernel, dim3((n + 255) / 256), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const int32_t*>(ctx->d_metrics),
                     out, ctx->cfg.batch, ctx->M);
  return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
}

int pcgrl_exact_diameter(pcgrl_ctx* ctx, int32_t* out, void* stream) {
  if (!ctx || !out) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  return exact_diameter_with(ctx, out, static_cast<int32_t*>(ctx->d_exact), ctx->exact_parts_log2,
                             static_cast<hipStream_t>(stream));
}

int pcgrl_exact_diameter_static(pcgrl_ctx* ctx, int32_t* out, int32_t parts_log2, void* stream) {
  if (!ctx || !out) return PCGRL_E_NULL;
  if (parts_log2 < -1 || (parts_log2 >= 0 && (1 << parts_log2) > ctx->S)) return PCGRL_E_CONFIG;
  const int lg = parts_log2 < 0 ? ctx->exact_parts_log2 : parts_log2;
  const size_t need = lg ? ((size_t)ctx->cfg.batch << lg) : 0;  // ints of partial results
  if (need > kStaticScratchInts) return PCGRL_E_SCRATCH;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  int32_t* partial = nullptr;
  if (lg) {
    const int rc = static_scratch(ctx->device, &partial);
    if (rc != PCGRL_OK) return rc;
  }
  return exact_diameter_with(ctx, out, partial, lg, static_cast<hipStream_t>(stream));
}

int pcgrl_observe(pcgrl_ctx* ctx, uint8_t* obs, void* stream) {
  if (!ctx || !obs) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  return launch_init(ctx, kInitObs, ctx->base.seed, obs, static_cast<hipStream_t>(stream));
}

int pcgrl_get_state(pcgrl_ctx* ctx, int8_t* tiles, uint8_t* frozen, int16_t* hw, int16_t* pos,
                    int32_t* counters, void* stream) {
  if (!ctx) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  const int n = ctx->cfg.batch * ctx->S;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->S == 64)
    hipLaunchKernelGGL(get_state_kernel<uint64_t>, dim3((n + 255) / 256), dim3(256), 0, st, ctx->base,
                       ctx->S, ctx->P, tiles, frozen, hw, pos, counters);
  else
    hipLaunchKernelGGL(get_state_kernel<uint32_t>, dim3((n + 255) / 256), dim3(256), 0, st, ctx->base,
                       ctx->S, ctx->P, tiles, frozen, hw, pos, counters);
  return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
}

int pcgrl_set_state(pcgrl_ctx* ctx, const int8_t* tiles, const uint8_t* frozen, const int16_t* hw,
                    const int16_t* pos, void* stream) {
  if (!ctx || !tiles || !hw || !pos) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  const int n = ctx->cfg.batch * ctx->S;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->S == 64)
    hipLaunchKernelGGL(set_state_kernel<uint64_t>, dim3((n + 255) / 256), dim3(256), 0, st, ctx->base,
                       ctx->S, ctx->P, ctx->K, tiles, frozen, hw, pos);
  else
    hipLaunchKernelGGL(set_state_kernel<uint32_t>, dim3((n + 255) / 256), dim3(256), 0, st, ctx->base,
                       ctx->S, ctx->P, ctx->K, tiles, frozen, hw, pos);
  if (hipGetLastError() != hipSuccess) return PCGRL_E_HIP;
  if (frozen) ctx->base.use_frozen = ctx->cfg.obs_frozen_channel ? 3 : 1;  // from now on steps have to look pinpoints up
  return launch_init(ctx, kInitMetrics, ctx->base.seed, nullptr, st);
}

int pcgrl_set_targets(pcgrl_ctx* ctx, const int32_t* targets, void* stream) {
  if (!ctx || !targets) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  const int n = ctx->cfg.batch * ctx->M;
  hipLaunchKernelGGL(set_targets_kernel, dim3((n + 255) / 256), dim3(256), 0,
                     static_cast<hipStream_t>(stream), targets, static_cast<uint32_t*>(ctx->d_targets) + kMaxMetrics,
                     ctx->cfg.batch, ctx->M);
  return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
}

int pcgrl_get_targets(pcgrl_ctx* ctx, int32_t* out, void* stream) {
  if (!ctx || !out) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  const int n = ctx->cfg.batch * ctx->M;
  hipLaunchKernelGGL(get_targets_kernel, dim3((n + 255) / 256), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint32_t*>(ctx->d_targets) + kMaxMetrics,
                     out, ctx->cfg.batch, ctx->M);
  return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
}

int pcgrl_obs_shape(const pcgrl_ctx* ctx, int32_t out[4]) {
  if (!ctx || !out) return PCGRL_E_NULL;
  out[0] = ctx->cfg.batch;
  out[1] = ctx->C;
  out[2] = ctx->cfg.obs_w;
  out[3] = ctx->cfg.obs_w;
  return PCGRL_OK;
}

int64_t pcgrl_obs_bytes(const pcgrl_ctx* ctx) { return ctx ? (int64_t)ctx->obs_bytes : PCGRL_E_NULL; }
int64_t pcgrl_obs_stride(const pcgrl_ctx* ctx) { return ctx ? (int64_t)ctx->obs_stride : PCGRL_E_NULL; }

int pcgrl_num_metrics(const pcgrl_ctx* ctx) { return ctx ? ctx->M : PCGRL_E_NULL; }
int pcgrl_num_tiles(const pcgrl_ctx* ctx) { return ctx ? ctx->K : PCGRL_E_NULL; }

int pcgrl_bad_action_count(pcgrl_ctx* ctx, uint64_t* out, void* stream) {
  if (!ctx || !out) return PCGRL_E_NULL;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned long long v = 0;
  if (hipMemcpyAsync(&v, ctx->d_bad, sizeof(v), hipMemcpyDeviceToHost, st) != hipSuccess) return PCGRL_E_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return PCGRL_E_HIP;
  *out = v;
  return PCGRL_OK;
}

int pcgrl_unpack_obs(const pcgrl_ctx* ctx, const uint8_t* packed, void* out, int32_t out_type, void* stream) {
  if (!ctx || !packed || !out) return PCGRL_E_NULL;
  if (ctx->cfg.obs_format != PCGRL_OBS_PACKED) return PCGRL_E_CONFIG;
  if (out_type < PCGRL_UNPACK_U8 || out_type > PCGRL_UNPACK_F32) return PCGRL_E_CONFIG;
  const int es = out_type == PCGRL_UNPACK_U8 ? 1 : out_type == PCGRL_UNPACK_F32 ? 4 : 2;
  if (((uintptr_t)out & (uintptr_t)(es - 1)) != 0) return PCGRL_E_CONFIG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  const int32_t cells = ctx->C * ctx->cfg.obs_w * ctx->cfg.obs_w;
  const dim3 grid((unsigned)ctx->cfg.batch), block(64);
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* o = static_cast<uint8_t*>(out);
  const int64_t stride = (int64_t)ctx->obs_stride;
  if (out_type == PCGRL_UNPACK_U8) hipLaunchKernelGGL(unpack_obs_kernel<1>, grid, block, 0, st, packed, stride, o, cells, 1u);
  else if (out_type == PCGRL_UNPACK_F16) hipLaunchKernelGGL(unpack_obs_kernel<2>, grid, block, 0, st, packed, stride, o, cells, 0x3C00u);
  else if (out_type == PCGRL_UNPACK_BF16) hipLaunchKernelGGL(unpack_obs_kernel<2>, grid, block, 0, st, packed, stride, o, cells, 0x3F80u);
  else hipLaunchKernelGGL(unpack_obs_kernel<4>, grid, block, 0, st, packed, stride, o, cells, 0x3F800000u);
  return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
}

int pcgrl_store_rate(uint8_t* dst, int64_t n_regions, int32_t region_bytes, int32_t store_mode,
                     int32_t order, void* stream) {
  if (!dst) return PCGRL_E_NULL;
  if (n_regions < 1 || region_bytes < 16 || (region_bytes & 15) != 0 || ((uintptr_t)dst & 15u) != 0)
    return PCGRL_E_CONFIG;
  if (order < PCGRL_STORE_ORDER_REGIONS || order > PCGRL_STORE_ORDER_REGIONS_BY_DIE) return PCGRL_E_CONFIG;
  if (order == PCGRL_STORE_ORDER_LINEAR && (region_bytes & 1023) != 0) return PCGRL_E_CONFIG;
  if (store_mode < PCGRL_OBS_STORE_CACHED || store_mode > PCGRL_OBS_STORE_THROUGH) return PCGRL_E_CONFIG;
  const int mode = store_mode == PCGRL_OBS_STORE_CACHED ? kStoreCached
                   : store_mode == PCGRL_OBS_STORE_STREAM ? kStoreStream : kStoreThrough;
  const int64_t grid = n_regions < (1 << 20) ? n_regions : (1 << 20);
  hipLaunchKernelGGL(store_rate_kernel, dim3((unsigned)grid), dim3(64), 0, static_cast<hipStream_t>(stream), dst,
                     n_regions, region_bytes, mode, order == PCGRL_STORE_ORDER_LINEAR ? 1 : 0,
                     order == PCGRL_STORE_ORDER_REGIONS_BY_DIE ? 1 : 0);
  return hipGetLastError() == hipSuccess ? PCGRL_OK : PCGRL_E_HIP;
}

int pcgrl_selftest(int device, int32_t* mismatches) {
  if (!mismatches) return PCGRL_E_NULL;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return PCGRL_E_DEVICE;
  DeviceGuard guard(device);
  if (!guard.ok) return PCGRL_E_DEVICE;
  int32_t* d = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&d), sizeof(int32_t)) != hipSuccess) return PCGRL_E_NOMEM;
  int rc = PCGRL_OK;
  if (hipMemset(d, 0, sizeof(int32_t)) != hipSuccess) rc = PCGRL_E_HIP;
  if (rc == PCGRL_OK) {
    hipLaunchKernelGGL(selftest_kernel, dim3(1), dim3(64), 0, nullptr, d);
    if (hipGetLastError() != hipSuccess) rc = PCGRL_E_HIP;
  }
  if (rc == PCGRL_OK && hipMemcpy(mismatches, d, sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
    rc = PCGRL_E_HIP;
  (void)hipFree(d);
  return rc;
}

}  // extern "C"
