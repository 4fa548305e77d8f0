/*
 * pcgrl.h -- C ABI of the MI355X (gfx950) batched PCGRL environment step.
 *
 * One context owns a batch of level-editing environments resident in GPU memory.  Each call to
 * pcgrl_step applies one tile edit per level, recomputes that level's region / path metrics and
 * tile counts, turns the change of the distance-to-target into a float32 reward, moves the agent
 * on and writes its egocentric, padded one-hot observation (paper: Methods / Training and
 * Methods / Task).  Nothing here allocates per call, synchronises, or touches host copies of the
 * per-environment arrays.
 *
 * Conventions for every entry point
 *   - Return value: PCGRL_OK (0) or a negative PCGRL_E_* code; no exceptions, no aborts.
 *     pcgrl_strerror() names a code.
 *   - "device pointer" = memory on the context's GPU, owned by the caller (for example a PyTorch
 *     tensor's data_ptr()); the library never frees it and never keeps it after the call's
 *     kernels have run.  "host pointer" = ordinary process memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued on
 *     it and the call returns without waiting, unless stated otherwise.
 *   - Calls on one context must be ordered by the caller (same stream, or events).
 *
 * Tile ids.  binary: 0 empty, 1 wall.  maze: 0 empty, 1 wall, 2 player, 3 door.
 *            dungeon: 0 empty, 1 wall, 2 player, 3 key, 4 door, 5 enemy, 6 chest.
 * Every tile except wall can be walked on and belongs to a region.
 *
 * Metric vector (int32, M entries per environment):
 *   [0] regions   number of 4-connected components of walkable cells   (Task / Binary domain)
 *   [1] path      binary : two-sweep diameter estimate of the component of the first walkable
 *                          cell in row-major order                      (Binary domain, footnote)
 *                 maze   : shortest player -> door distance            (Task / Maze domain)
 *                 dungeon: shortest player -> key -> door distance     (Task / Dungeon domain)
 *   [2] nearest enemy distance from the player (dungeon only)           (Task / Dungeon domain)
 *   then the count of each tile id 0..K-1 inside the active map.
 *   M = 4 (binary), 6 (maze), 10 (dungeon).  Distances count edges; a quantity that does not
 *   exist (no source, no destination, no connection) is 0.
 */
#ifndef PCGRL_H
#define PCGRL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PCGRL_OK 0
#define PCGRL_E_NULL (-1)     /* a required pointer is NULL */
#define PCGRL_E_CONFIG (-2)   /* a configuration field is out of range */
#define PCGRL_E_HIP (-3)      /* a HIP runtime call failed */
#define PCGRL_E_NOMEM (-4)    /* device allocation failed */
#define PCGRL_E_DEVICE (-5)   /* the device is not a gfx950 part, does not exist or cannot be made current */
#define PCGRL_E_SCRATCH (-6)  /* pcgrl_exact_diameter_static: more partial results than its static array holds */

#define PCGRL_BINARY 0
#define PCGRL_MAZE 1
#define PCGRL_DUNGEON 2

#define PCGRL_PAD_BORDER 0 /* cells outside the map set an extra channel K (Discussion: border tiles) */
#define PCGRL_PAD_WALL 1   /* cells outside the map read as wall */

#define PCGRL_POS_SCAN 0   /* row-major scan of the active map, wrapping (Methods / Training) */
#define PCGRL_POS_RANDOM 1 /* seeded uniform position every step */

#define PCGRL_REGIONS_INCREMENTAL 0 /* update the region count from floods around the edited cell */
#define PCGRL_REGIONS_RECOUNT 1     /* count all components again after each modifying edit */

#define PCGRL_OBS_STORE_AUTO 0   /* choose from the bytes of one step's observations (pcgrl_step) or of
                                    all the observation slots of the call (pcgrl_rollout) */
#define PCGRL_OBS_STORE_CACHED 1 /* ordinary stores */
#define PCGRL_OBS_STORE_STREAM 2 /* non-temporal stores */
#define PCGRL_OBS_STORE_THROUGH 3 /* stores that write through the L2 as they are issued */

#define PCGRL_SPLIT_AUTO 0 /* decide from the batch, the level size and the observation size */
#define PCGRL_SPLIT_OFF 1  /* one wavefront per level group does the whole step */
#define PCGRL_SPLIT_ON 2   /* pcgrl_step and pcgrl_rollout run a metrics wavefront and observation
                              wavefronts per group of levels (each holds the levels itself) */

#define PCGRL_OBS_ONEHOT_U8 0 /* uint8 [batch][C][obs_w][obs_w], one byte per one-hot cell */
#define PCGRL_OBS_PACKED 1    /* the same cells as bits: uint8 [batch][ceil(C*obs_w*obs_w / 8)], cell j of
                                 a level (j = (c*obs_w + i)*obs_w + k) is bit j%8 of its byte j/8;
                                 eight times fewer bytes for a consumer that unpacks on the fly */

#define PCGRL_MAX_METRICS 16
#define PCGRL_MAX_TILES 8

typedef struct pcgrl_ctx pcgrl_ctx; /* opaque; owns its device state */

typedef struct {
  int32_t problem;      /* PCGRL_BINARY / MAZE / DUNGEON                     (Methods / Task) */
  int32_t batch;        /* number of environments, >= 1 */
  int32_t max_h, max_w; /* buffer that holds every map shape, each in 1..64 */
  int32_t min_h, min_w; /* equal to max_* for a fixed shape; otherwise height and width are drawn
                           uniformly and independently in [min, max] at the start of every episode
                           and the map sits in the top-left corner (Task / Randomized map shapes) */
  int32_t obs_w;        /* side of the observation window, 1..63; the agent's cell is cell
                           (obs_w/2, obs_w/2) of the window             (Methods / Training) */
  int32_t pad_mode;     /* PCGRL_PAD_* */
  int32_t pos_mode;     /* PCGRL_POS_* */
  int32_t n_frozen;     /* pinpoint cells per episode, 0..8: distinct seeded cells of the active
                           map that keep their initial tile                (Task / Pinpoint tiles) */
  int32_t max_steps;    /* >= 1; done when the episode's step count reaches it */
  int32_t max_changes;  /* 0 = off; otherwise done when that many edits modified the map */
  int32_t autoreset;    /* non-zero: a finished episode is replaced by a fresh seeded one inside
                           the same step; reward and done describe the finished transition, the
                           observation and cached metrics the new episode's first state */
  int32_t regions_mode; /* PCGRL_REGIONS_*; both give the same counts */
  int32_t levels_per_wave; /* tuning only, results do not depend on it: 0 = automatic; 1, 2 or 4 =
                           how many levels share one 64-lane wavefront (at most 64 / S, S = 16, 32
                           or 64 covering max_h and max_w; larger requests are rounded down) */
  int32_t obs_store_mode;  /* tuning only: PCGRL_OBS_STORE_* */
  int32_t split_step;      /* tuning only: PCGRL_SPLIT_* */
  int32_t obs_format;      /* PCGRL_OBS_*: every `obs` argument below has this format */
  uint32_t init_cdf[PCGRL_MAX_TILES]; /* non-decreasing cumulative tile probabilities scaled by
                           2^32 (entry k = P(tile <= k)); the last tile takes the rest; all zero =
                           start from an all-empty map                      (Methods / Task) */
  float weights[PCGRL_MAX_METRICS];     /* reward weight of each metric      (Methods / Training) */
  int32_t target_lo[PCGRL_MAX_METRICS]; /* default target range of each metric (clamped to */
  int32_t target_hi[PCGRL_MAX_METRICS]; /* 0..65535); the loss of a metric v is max(0, lo - v, v - hi) */
  int32_t pinpoint_tile[8]; /* tile id written to the j-th pinpoint cell when an episode starts, so
                           that pivotal tiles (player, door, key) sit frozen at seeded cells;
                           -1 keeps the tile drawn there               (Task / Pinpoint tiles) */
  uint32_t ctrl_mask;   /* bit i set: metric i is controlled -- at every episode start its target
                           becomes one value drawn uniformly from [ctrl_lo[i], ctrl_hi[i]]
                           (0 <= lo <= hi <= 65535), lo = hi = that value  (Methods / Training:
                           the user or a curriculum varies target path length or nearest enemy) */
  int32_t ctrl_lo[PCGRL_MAX_METRICS];
  int32_t ctrl_hi[PCGRL_MAX_METRICS];
  int32_t obs_frozen_channel; /* non-zero: the observation gets one more (last) channel that is 1 on
                           the pinpoint cells in view, so that the agent can see what it cannot edit */
  int32_t split_obs_levels; /* tuning only: when a step runs as metrics wavefront + observation
                           wavefronts (PCGRL_SPLIT_*), how many levels one observation wavefront
                           writes: 0 = automatic; 1, 2 or 4, at most what the metrics wavefront
                           holds (levels_per_wave); each workgroup then has that many more
                           observation wavefronts */
  int32_t obs_pitch;    /* layout of every `obs` argument: 0 = dense, one level's observation
                           directly after the other; > 0 = bytes from one level's observation to the
                           next (a multiple of 16, not less than the observation itself);
                           PCGRL_OBS_PITCH_LINES = the observation's size rounded up to a multiple
                           of 128 bytes, so that no two levels share a cache line (stores whose
                           lines are written by one wavefront only reach memory about half as fast
                           again).  The bytes between two observations are written as zeros.  The
                           caller sees [batch][pitch] bytes, e.g. as a strided [batch][C][ow][ow] view */
  int32_t rollout_turns; /* tuning only, results do not depend on it: 0 = automatic; 1, 2 or 4 = how
                           many observation wavefronts take the steps of a pcgrl_rollout in turn
                           (each keeps its own copy of the levels and writes the observation of
                           every n-th step).  Pays where the batch leaves most of the chip idle:
                           the automatic choice takes turns only while every wavefront still has
                           a SIMD to itself; a workgroup holds at most four observation wavefronts */
} pcgrl_config;

#define PCGRL_OBS_PITCH_LINES (-1)

/* Fills *cfg with this library's defaults for a problem: fixed 16x16 map, window 31, border
 * padding, scan order, no pinpoints, no controlled metric, 1000 steps, autoreset, uniform initial
 * tiles, and the reward
 * table (one region, path as long as possible, one player / key / door, 2..5 enemies, nearest
 * enemy >= 4).  cfg: host pointer. */
int pcgrl_config_default(int32_t problem, pcgrl_config* cfg);

/* Creates a context on GPU `device` and allocates all device state (about
 * 3*S*8 + 170 bytes per environment, S = 16, 32 or 64 covering max_h and max_w): the many
 * environments that are stepped in lockstep on one GPU (Methods / Jax implementation; no passage
 * defines the call itself).  The environments start as if pcgrl_reset(seed = 0) had been called.
 * Synchronises.
 * cfg, out: host pointers.  Errors: E_NULL, E_CONFIG, E_DEVICE, E_NOMEM, E_HIP. */
int pcgrl_create(pcgrl_ctx** out, const pcgrl_config* cfg, int device);

/* Frees the context and its device memory (no passage of the paper: resource management).
 * Synchronises the device first.  NULL is accepted. */
int pcgrl_destroy(pcgrl_ctx* ctx);

/* Starts episode 0 of every environment from `seed` (Methods / Task: the initial map is drawn
 * tile by tile from a weighted distribution, or left empty; Task / Randomized map shapes; Task /
 * Pinpoint tiles): shape, tiles, pinpoints, first position (all from a counter-based generator
 * keyed by seed, global environment index and episode, so results do not depend on batch size),
 * default target ranges, full metrics.
 * obs: device pointer, uint8 [batch][C][obs_w][obs_w], or NULL to skip the observation. */
int pcgrl_reset(pcgrl_ctx* ctx, uint64_t seed, uint8_t* obs, void* stream);

/* One environment step for the whole batch (Methods / Training; Methods / Task).
 *   actions: device, int32 [batch]; the tile to write at the agent's cell.  A value outside
 *            0..K-1 is a no-op edit (counted, see pcgrl_bad_action_count); so is writing the tile
 *            already there or writing to a frozen cell.
 *   obs    : device, uint8 [batch][C][obs_w][obs_w], planar one-hot window centred on the agent's
 *            NEW cell; C = K, plus 1 under PCGRL_PAD_BORDER, plus 1 with obs_frozen_channel
 *            (bit-packed under PCGRL_OBS_PACKED).  May be NULL.
 *   reward : device, float32 [batch]: sum over metrics, in index order, of
 *            weight * (loss before - loss after), each product and each partial sum rounded to
 *            float32 (no fused multiply-add); exactly 0 when the edit was a no-op.
 *   done   : device, uint8 [batch].
 * reward and done may be NULL.
 * The call only enqueues one kernel launch, so it may be captured into a HIP graph; a captured
 * launch keeps the arguments, the reset seed and the context's host-side settings that were
 * current when it was captured: capture again after pcgrl_reset with another seed and after a
 * pcgrl_set_state that passes a frozen mask to a context configured without pinpoints (from then
 * on steps look pinpoints up, which launches captured before do not). */
int pcgrl_step(pcgrl_ctx* ctx, const int32_t* actions, uint8_t* obs, float* reward, uint8_t* done,
               void* stream);

/* n_steps consecutive environment steps in ONE launch, with results identical to n_steps calls of
 * pcgrl_step; the levels stay in registers in between, so per step only the action is read and
 * the outputs are written (the random-agent rollout of Results / Speed comparison, and the remedy
 * for batches too small to hide a launch per step).
 *   actions: device, int32 [n_steps][batch]
 *   obs    : device, uint8 [obs_slots][batch][C][obs_w][obs_w]; step t writes slot t % obs_slots
 *            (obs_slots = n_steps keeps every observation, 1 keeps only the last).  May be NULL.
 *   reward : device, float32 [n_steps][batch], may be NULL
 *   done   : device, uint8 [n_steps][batch], may be NULL
 * Errors: E_NULL; E_CONFIG if n_steps is not in 1..2^20 or obs_slots is not in 1..n_steps. */
int pcgrl_rollout(pcgrl_ctx* ctx, const int32_t* actions, int32_t n_steps, uint8_t* obs,
                  int32_t obs_slots, float* reward, uint8_t* done, void* stream);

/* Copies the cached metric vectors: the region / path / tile-count measures of Methods / Task
 * (Binary, Maze and Dungeon domains) that the reward is computed from, as listed at the top of
 * this file.  out: device, int32 [batch][M]. */
int pcgrl_metrics(pcgrl_ctx* ctx, int32_t* out, void* stream);

/* Exact diameter of every level: the largest shortest-path distance between any two connected
 * walkable cells (the graph diameter that the two-sweep estimate of Task / Binary domain stands
 * for), by a breadth-first sweep from every walkable cell.  A diagnostic for the error of the
 * two-sweep estimate, not part of a step: the cost grows with (walkable cells) x (eccentricity),
 * about a million vector instructions for one open 64x64 level.  For small batches the sources of
 * a level are shared out over several workgroups, whose partial results go through a buffer that
 * the context owns.  out: device, int32 [batch]. */
int pcgrl_exact_diameter(pcgrl_ctx* ctx, int32_t* out, void* stream);

/* pcgrl_exact_diameter for callers that cannot allocate device memory and want nothing allocated
 * on their behalf (code under HIP graph capture, tight serving loops, harnesses that forbid it):
 * the same kernels and the same results, with the partial results (one int per level and part) in
 * a static device array of the library, 1 MiB = 262 144 ints per GPU, held until the process ends,
 * instead of the context's own buffer.  Calls no allocating routine.
 *   parts_log2: a level's sources are shared out over 1 << parts_log2 workgroups (at most one per
 *               row of the 16 / 32 / 64-row buffer); -1 = what pcgrl_exact_diameter uses.
 * Errors: E_NULL; E_CONFIG if parts_log2 is out of range; E_SCRATCH if batch << parts_log2 exceeds
 * 262 144 (with one part the array is not used and any batch is accepted).
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (different streams or
 * contexts) race; calls ordered on one stream do not.  Nothing in the array has to start at zero
 * (every word that is read was written by the same call). */
int pcgrl_exact_diameter_static(pcgrl_ctx* ctx, int32_t* out, int32_t parts_log2, void* stream);

/* Writes the current observation of every environment without stepping: the egocentric window of
 * Methods / Training around the agent's cell, padded as Discussion (border tiles) describes, in
 * the layout of pcgrl_step's `obs`.  obs: device. */
int pcgrl_observe(pcgrl_ctx* ctx, uint8_t* obs, void* stream);

/* Reads the environments back in a plain layout -- the map of tiles an agent edits (Methods /
 * Training), its frozen cells (Task / Pinpoint tiles) and its shape (Task / Randomized map shapes)
 * (all device pointers, any may be NULL):
 *   tiles int8 [batch][max_h][max_w] (-1 outside the active map), frozen uint8 same shape,
 *   hw int16 [batch][2], pos int16 [batch][2], counters int32 [batch][3] = step count,
 *   modifying edits, episode number. */
int pcgrl_get_state(pcgrl_ctx* ctx, int8_t* tiles, uint8_t* frozen, int16_t* hw, int16_t* pos,
                    int32_t* counters, void* stream);

/* Installs levels chosen by the caller -- the designer-placed layouts of Task / Pinpoint tiles.
 * Same layouts as pcgrl_get_state; frozen may be NULL (nothing frozen), the rest is required.
 * Cells outside hw are ignored; a tile id outside 0..K-1 is stored as empty; hw and pos are
 * clamped into range.  Step and change counters restart at 0, targets are kept, metrics are
 * recomputed from scratch. */
int pcgrl_set_state(pcgrl_ctx* ctx, const int8_t* tiles, const uint8_t* frozen, const int16_t* hw,
                    const int16_t* pos, void* stream);

/* Per-environment target ranges (control targets of Methods / Training).
 * targets: device, int32 [batch][M][2] = (lo, hi), each clamped to 0..65535 (no metric of a
 * 64x64 level exceeds 4096).  They stay in force until the next pcgrl_reset, which restores the
 * configuration's defaults; the targets of controlled metrics (ctrl_mask) are redrawn whenever an
 * episode starts. */
int pcgrl_set_targets(pcgrl_ctx* ctx, const int32_t* targets, void* stream);

/* Copies the target ranges now in force (Methods / Training: a controllable generator observes
 * the targets it is rewarded for approaching; a policy conditioned on them reads them here).
 * out: device, int32 [batch][M][2]. */
int pcgrl_get_targets(pcgrl_ctx* ctx, int32_t* out, void* stream);

/* Shape queries (host side, no GPU work).  The observation is one channel per tile type over the
 * window of Methods / Training (plus the border channel of Discussion, plus the pinpoint channel
 * if configured).  out: host pointer to 4 ints = batch, C, obs_w, obs_w. */
int pcgrl_obs_shape(const pcgrl_ctx* ctx, int32_t out[4]);
int64_t pcgrl_obs_bytes(const pcgrl_ctx* ctx); /* bytes of one level's observation in obs_format */
int64_t pcgrl_obs_stride(const pcgrl_ctx* ctx); /* bytes from one level's observation to the next
                                                    (pcgrl_obs_bytes, or the pitch obs_pitch asks for);
                                                    an `obs` argument holds batch times this many bytes */
int pcgrl_num_metrics(const pcgrl_ctx* ctx);
int pcgrl_num_tiles(const pcgrl_ctx* ctx);

/* Number of out-of-range actions seen since creation.  Waits for `stream`.  out: host pointer. */
int pcgrl_bad_action_count(pcgrl_ctx* ctx, uint64_t* out, void* stream);

/* The consumer's side of PCGRL_OBS_PACKED (Methods, model figure: the observation feeds the
 * first convolution of the policy and value networks): turns bit-packed observations, as every
 * `obs` argument of a context with obs_format = PCGRL_OBS_PACKED holds them, back into one-hot
 * elements of the type a network wants, so that a rollout can be kept in HBM at an eighth of its
 * size and widened only when it is read.
 *   packed : device, uint8 [batch][pcgrl_obs_stride(ctx)], one call's worth (one slot of a rollout)
 *   out    : device, [batch][C][obs_w][obs_w] contiguous elements of out_type (aligned to the
 *            element size), each 0 or 1
 *   out_type: PCGRL_UNPACK_U8 / _F16 / _BF16 / _F32
 * Errors: E_NULL; E_CONFIG if the context's format is not packed, out_type is unknown or out is
 * misaligned. */
#define PCGRL_UNPACK_U8 0
#define PCGRL_UNPACK_F16 1
#define PCGRL_UNPACK_BF16 2
#define PCGRL_UNPACK_F32 3
int pcgrl_unpack_obs(const pcgrl_ctx* ctx, const uint8_t* packed, void* out, int32_t out_type, void* stream);

/* Measurement aid (no passage of the paper: it is the yardstick its store-bound steps are held
 * against).  One launch that does nothing but write n_regions * region_bytes bytes to dst with
 * aligned 16-byte stores of the kind `store_mode` names (PCGRL_OBS_STORE_CACHED / _STREAM /
 * _THROUGH).  order: PCGRL_STORE_ORDER_REGIONS = one wavefront per contiguous region of
 * region_bytes, workgroup b takes region b -- the pattern of the observation writer of a step;
 * _REGIONS_BY_DIE = the same with consecutive regions on the same accelerator die, as a rollout
 * deals them; _LINEAR = one sweep in which consecutive wavefronts write consecutive 1 KiB pieces.
 * dst: device pointer on the current device (there is no context), 16-byte aligned, at least
 * n_regions * region_bytes bytes; its contents afterwards are unspecified.
 * Errors: E_NULL; E_CONFIG if n_regions < 1, region_bytes is not a positive multiple of 16 (of
 * 1024 for the linear order), dst is misaligned, or store_mode / order is out of range. */
#define PCGRL_STORE_ORDER_REGIONS 0
#define PCGRL_STORE_ORDER_LINEAR 1
#define PCGRL_STORE_ORDER_REGIONS_BY_DIE 2
int pcgrl_store_rate(uint8_t* dst, int64_t n_regions, int32_t region_bytes, int32_t store_mode,
                     int32_t order, void* stream);

/* Checks on the GPU that the cross-lane row exchange used by the flood kernels moves data the way
 * the kernels assume (each of the 3 lane groupings, both directions).  Synchronises.
 * mismatches: host pointer, receives the number of lanes that disagreed (0 = good). */
int pcgrl_selftest(int device, int32_t* mismatches);

const char* pcgrl_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
