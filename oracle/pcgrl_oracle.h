/*
 * pcgrl_oracle.h -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded CPU implementation of the batched PCGRL
 * environment step (narrow representation; binary / maze / dungeon problems;
 * frozen pinpoint tiles; randomized map shapes; egocentric padded one-hot
 * observation).  It exists only so that tests, the smoke check and the
 * benchmark's CPU-baseline leg have something obviously correct to compare the
 * GPU library with.  It shares no code, header, table or helper with the GPU
 * library and must never be reached from the product path.
 *
 * Everything is written cell by cell on an int8 grid: FIFO-queue breadth-first
 * search, explicit-stack flood fill, no bitboards, no SIMD.
 *
 * Parity status of the building blocks (what pins them is in tests/):
 *   regions, BFS distances, two-pass diameter, maze / dungeon path lengths,
 *   nearest enemy, tile counts, reward, observation, scan order, frozen
 *   tiles                      -> pinned (brute force, closed forms, invariants)
 *   mix64, draw, env_key       -> pinned (published splitmix64 output sequence:
 *                                 draw(key, 0, i) is output i+1 of that generator
 *                                 seeded with key, a stream shifts the seed, and
 *                                 the inner hash of env_key is output env+1 of
 *                                 the generator seeded with the seed)
 *   below, and which stream / counter / half-word each draw of an episode
 *   uses                       -> pinned (hand-computed cases; the episode's
 *                                 shape, tiles, pinpoints, positions and control
 *                                 targets rebuilt in the tests from draw alone)
 *   the episode multiplier of env_key, the default weights and target table,
 *   the chest tile of the 7-tile dungeon -> parity unpinned (this build's own
 *   choices: no external fixed point exists; the paper leaves them to code
 *   bases that are not reproduced here)
 */
#ifndef PCGRL_ORACLE_H
#define PCGRL_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* problems (Methods / Task: binary, maze, dungeon paragraphs) */
#define ORC_BINARY 0
#define ORC_MAZE 1
#define ORC_DUNGEON 2
/* what an observation shows outside the active map (Discussion: border tiles) */
#define ORC_PAD_BORDER 0 /* extra channel K marks cells outside the map */
#define ORC_PAD_WALL 1   /* cells outside the map read as wall (channel 1) */
/* how the agent is moved after its edit (Methods / Training) */
#define ORC_POS_SCAN 0   /* row-major scan of the active map, wraps */
#define ORC_POS_RANDOM 1 /* seeded uniform position each step */

#define ORC_MAX_METRICS 16
#define ORC_MAX_TILES 8

typedef struct {
  int32_t problem;
  int32_t batch;
  int32_t max_h, max_w; /* padded buffer, each <= 64 */
  int32_t min_h, min_w; /* == max_* for a fixed shape, else uniform draw per episode */
  int32_t obs_w;        /* observation window side, 1..127 */
  int32_t pad_mode;
  int32_t pos_mode;
  int32_t n_frozen;  /* pinpoint cells per episode, <= 8 */
  int32_t max_steps; /* done when t >= max_steps */
  int32_t max_changes; /* 0 = no change budget */
  int32_t autoreset;
  uint32_t init_cdf[ORC_MAX_TILES]; /* cumulative tile probabilities * 2^32; all 0 = empty start */
  float weights[ORC_MAX_METRICS];
  int32_t target_lo[ORC_MAX_METRICS];
  int32_t target_hi[ORC_MAX_METRICS];
  int32_t pinpoint_tile[8]; /* tile written to the j-th pinpoint cell at episode start; -1 keeps the drawn tile */
  uint32_t ctrl_mask;       /* bit i: metric i's target is drawn anew every episode ... */
  int32_t ctrl_lo[ORC_MAX_METRICS]; /* ... uniformly from [ctrl_lo[i], ctrl_hi[i]] and used as an */
  int32_t ctrl_hi[ORC_MAX_METRICS]; /* exact target (lo = hi = the drawn value) */
  int32_t obs_frozen_channel; /* non-zero: one more (last) channel marks the pinpoint cells in view */
} orc_config;

typedef struct orc_ctx orc_ctx;

/* number of tile types / metrics / observation channels of a configuration */
int orc_num_tiles(int problem);
int orc_num_metrics(int problem);
int orc_num_channels(const orc_config* cfg);

orc_ctx* orc_create(const orc_config* cfg); /* NULL on a bad configuration */
void orc_destroy(orc_ctx* ctx);

/* obs: uint8 [batch][C][obs_w][obs_w] (may be NULL); all buffers are host memory */
void orc_reset(orc_ctx* ctx, uint64_t seed, uint8_t* obs);
/* steps envs [env_lo, env_hi); outputs are indexed by absolute env number */
void orc_step_range(orc_ctx* ctx, int env_lo, int env_hi, const int32_t* actions, uint8_t* obs,
                    float* reward, uint8_t* done);
void orc_step(orc_ctx* ctx, const int32_t* actions, uint8_t* obs, float* reward, uint8_t* done);
void orc_metrics(const orc_ctx* ctx, int32_t* out /* [batch][M] */);
void orc_observe(const orc_ctx* ctx, uint8_t* obs);
void orc_exact_diameters(const orc_ctx* ctx, int32_t* out /* [batch] */);

/* tiles int8 [batch][max_h][max_w] (-1 outside the active map), frozen uint8 same shape,
 * hw int16 [batch][2], pos int16 [batch][2], counters int32 [batch][3] = t, n_changes, episode */
void orc_get_state(const orc_ctx* ctx, int8_t* tiles, uint8_t* frozen, int16_t* hw, int16_t* pos,
                   int32_t* counters);
/* installs a level; frozen may be NULL (nothing frozen); t and n_changes restart at 0;
 * cached metrics are recomputed */
void orc_set_state(orc_ctx* ctx, const int8_t* tiles, const uint8_t* frozen, const int16_t* hw,
                   const int16_t* pos);
void orc_set_targets(orc_ctx* ctx, const int32_t* targets /* [batch][M][2] */);
void orc_get_targets(const orc_ctx* ctx, int32_t* targets /* [batch][M][2] */);

/* ---- building blocks, exported so that tests can pin each one on its own ---- */
uint64_t orc_mix64(uint64_t z);
uint64_t orc_env_key(uint64_t seed, uint64_t env, uint64_t episode);
uint64_t orc_draw(uint64_t key, uint32_t stream, uint32_t counter);
int orc_below(uint32_t r, int n); /* uniform integer in [0, n) from 32 random bits */
/* all on one level: tiles int8 [h][w] with row pitch `pitch` */
int orc_regions(const int8_t* tiles, int h, int w, int pitch);
/* dist int32 [h][w] (pitch w): edges from the nearest cell whose tile == src_tile
 * (src_tile < 0: the single cell src_index = y*w+x), -1 where unreachable */
void orc_bfs(const int8_t* tiles, int h, int w, int pitch, int src_tile, int src_index,
             int32_t* dist);
int orc_diameter_two_pass(const int8_t* tiles, int h, int w, int pitch);
/* exact diameter: the largest shortest-path distance between any two connected walkable cells */
int orc_exact_diameter(const int8_t* tiles, int h, int w, int pitch);
int orc_path_nearest(const int8_t* tiles, int h, int w, int pitch, int src_tile, int dst_tile);
int orc_path_dungeon(const int8_t* tiles, int h, int w, int pitch);
/* full metric vector of one level for a problem */
void orc_level_metrics(int problem, const int8_t* tiles, int h, int w, int pitch, int32_t* m);
int orc_loss(int v, int lo, int hi);

#ifdef __cplusplus
}
#endif
#endif
