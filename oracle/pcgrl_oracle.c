/*
 * pcgrl_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT (see pcgrl_oracle.h).
 *
 * Plain CPU implementation of the PCGRL environment step, one cell at a time.
 * Passages followed (paper sections):
 *   Methods / Training            narrow representation: the agent may change the tile it
 *                                 stands on, is then moved on in a scan of the map, and sees
 *                                 an egocentric, padded patch; reward = drop of the loss
 *                                 between the level's metrics and their targets.
 *   Methods / Task                map initialisation (weighted draw or empty); metrics are
 *                                 recomputed only when the edit modified the map.
 *   Task / Binary domain + fn.    diameter by two shortest-path sweeps; regions by flood fill.
 *   Task / Maze domain            player -> door path, one connected region.
 *   Task / Dungeon domain         player -> key -> door path, nearest enemy, tile counts.
 *   Task / Pinpoint tiles         frozen cells that edits cannot change.
 *   Task / Randomized map shapes  per-episode rectangle inside a fixed buffer.
 *   Discussion                    border tiles around the active map in the observation.
 *
 * Where the paper is silent the reading taken is stated at the function.
 */
#include "pcgrl_oracle.h"

#include <stdlib.h>
#include <string.h>

#define TILE_EMPTY 0
#define TILE_WALL 1
#define MAZE_PLAYER 2
#define MAZE_DOOR 3
#define DUN_PLAYER 2
#define DUN_KEY 3
#define DUN_DOOR 4
#define DUN_ENEMY 5
#define DUN_CHEST 6

#define MAXC (64 * 64)

typedef struct {
  int8_t* tiles;   /* [max_h][max_w], -1 outside the active map */
  uint8_t* frozen; /* [max_h][max_w] */
  int h, w;
  int py, px;
  int t, n_changes, episode;
  int32_t m[ORC_MAX_METRICS];
  int32_t tgt[ORC_MAX_METRICS][2];
} orc_env;

struct orc_ctx {
  orc_config cfg;
  uint64_t seed;
  int K, M, C;
  orc_env* env;
};

/* ------------------------------------------------------------------ sizes */

int orc_num_tiles(int problem) {
  if (problem == ORC_BINARY) return 2;
  if (problem == ORC_MAZE) return 4;
  if (problem == ORC_DUNGEON) return 7;
  return 0;
}

/* metric vector: [regions, path, (nearest enemy: dungeon only), count of tile 0..K-1] */
int orc_num_metrics(int problem) {
  int k = orc_num_tiles(problem);
  if (k == 0) return 0;
  return (problem == ORC_DUNGEON ? 3 : 2) + k;
}

int orc_num_channels(const orc_config* cfg) {
  return orc_num_tiles(cfg->problem) + (cfg->pad_mode == ORC_PAD_BORDER ? 1 : 0) +
         (cfg->obs_frozen_channel ? 1 : 0);
}

/* --------------------------------------------------- counter-based numbers */

/* The output mixing function of the published splitmix64 generator. */
uint64_t orc_mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

#define GOLDEN 0x9E3779B97F4A7C15ull
#define EPISODE_MUL 0xD1B54A32D192ED03ull

/* One key per (seed, global env index, episode): results do not depend on how a
 * batch is partitioned. */
uint64_t orc_env_key(uint64_t seed, uint64_t env, uint64_t episode) {
  uint64_t k0 = orc_mix64(seed + GOLDEN * (env + 1));
  return orc_mix64(k0 ^ (EPISODE_MUL * (episode + 1)));
}

/* stream 0: shape (counter 0 = height, 1 = width); 1: tiles (counter = y*max_w+x);
 * 2: pinpoint positions (counter = attempt); 3: agent position (counter = t);
 * 4: control targets (counter = metric index). */
uint64_t orc_draw(uint64_t key, uint32_t stream, uint32_t counter) {
  uint64_t c = ((uint64_t)stream << 32) + (uint64_t)counter + 1;
  return orc_mix64(key + GOLDEN * c);
}

static uint32_t hi32(uint64_t u) { return (uint32_t)(u >> 32); }
static uint32_t lo32(uint64_t u) { return (uint32_t)u; }
/* uniform integer in [0, n) from 32 random bits: multiply and keep the high word */
static int below(uint32_t r, int n) { return (int)(((uint64_t)r * (uint64_t)n) >> 32); }
int orc_below(uint32_t r, int n) { return below(r, n); }

/* ------------------------------------------------------ graph primitives */

/* Reading: every real tile except wall can be walked on and belongs to a region;
 * cells outside the active map (-1) cannot. */
static int passable(int8_t t) { return t >= 0 && t != TILE_WALL; }

static const int DY[4] = {-1, 0, 0, 1};
static const int DX[4] = {0, -1, 1, 0};

/* Number of 4-connected components of passable cells (flood fill, Binary domain). */
int orc_regions(const int8_t* tiles, int h, int w, int pitch) {
  static __thread uint8_t seen[MAXC];
  static __thread int stack[MAXC];
  int count = 0;
  memset(seen, 0, (size_t)(h * w));
  for (int y = 0; y < h; ++y)
    for (int x = 0; x < w; ++x) {
      if (!passable(tiles[y * pitch + x]) || seen[y * w + x]) continue;
      ++count;
      int sp = 0;
      stack[sp++] = y * w + x;
      seen[y * w + x] = 1;
      while (sp > 0) {
        int c = stack[--sp];
        int cy = c / w, cx = c % w;
        for (int d = 0; d < 4; ++d) {
          int ny = cy + DY[d], nx = cx + DX[d];
          if (ny < 0 || ny >= h || nx < 0 || nx >= w) continue;
          if (!passable(tiles[ny * pitch + nx]) || seen[ny * w + nx]) continue;
          seen[ny * w + nx] = 1;
          stack[sp++] = ny * w + nx;
        }
      }
    }
  return count;
}

/* Breadth-first search on the unit-weight grid graph (what the paper calls Dijkstra's
 * algorithm on a tile map).  Distances are numbers of edges; a source has distance 0. */
static void bfs_from_marks(const int8_t* tiles, int h, int w, int pitch, const uint8_t* is_src,
                           int32_t* dist) {
  static __thread int queue[MAXC];
  int head = 0, tail = 0;
  for (int i = 0; i < h * w; ++i) dist[i] = -1;
  for (int y = 0; y < h; ++y)
    for (int x = 0; x < w; ++x)
      if (is_src[y * w + x] && passable(tiles[y * pitch + x])) {
        dist[y * w + x] = 0;
        queue[tail++] = y * w + x;
      }
  while (head < tail) {
    int c = queue[head++];
    int cy = c / w, cx = c % w;
    for (int d = 0; d < 4; ++d) {
      int ny = cy + DY[d], nx = cx + DX[d];
      if (ny < 0 || ny >= h || nx < 0 || nx >= w) continue;
      if (!passable(tiles[ny * pitch + nx]) || dist[ny * w + nx] >= 0) continue;
      dist[ny * w + nx] = dist[c] + 1;
      queue[tail++] = ny * w + nx;
    }
  }
}

void orc_bfs(const int8_t* tiles, int h, int w, int pitch, int src_tile, int src_index,
             int32_t* dist) {
  static __thread uint8_t src[MAXC];
  for (int y = 0; y < h; ++y)
    for (int x = 0; x < w; ++x)
      src[y * w + x] = src_tile >= 0 ? (tiles[y * pitch + x] == src_tile) : (y * w + x == src_index);
  bfs_from_marks(tiles, h, w, pitch, src, dist);
}

/* Binary domain, footnote: sweep from a tile x, take the far end y of the longest shortest
 * path from x, sweep again from y; the longest distance from y is the estimate.
 * Readings: x is the first passable cell in row-major order (one admissible draw of the
 * paper's random tile, made deterministic); among several cells at the largest distance from
 * x, y is the one with the lowest row-major index; no passable cell gives 0. */
int orc_diameter_two_pass(const int8_t* tiles, int h, int w, int pitch) {
  static __thread int32_t dist[MAXC];
  int x0 = -1;
  for (int i = 0; i < h * w && x0 < 0; ++i)
    if (passable(tiles[(i / w) * pitch + (i % w)])) x0 = i;
  if (x0 < 0) return 0;
  orc_bfs(tiles, h, w, pitch, -1, x0, dist);
  int far = 0, y0 = x0;
  for (int i = 0; i < h * w; ++i)
    if (dist[i] > far) {
      far = dist[i];
      y0 = i;
    }
  orc_bfs(tiles, h, w, pitch, -1, y0, dist);
  far = 0;
  for (int i = 0; i < h * w; ++i)
    if (dist[i] > far) far = dist[i];
  return far;
}

/* Task / Binary domain: the graph diameter of the walkable cells (the quantity the two-sweep
 * estimate stands for), computed exactly: one breadth-first search from every walkable cell,
 * the largest distance found. */
int orc_exact_diameter(const int8_t* tiles, int h, int w, int pitch) {
  static __thread int32_t dist[MAXC];
  int best = 0;
  for (int s = 0; s < h * w; ++s) {
    if (!passable(tiles[(s / w) * pitch + (s % w)])) continue;
    orc_bfs(tiles, h, w, pitch, -1, s, dist);
    for (int i = 0; i < h * w; ++i)
      if (dist[i] > best) best = dist[i];
  }
  return best;
}

/* Shortest distance from any cell of tile src_tile to any cell of tile dst_tile.
 * Reading: with several sources or destinations the nearest pair counts (this is the paper's
 * single player / single door quantity when there is one of each); no source, no destination
 * or no connection gives 0. */
int orc_path_nearest(const int8_t* tiles, int h, int w, int pitch, int src_tile, int dst_tile) {
  static __thread int32_t dist[MAXC];
  orc_bfs(tiles, h, w, pitch, src_tile, -1, dist);
  int best = -1;
  for (int y = 0; y < h; ++y)
    for (int x = 0; x < w; ++x)
      if (tiles[y * pitch + x] == dst_tile && dist[y * w + x] >= 0)
        if (best < 0 || dist[y * w + x] < best) best = dist[y * w + x];
  return best < 0 ? 0 : best;
}

/* Dungeon domain: shortest player -> key -> door path.
 * Reading for several instances: leg 1 is the distance d1 from the players to the nearest
 * key; leg 2 starts from every key at exactly that distance and ends at the nearest door;
 * the result is d1 + d2, or 0 when either leg does not exist. */
int orc_path_dungeon(const int8_t* tiles, int h, int w, int pitch) {
  static __thread int32_t dist[MAXC];
  static __thread uint8_t src[MAXC];
  orc_bfs(tiles, h, w, pitch, DUN_PLAYER, -1, dist);
  int d1 = -1;
  for (int y = 0; y < h; ++y)
    for (int x = 0; x < w; ++x)
      if (tiles[y * pitch + x] == DUN_KEY && dist[y * w + x] >= 0)
        if (d1 < 0 || dist[y * w + x] < d1) d1 = dist[y * w + x];
  if (d1 < 0) return 0;
  for (int y = 0; y < h; ++y)
    for (int x = 0; x < w; ++x)
      src[y * w + x] = (tiles[y * pitch + x] == DUN_KEY && dist[y * w + x] == d1);
  bfs_from_marks(tiles, h, w, pitch, src, dist);
  int d2 = -1;
  for (int y = 0; y < h; ++y)
    for (int x = 0; x < w; ++x)
      if (tiles[y * pitch + x] == DUN_DOOR && dist[y * w + x] >= 0)
        if (d2 < 0 || dist[y * w + x] < d2) d2 = dist[y * w + x];
  if (d2 < 0) return 0;
  return d1 + d2;
}

void orc_level_metrics(int problem, const int8_t* tiles, int h, int w, int pitch, int32_t* m) {
  int K = orc_num_tiles(problem);
  int base = problem == ORC_DUNGEON ? 3 : 2;
  m[0] = orc_regions(tiles, h, w, pitch);
  if (problem == ORC_BINARY) {
    m[1] = orc_diameter_two_pass(tiles, h, w, pitch);
  } else if (problem == ORC_MAZE) {
    m[1] = orc_path_nearest(tiles, h, w, pitch, MAZE_PLAYER, MAZE_DOOR);
  } else {
    m[1] = orc_path_dungeon(tiles, h, w, pitch);
    m[2] = orc_path_nearest(tiles, h, w, pitch, DUN_PLAYER, DUN_ENEMY);
  }
  for (int k = 0; k < K; ++k) m[base + k] = 0;
  for (int y = 0; y < h; ++y)
    for (int x = 0; x < w; ++x) {
      int t = tiles[y * pitch + x];
      if (t >= 0 && t < K) m[base + t] += 1;
    }
}

/* Distance of a metric from its target range [lo, hi]; an exact target has lo == hi, a metric
 * to be maximised has lo == hi == a constant no value can reach. */
int orc_loss(int v, int lo, int hi) {
  int l = 0;
  if (lo - v > l) l = lo - v;
  if (v - hi > l) l = v - hi;
  return l;
}

/* ------------------------------------------------------------ environment */

static int cfg_ok(const orc_config* c) {
  if (orc_num_tiles(c->problem) == 0) return 0;
  if (c->batch < 1) return 0;
  if (c->max_h < 1 || c->max_h > 64 || c->max_w < 1 || c->max_w > 64) return 0;
  if (c->min_h < 1 || c->min_h > c->max_h || c->min_w < 1 || c->min_w > c->max_w) return 0;
  if (c->obs_w < 1 || c->obs_w > 127) return 0;
  if (c->pad_mode != ORC_PAD_BORDER && c->pad_mode != ORC_PAD_WALL) return 0;
  if (c->pos_mode != ORC_POS_SCAN && c->pos_mode != ORC_POS_RANDOM) return 0;
  if (c->n_frozen < 0 || c->n_frozen > 8 || c->n_frozen > c->min_h * c->min_w) return 0;
  if (c->max_steps < 1 || c->max_changes < 0) return 0;
  for (int j = 0; j < 8; ++j)
    if (c->pinpoint_tile[j] < -1 || c->pinpoint_tile[j] >= orc_num_tiles(c->problem)) return 0;
  for (int i = 0; i < orc_num_metrics(c->problem); ++i)
    if (((c->ctrl_mask >> i) & 1u) && (c->ctrl_lo[i] < 0 || c->ctrl_hi[i] < c->ctrl_lo[i] || c->ctrl_hi[i] > 65535)) return 0;
  return 1;
}

orc_ctx* orc_create(const orc_config* cfg) {
  if (!cfg || !cfg_ok(cfg)) return NULL;
  orc_ctx* ctx = (orc_ctx*)calloc(1, sizeof(orc_ctx));
  ctx->cfg = *cfg;
  ctx->K = orc_num_tiles(cfg->problem);
  ctx->M = orc_num_metrics(cfg->problem);
  ctx->C = orc_num_channels(cfg);
  ctx->env = (orc_env*)calloc((size_t)cfg->batch, sizeof(orc_env));
  size_t cells = (size_t)cfg->max_h * (size_t)cfg->max_w;
  for (int b = 0; b < cfg->batch; ++b) {
    orc_env* e = &ctx->env[b];
    e->tiles = (int8_t*)malloc(cells);
    e->frozen = (uint8_t*)calloc(cells, 1);
    memset(e->tiles, -1, cells);
    e->h = cfg->max_h;
    e->w = cfg->max_w;
    for (int i = 0; i < ctx->M; ++i) {
      e->tgt[i][0] = cfg->target_lo[i];
      e->tgt[i][1] = cfg->target_hi[i];
    }
  }
  return ctx;
}

void orc_destroy(orc_ctx* ctx) {
  if (!ctx) return;
  for (int b = 0; b < ctx->cfg.batch; ++b) {
    free(ctx->env[b].tiles);
    free(ctx->env[b].frozen);
  }
  free(ctx->env);
  free(ctx);
}

static void env_metrics(const orc_ctx* ctx, orc_env* e) {
  orc_level_metrics(ctx->cfg.problem, e->tiles, e->h, e->w, ctx->cfg.max_w, e->m);
}

/* Start of an episode (Task: initialisation, pinpoints, randomized shapes).
 * Readings: the active map is anchored at the top-left corner of the buffer; pinpoint cells
 * are distinct cells of the active map that keep their initial tile; a scan starts at (0,0). */
static void env_begin_episode(const orc_ctx* ctx, int b, int episode) {
  const orc_config* c = &ctx->cfg;
  orc_env* e = &ctx->env[b];
  uint64_t key = orc_env_key(ctx->seed, (uint64_t)b, (uint64_t)episode);
  size_t cells = (size_t)c->max_h * (size_t)c->max_w;
  e->episode = episode;
  e->h = c->max_h;
  e->w = c->max_w;
  if (c->min_h < c->max_h) e->h = c->min_h + below(hi32(orc_draw(key, 0, 0)), c->max_h - c->min_h + 1);
  if (c->min_w < c->max_w) e->w = c->min_w + below(hi32(orc_draw(key, 0, 1)), c->max_w - c->min_w + 1);

  int empty_start = 1;
  for (int k = 0; k < ORC_MAX_TILES; ++k)
    if (c->init_cdf[k] != 0) empty_start = 0;
  memset(e->tiles, -1, cells);
  memset(e->frozen, 0, cells);
  for (int y = 0; y < e->h; ++y)
    for (int x = 0; x < e->w; ++x) {
      int tile = 0;
      if (!empty_start) {
        uint32_t r = hi32(orc_draw(key, 1, (uint32_t)(y * c->max_w + x)));
        tile = ctx->K - 1;
        for (int k = 0; k < ctx->K - 1; ++k)
          if (r < c->init_cdf[k]) {
            tile = k;
            break;
          }
      }
      e->tiles[y * c->max_w + x] = (int8_t)tile;
    }

  int placed = 0;
  for (uint32_t a = 0; a < 64 && placed < c->n_frozen; ++a) {
    uint64_t u = orc_draw(key, 2, a);
    int y = below(hi32(u), e->h), x = below(lo32(u), e->w);
    if (!e->frozen[y * c->max_w + x]) {
      /* Task / Pinpoint tiles: a pivotal tile (player, door, ...) frozen at an arbitrary cell */
      e->frozen[y * c->max_w + x] = 1;
      if (c->pinpoint_tile[placed] >= 0) e->tiles[y * c->max_w + x] = (int8_t)c->pinpoint_tile[placed];
      ++placed;
    }
  }
  /* Methods / Training: the target of a controlled metric varies from episode to episode */
  for (int i = 0; i < ctx->M; ++i)
    if ((c->ctrl_mask >> i) & 1u) {
      int v = c->ctrl_lo[i] + below(hi32(orc_draw(key, 4, (uint32_t)i)), c->ctrl_hi[i] - c->ctrl_lo[i] + 1);
      e->tgt[i][0] = v;
      e->tgt[i][1] = v;
    }

  e->t = 0;
  e->n_changes = 0;
  e->py = 0;
  e->px = 0;
  if (c->pos_mode == ORC_POS_RANDOM) {
    uint64_t u = orc_draw(key, 3, 0);
    e->py = below(hi32(u), e->h);
    e->px = below(lo32(u), e->w);
  }
  env_metrics(ctx, e);
}

/* Egocentric observation (Methods / Training; Discussion): window of obs_w x obs_w cells whose
 * cell (r, r), r = obs_w / 2 rounded down, is the agent's cell; one channel per tile type;
 * cells outside the active map show the border channel (or wall under ORC_PAD_WALL). */
static void env_observe(const orc_ctx* ctx, const orc_env* e, uint8_t* obs) {
  const orc_config* c = &ctx->cfg;
  int ow = c->obs_w, r = ow / 2;
  int pad = c->pad_mode == ORC_PAD_BORDER ? ctx->K : TILE_WALL;
  memset(obs, 0, (size_t)ctx->C * (size_t)ow * (size_t)ow);
  for (int i = 0; i < ow; ++i)
    for (int j = 0; j < ow; ++j) {
      int p = e->py - r + i, q = e->px - r + j;
      int ch = pad;
      int in = p >= 0 && p < e->h && q >= 0 && q < e->w;
      if (in) ch = e->tiles[p * c->max_w + q];
      obs[((size_t)ch * ow + i) * ow + j] = 1;
      /* optional last channel: which cells in view the agent cannot change (pinpoints) */
      if (c->obs_frozen_channel && in && e->frozen[p * c->max_w + q])
        obs[((size_t)(ctx->C - 1) * ow + i) * ow + j] = 1;
    }
}

void orc_reset(orc_ctx* ctx, uint64_t seed, uint8_t* obs) {
  size_t osz = (size_t)ctx->C * ctx->cfg.obs_w * ctx->cfg.obs_w;
  ctx->seed = seed;
  for (int b = 0; b < ctx->cfg.batch; ++b) {
    orc_env* e = &ctx->env[b];
    for (int i = 0; i < ctx->M; ++i) {
      e->tgt[i][0] = ctx->cfg.target_lo[i];
      e->tgt[i][1] = ctx->cfg.target_hi[i];
    }
    env_begin_episode(ctx, b, 0);
    if (obs) env_observe(ctx, e, obs + (size_t)b * osz);
  }
}

/* One step of one environment. */
static void env_step(orc_ctx* ctx, int b, int action, uint8_t* obs, float* reward, uint8_t* done) {
  const orc_config* c = &ctx->cfg;
  orc_env* e = &ctx->env[b];
  int cell = e->py * c->max_w + e->px;
  int old = e->tiles[cell];
  int changed = action >= 0 && action < ctx->K && !e->frozen[cell] && action != old;
  float r = 0.0f;
  if (changed) {
    int32_t old_m[ORC_MAX_METRICS];
    memcpy(old_m, e->m, sizeof(old_m));
    e->tiles[cell] = (int8_t)action;
    e->n_changes += 1;
    env_metrics(ctx, e);
    /* reward = sum over metrics, in index order, of weight * (old loss - new loss); the
     * difference is formed in integers, then one float32 multiply and one float32 add */
    for (int i = 0; i < ctx->M; ++i) {
      int dl = orc_loss(old_m[i], e->tgt[i][0], e->tgt[i][1]) - orc_loss(e->m[i], e->tgt[i][0], e->tgt[i][1]);
      float term = c->weights[i] * (float)dl;
      r = r + term;
    }
  }
  e->t += 1;
  int d = (e->t >= c->max_steps) || (c->max_changes > 0 && e->n_changes >= c->max_changes);
  if (d && c->autoreset) {
    /* reward and done describe the transition that just ended; the observation and the cached
     * metrics describe the first state of the next episode */
    env_begin_episode(ctx, b, e->episode + 1);
  } else if (c->pos_mode == ORC_POS_SCAN) {
    e->px += 1;
    if (e->px >= e->w) {
      e->px = 0;
      e->py += 1;
      if (e->py >= e->h) e->py = 0;
    }
  } else {
    uint64_t key = orc_env_key(ctx->seed, (uint64_t)b, (uint64_t)e->episode);
    uint64_t u = orc_draw(key, 3, (uint32_t)e->t);
    e->py = below(hi32(u), e->h);
    e->px = below(lo32(u), e->w);
  }
  if (reward) *reward = r;
  if (done) *done = (uint8_t)d;
  if (obs) env_observe(ctx, e, obs);
}

void orc_step_range(orc_ctx* ctx, int env_lo, int env_hi, const int32_t* actions, uint8_t* obs,
                    float* reward, uint8_t* done) {
  size_t osz = (size_t)ctx->C * ctx->cfg.obs_w * ctx->cfg.obs_w;
  for (int b = env_lo; b < env_hi; ++b)
    env_step(ctx, b, actions[b], obs ? obs + (size_t)b * osz : NULL, reward ? reward + b : NULL,
             done ? done + b : NULL);
}

void orc_step(orc_ctx* ctx, const int32_t* actions, uint8_t* obs, float* reward, uint8_t* done) {
  orc_step_range(ctx, 0, ctx->cfg.batch, actions, obs, reward, done);
}

void orc_metrics(const orc_ctx* ctx, int32_t* out) {
  for (int b = 0; b < ctx->cfg.batch; ++b)
    for (int i = 0; i < ctx->M; ++i) out[(size_t)b * ctx->M + i] = ctx->env[b].m[i];
}

void orc_exact_diameters(const orc_ctx* ctx, int32_t* out) {
  for (int b = 0; b < ctx->cfg.batch; ++b)
    out[b] = orc_exact_diameter(ctx->env[b].tiles, ctx->env[b].h, ctx->env[b].w, ctx->cfg.max_w);
}

void orc_observe(const orc_ctx* ctx, uint8_t* obs) {
  size_t osz = (size_t)ctx->C * ctx->cfg.obs_w * ctx->cfg.obs_w;
  for (int b = 0; b < ctx->cfg.batch; ++b) env_observe(ctx, &ctx->env[b], obs + (size_t)b * osz);
}

void orc_get_state(const orc_ctx* ctx, int8_t* tiles, uint8_t* frozen, int16_t* hw, int16_t* pos,
                   int32_t* counters) {
  size_t cells = (size_t)ctx->cfg.max_h * (size_t)ctx->cfg.max_w;
  for (int b = 0; b < ctx->cfg.batch; ++b) {
    const orc_env* e = &ctx->env[b];
    if (tiles) memcpy(tiles + b * cells, e->tiles, cells);
    if (frozen) memcpy(frozen + b * cells, e->frozen, cells);
    if (hw) {
      hw[2 * b] = (int16_t)e->h;
      hw[2 * b + 1] = (int16_t)e->w;
    }
    if (pos) {
      pos[2 * b] = (int16_t)e->py;
      pos[2 * b + 1] = (int16_t)e->px;
    }
    if (counters) {
      counters[3 * b] = e->t;
      counters[3 * b + 1] = e->n_changes;
      counters[3 * b + 2] = e->episode;
    }
  }
}

void orc_set_state(orc_ctx* ctx, const int8_t* tiles, const uint8_t* frozen, const int16_t* hw,
                   const int16_t* pos) {
  const orc_config* c = &ctx->cfg;
  size_t cells = (size_t)c->max_h * (size_t)c->max_w;
  for (int b = 0; b < c->batch; ++b) {
    orc_env* e = &ctx->env[b];
    e->h = hw[2 * b];
    e->w = hw[2 * b + 1];
    e->py = pos[2 * b];
    e->px = pos[2 * b + 1];
    for (int y = 0; y < c->max_h; ++y)
      for (int x = 0; x < c->max_w; ++x) {
        int in = y < e->h && x < e->w;
        size_t i = (size_t)y * c->max_w + x;
        e->tiles[i] = in ? tiles[b * cells + i] : (int8_t)-1;
        e->frozen[i] = (in && frozen) ? (frozen[b * cells + i] != 0) : 0;
      }
    e->t = 0;
    e->n_changes = 0;
    env_metrics(ctx, e);
  }
}

void orc_get_targets(const orc_ctx* ctx, int32_t* targets) {
  for (int b = 0; b < ctx->cfg.batch; ++b)
    for (int i = 0; i < ctx->M; ++i) {
      targets[((size_t)b * ctx->M + i) * 2] = ctx->env[b].tgt[i][0];
      targets[((size_t)b * ctx->M + i) * 2 + 1] = ctx->env[b].tgt[i][1];
    }
}

void orc_set_targets(orc_ctx* ctx, const int32_t* targets) {
  for (int b = 0; b < ctx->cfg.batch; ++b)
    for (int i = 0; i < ctx->M; ++i) {
      ctx->env[b].tgt[i][0] = targets[((size_t)b * ctx->M + i) * 2];
      ctx->env[b].tgt[i][1] = targets[((size_t)b * ctx->M + i) * 2 + 1];
    }
}
