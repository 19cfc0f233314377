/*
 * pgxhex.h -- C ABI of the batched Hex environment for AMD MI355X (gfx950); part of libpgxgo.so.
 *
 * The library implements the environment API of the Pgx paper (arXiv 2303.17503, Fig. 2: init / step /
 * observation / legal_action_mask / rewards / terminated / current_player) for Hex on the 11x11 board
 * (Table 1; Appendix C, "Hex").  Every rule step runs in HIP kernels on the device; this header is the only
 * boundary.  No type of any other library appears in a signature.
 *
 * Conventions
 *   - Pointers named *_dev are DEVICE pointers owned by the caller; the library never frees them.
 *   - All work is enqueued on the HIP stream given in pgxhex_opts.stream (NULL = the default stream) and is
 *     asynchronous with respect to the host.  Only pgxhex_init (once) and pgxhex_sync synchronise.
 *   - Every function returns PGXHEX_OK (0) or a negative error code; nothing throws or aborts.  An action that
 *     is illegal *in the game* is not an API error: it ends that game, the offender gets -1, the opponent +1.
 *   - Cell index p = row * 11 + col.  Action p places a stone on p; action 121 is the swap, on offer on the
 *     second turn only (Appendix C "Hex", Action); action -1 leaves that environment untouched (an extension).
 *   - Rules (Appendix C "Hex"): the players place stones in turn; a player who joins their two sides wins; there
 *     is no draw.  Where the paper is silent: Black moves first and joins row 0 with row 10, White joins column 0
 *     with column 10; cell (r,c) touches (r,c-1) (r,c+1) (r-1,c) (r-1,c+1) (r+1,c) (r+1,c-1); the swap takes
 *     Black's lone stone at (r,c) off and puts a white stone on (c,r), and Black moves next.
 *   - Layouts are tight: legal mask uint8 [batch][122], observation uint8 [batch][11][11][4] with planes
 *     (mover's stones, opponent's stones, all ones when Black is to move, all ones when the swap is legal).
 *     Base pointers need no particular alignment.
 */
#ifndef PGXHEX_H_
#define PGXHEX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PGXHEX_OK 0
#define PGXHEX_EINVAL (-1) /* null pointer, batch <= 0, buffer too small or misaligned */
#define PGXHEX_EHIP (-2)   /* a HIP runtime call failed; see pgxhex_last_hip_error() */
#define PGXHEX_ENOMEM (-3) /* host allocation of the handle failed */

#define PGXHEX_N 11
#define PGXHEX_ACTIONS 122   /* Table 1 */
#define PGXHEX_OBS_BYTES 484 /* 11 * 11 * 4, Table 1 */

typedef struct pgxhex_ctx* pgxhex_t; /* opaque host-side handle */

typedef struct {
  int32_t auto_reset; /* 1: a finished game is re-initialised within the same step call (Sec. 4.1) */
  void* stream;       /* hipStream_t of the caller; NULL = default stream */
} pgxhex_opts;

/* Bytes of device memory pgxhex_init needs for `batch` games; 0 if batch <= 0.  The caller allocates that many
 * bytes, 256-byte aligned. */
size_t pgxhex_state_bytes(int32_t batch);

/* Fig. 2 "init": creates `batch` games on the empty board, Black to move, and draws for each game which player
 * id (0/1) holds Black from bit 0 of hash(seed, 1, env, episode) (Fig. 2: current_player is independent of the
 * colour).  state_dev: caller-owned device buffer of at least pgxhex_state_bytes() bytes that must outlive the
 * handle; opts may be NULL (no auto-reset, default stream).  Synchronises the stream once. */
int pgxhex_init(pgxhex_t* out, int32_t batch, uint32_t seed, const pgxhex_opts* opts, void* state_dev, size_t state_bytes);

/* Frees the host handle; device memory stays with the caller. */
int pgxhex_destroy(pgxhex_t h);

/* Starts a new episode in every game (episode counters advance, seats are redrawn) and rewrites bound outputs. */
int pgxhex_reset(pgxhex_t h);

/* Buffers the step calls write to; any may be NULL (that output is then not produced; rewards and terminated
 * fall back to buffers inside the state).  Bound mask / observation buffers are filled for the current state. */
int pgxhex_bind_outputs(pgxhex_t h, uint8_t* mask_dev /* [batch][122] */, uint8_t* obs_dev /* [batch][484] */,
                        float* rewards_dev /* [batch][2] by player id */, uint8_t* terminated_dev /* [batch] */);

/* Switches the buffers the step calls write to WITHOUT touching their contents (no emission, no copy): for callers
 * that record a trajectory by stepping into a different slice every ply.  NULL handling as in pgxhex_bind_outputs.
 * What the new buffers hold for a game is undefined until a step call has written it (action -1 writes nothing). */
int pgxhex_set_output_buffers(pgxhex_t h, uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev);

/* Fig. 2 "step": applies actions_dev[batch] (int32) to every game: legality gate, placement or swap, winner test
 * (Appendix C "Hex", Rules), rewards +1/-1 (Reward), auto-reset, next legal mask and observation. */
int pgxhex_step(pgxhex_t h, const int32_t* actions_dev);

/* Uniform random legal action per game (Sec. 4.1 random policy): the k-th legal action in ascending order,
 * k = hash(seed, 0, env, t) mod legal_count; 0 if nothing is legal (a finished game on a full board); -1 for
 * games with t < start_t_dev[env] (start_t_dev may be NULL). */
int pgxhex_random_actions(pgxhex_t h, uint32_t seed, uint32_t t, const int32_t* start_t_dev, int32_t* actions_dev);

/* pgxhex_step followed by pgxhex_random_actions(seed, t, ...) on the new state, in one launch.
 * next_actions_dev must not alias actions_dev. */
int pgxhex_step_sample(pgxhex_t h, const int32_t* actions_dev, uint32_t seed, uint32_t t, const int32_t* start_t_dev,
                       int32_t* next_actions_dev);

/* `steps` plies of uniform random legal play in ONE kernel launch (Sec. 2: all-on-device loops; Sec. 4.1: random
 * policy with auto-reset).  Exactly equivalent to
 *   for i in 0..steps-1: pgxhex_random_actions(seed, t0+i, start_t_dev, a); pgxhex_step(a)
 * but the game state stays in registers between plies.  The outputs of ply i go to slice (i mod slices) of the
 * caller's trajectory buffers, each of which may be NULL: actions_dev [slices][batch] int32, rewards_dev
 * [slices][batch][2] float32, terminated_dev [slices][batch] uint8, mask_dev [slices][batch][122],
 * obs_dev [slices][batch][484] (mask and observation are those AFTER the ply; an environment that still waits for
 * its start time reports action -1, zero rewards and terminated 0).  Buffers bound with pgxhex_bind_outputs are
 * not touched. */
int pgxhex_rollout(pgxhex_t h, int32_t steps, int32_t slices, uint32_t seed, uint32_t t0, const int32_t* start_t_dev,
                   int32_t* actions_dev, float* rewards_dev, uint8_t* terminated_dev, uint8_t* mask_dev, uint8_t* obs_dev);

/* Getters for the current state; each enqueues one kernel or copy into the caller's buffer. */
int pgxhex_legal_mask(pgxhex_t h, uint8_t* dst_dev /* [batch][122] */);
int pgxhex_observe(pgxhex_t h, uint8_t* dst_dev /* [batch][484] */);
int pgxhex_rewards(pgxhex_t h, float* dst_dev /* [batch][2], values of the last step call */);
int pgxhex_terminated(pgxhex_t h, uint8_t* dst_dev /* [batch], values of the last step call */);
int pgxhex_current_player(pgxhex_t h, uint8_t* dst_dev /* [batch] player id to move */);

/* Canonical state for tests, checkpoints and search; any pointer may be NULL on export.
 *   board [batch][121] int8 (0 empty, +1 black, -1 white); to_play int8 (+1 / -1); steps int32; terminated uint8;
 *   black_player uint8; episode uint32; illegal uint32 (count of illegal actions received). */
int pgxhex_export_state(pgxhex_t h, int8_t* board_dev, int8_t* to_play_dev, int32_t* steps_dev, uint8_t* terminated_dev,
                        uint8_t* black_player_dev, uint32_t* episode_dev, uint32_t* illegal_dev);
/* All pointers required.  Rewards are cleared, terminated is taken from the argument, the illegal-action
 * counters are kept, bound outputs are rewritten. */
int pgxhex_import_state(pgxhex_t h, const int8_t* board_dev, const int8_t* to_play_dev, const int32_t* steps_dev,
                        const uint8_t* terminated_dev, const uint8_t* black_player_dev, const uint32_t* episode_dev);

/* Launch-shape knob of pgxhex_step / pgxhex_step_sample / pgxhex_rollout: 1 = a board row per lane (5 boards per wavefront), 2 = a whole
 * board per lane (64 boards per wavefront; pays from about 28 k games on, in the rollout kernel from about 20 k), 0 = the
 * automatic choice by batch size.  Results do not depend on it.  Returns the mapping the step calls now use (1 or 2), or
 * a negative error code. */
int pgxhex_set_mapping(pgxhex_t h, int32_t mapping);

/* Waits for the handle's stream. */
int pgxhex_sync(pgxhex_t h);

/* Boards one 64-lane wavefront holds (5). */
int32_t pgxhex_boards_per_wavefront(void);

const char* pgxhex_strerror(int code);
int pgxhex_last_hip_error(void); /* hipError_t of the last failed runtime call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* PGXHEX_H_ */
