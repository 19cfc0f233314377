/*
 * pgxgo.h -- C ABI of the batched Go environment for AMD MI355X (gfx950).
 *
 * The library implements the environment API of the Pgx paper (arXiv 2303.17503,
 * Fig. 2: init / step / observation / legal_action_mask / rewards / terminated /
 * current_player) for the Go 9x9 and Go 19x19 games (Table 1; Appendix C, "Go").
 * Every rule step runs in HIP kernels on the device; this header is the only
 * boundary.  No type of any other library appears in a signature.
 *
 * Conventions
 *   - Pointers named *_dev are DEVICE pointers owned by the caller (for example the
 *     data_ptr() of a torch tensor).  The library never frees them.  Pointers without
 *     that suffix are HOST pointers.
 *   - All work is enqueued on the HIP stream given in pgxgo_opts.stream (NULL = the
 *     default stream) and is asynchronous with respect to the host.  No entry point
 *     synchronises the device except pgxgo_init (once) and pgxgo_sync.
 *   - Every function returns PGXGO_OK (0) or a negative error code; nothing throws or
 *     aborts.  An action that is illegal *in the game* is not an API error: it ends that
 *     game, the offender gets -1 and the opponent +1.
 *   - Point index p = row * N + col (row-major), action p places a stone on p,
 *     action N*N is pass (Appendix C "Go", Action: the last action is pass),
 *     action -1 leaves that environment untouched (an extension used for staggered starts).
 *   - Rules: Tromp-Taylor area scoring, komi added to White (Appendix C "Go").  Where the
 *     paper is silent: simple ko (the ban lasts one ply), suicide is illegal, a game ends
 *     after two consecutive passes or max_steps plies, and is then scored by area.
 */
#ifndef PGXGO_H_
#define PGXGO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PGXGO_OK 0
#define PGXGO_EINVAL (-1) /* null pointer, unsupported board size, batch <= 0, pitch too small, buffer too small */
#define PGXGO_EHIP (-2)   /* a HIP runtime call failed; see pgxgo_last_hip_error() */
#define PGXGO_ENOMEM (-3) /* host allocation of the handle failed */
#define PGXGO_ELIMIT (-4) /* pgxgo_init_static: the games do not fit the library's static state buffer */

#define PGXGO_STATIC_STATE_BYTES (8u << 20) /* size of that buffer, per GPU the library runs on */

typedef struct pgxgo_ctx* pgxgo_t; /* opaque host-side handle */

typedef struct {
  int32_t komi_x2;    /* twice the komi given to White; 15 = 7.5.  (The paper's default 6.5 is 13.) */
  int32_t max_steps;  /* ply cap per game; 0 selects 2*N*N */
  int32_t auto_reset; /* 1: a finished game is re-initialised within the same step call (Sec. 4.1) */
  int32_t obs_pitch;  /* bytes between consecutive environments in observation buffers; 0 = N*N*17 (tight) */
  int32_t mask_pitch; /* bytes between consecutive environments in legal-mask buffers; 0 = N*N+1 (tight) */
  /* Pad bytes between the environments' records are left untouched, with one exception: the line-padded pitches
   * (N*N*17 and N*N+1 rounded up to the next multiple of 128: 6144 / 384 at 19x19, 1408 / 128 at 9x9), where they are
   * written as zeros together with the record.  With both pitches dense or line-padded a wavefront writes its boards
   * as one run of bytes; with line-padded pitches and 128-byte aligned buffers that run consists of whole 128-byte
   * lines only, which is the fastest layout for outputs that have to reach DRAM (every ply into fresh memory). */
  void* stream;       /* hipStream_t of the caller; NULL = default stream */
} pgxgo_opts;

/* Bytes of device memory pgxgo_init needs for `batch` games of size board_size (9 or 19);
 * 0 if the arguments are invalid.  The caller allocates that many bytes, 256-byte aligned. */
size_t pgxgo_state_bytes(int32_t batch, int32_t board_size);

/* Fig. 2 "init": creates `batch` games on the empty board, Black to move, and draws for each
 * game which player id (0/1) holds Black from bit 0 of hash(seed, 1, env, episode)
 * (Fig. 2: current_player is drawn by a PRNG and is independent of the colour).
 * state_dev/state_bytes: caller-owned device buffer of at least pgxgo_state_bytes() bytes that
 * holds all game state until pgxgo_destroy.  opts may be NULL (defaults: komi 7.5, cap 2*N*N,
 * no auto-reset, tight pitches, default stream).  Synchronises once before returning. */
int pgxgo_init(pgxgo_t* out, int32_t batch, int32_t board_size, uint32_t seed, const pgxgo_opts* opts,
               void* state_dev, size_t state_bytes);

/* pgxgo_init for callers that cannot allocate: code under HIP graph capture, serving loops and harnesses in which
 * hipMalloc (or any allocating routine) is forbidden.  Same arguments and result as pgxgo_init, except that the game
 * state lives in a buffer of PGXGO_STATIC_STATE_BYTES that is part of the library image (each GPU the library runs on
 * holds its own copy until the process ends) and the handle is a static object: the call allocates nothing on the
 * host or the device, does not synchronise, and only enqueues the kernel that (re)writes the state of `batch` games
 * on opts->stream.  The device is the current one.  Limits: pgxgo_state_bytes(batch, board_size) must not exceed
 * PGXGO_STATIC_STATE_BYTES (about 7800 games of 19x19 or 23000 of 9x9), else PGXGO_ELIMIT.  There is ONE such state
 * and ONE such handle per GPU: a second call on the same GPU re-initialises them and invalidates the earlier
 * handle's games, and calls that overlap on one GPU (two streams, two threads) race.  Every other entry point works
 * on the handle as on any other; pgxgo_destroy on it frees nothing.  Outputs still go to the caller's buffers. */
int pgxgo_init_static(pgxgo_t* out, int32_t batch, int32_t board_size, uint32_t seed, const pgxgo_opts* opts);

/* Frees the host handle only (device buffers belong to the caller). */
int pgxgo_destroy(pgxgo_t h);

/* Starts a new episode in every environment (episode counters advance, seats are redrawn). */
int pgxgo_reset(pgxgo_t h);

/* Output buffers that pgxgo_step fills directly, so that no copy is needed afterwards.
 *   mask_dev [batch][mask_pitch] uint8 0/1 : legal_action_mask of the player to move (Fig. 2)
 *   obs_dev  [batch][obs_pitch]  uint8 0/1 : observation of the player to move, laid out
 *            [N][N][17]: planes 2i / 2i+1 = mover's / opponent's stones i plies ago (i = 0..7),
 *            plane 16 = 1 when Black is to move (Appendix C "Go", Observation)
 *   rewards_dev [batch][2] float32, indexed by player id: +1 / -1 / 0 (Appendix C "Go", Reward);
 *            non-zero only in the step call that ends a game
 *   terminated_dev [batch] uint8 : 1 if the game ended in this step call (or had ended before,
 *            without auto-reset)
 * Any pointer may be NULL: mask/obs are then not written by step (pgxgo_legal_mask and
 * pgxgo_observe still work), rewards/terminated go to internal arrays read by the getters. */
int pgxgo_bind_outputs(pgxgo_t h, uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev);

/* Switches the buffers pgxgo_step writes to WITHOUT touching their contents (no emission, no copy): for callers
 * that record a trajectory by stepping into a different slice every ply.  Same meanings and NULL handling as
 * pgxgo_bind_outputs.  What the new buffers hold for an environment is undefined until a step call has written it
 * (an environment stepped with action -1 writes nothing). */
int pgxgo_set_output_buffers(pgxgo_t h, uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev);

/* Fig. 2 legal_action_mask and observation of the current state in ONE launch (either pointer may be NULL, not both);
 * the two getters pgxgo_legal_mask / pgxgo_observe below are this call with one buffer. */
int pgxgo_emit(pgxgo_t h, uint8_t* mask_dev /* [batch][mask_pitch] */, uint8_t* obs_dev /* [batch][obs_pitch] */);

/* Fig. 2 "step": applies actions_dev[batch] (int32) to all games: legality gate, stone placement,
 * chain merge, liberty count, capture, ko, history push, termination and area scoring,
 * optional auto-reset, then the next mover's legal mask and observation.  With auto-reset the
 * rewards/terminated of the finishing ply are returned together with the fresh game's mask and
 * observation.  A game that ended earlier (no auto-reset) is frozen and reports zero rewards. */
int pgxgo_step(pgxgo_t h, const int32_t* actions_dev);

/* Uniform random legal actions (Sec. 4.1 random policy): actions_dev[e] = the k-th legal action in
 * ascending index order, k = hash(seed, 0, e, t) mod legal_count, where
 * mix(x): x^=x>>16; x*=0x7feb352d; x^=x>>15; x*=0x846ca68b; x^=x>>16 and
 * hash(s,tag,e,t) = mix(mix(mix(s + 0x9E3779B9*(tag+1)) ^ e) ^ t) in uint32 arithmetic.
 * start_t_dev (nullable, int32[batch]): environments with t < start_t_dev[e] get action -1. */
int pgxgo_random_actions(pgxgo_t h, uint32_t seed, uint32_t t, const int32_t* start_t_dev, int32_t* actions_dev);

/* pgxgo_step followed by pgxgo_random_actions(seed, t, start_t_dev, next_actions_dev) on the new
 * position, in one kernel launch.  next_actions_dev must not alias actions_dev. */
int pgxgo_step_sample(pgxgo_t h, const int32_t* actions_dev, uint32_t seed, uint32_t t, const int32_t* start_t_dev,
                      int32_t* next_actions_dev);

/* `steps` plies of uniform random legal play in ONE kernel launch (Sec. 2: all-on-device loops in the style
 * of the Anakin architecture; Sec. 4.1: random policy with auto-reset).  Exactly equivalent to
 *   for i in 0..steps-1: pgxgo_random_actions(seed, t0+i, start_t_dev, a); pgxgo_step(a)
 * but the game state stays in registers between plies and only outputs go to memory.  The outputs of ply i
 * are written to slice (i mod slices) of the caller's trajectory buffers, each of which may be NULL:
 *   actions_dev [slices][batch] int32 (the drawn action, -1 while an environment waits for its start time),
 *   rewards_dev [slices][batch][2] float32, terminated_dev [slices][batch] uint8,
 *   mask_dev [slices][batch][mask_pitch] uint8, obs_dev [slices][batch][obs_pitch] uint8,
 * with the meanings of pgxgo_bind_outputs (the legal mask and observation are those AFTER the ply).
 * slices = 1 overwrites one set of buffers every ply; slices = steps records the whole trajectory.
 * Buffers bound with pgxgo_bind_outputs are not touched. */
int pgxgo_rollout(pgxgo_t h, int32_t steps, int32_t slices, uint32_t seed, uint32_t t0, const int32_t* start_t_dev,
                  int32_t* actions_dev, float* rewards_dev, uint8_t* terminated_dev, uint8_t* mask_dev, uint8_t* obs_dev);

/* Search-facing step (Sec. 5: tree search calls step from copies of earlier states).  The handle's `batch`
 * environments are treated as a pool of state slots; for i in 0..n-1 (n <= batch):
 *     state[dst_slots_dev[i]] = step(state[src_slots_dev[i]], actions_dev[i])
 * with the semantics of pgxgo_step (action -1 = copy unchanged).  The source slot keeps its state unless it is
 * also the destination of the same entry.  Outputs of entry i go to row i of the optional buffers
 * mask_dev [n][mask_pitch], obs_dev [n][obs_pitch], rewards_dev [n][2], terminated_dev [n]; buffers bound with
 * pgxgo_bind_outputs are not touched.  The environment index used for the seat draw on auto-reset is the
 * destination slot.  The caller guarantees that destination slots are pairwise distinct and that no
 * destination is the source of ANOTHER entry of the same call (the entries run concurrently).  A copied
 * entry (action -1) reports zero rewards and the terminated flag of its state.  An entry with a slot index
 * outside [0, batch) touches no state, reports terminated = 255 and gets zero-filled mask/observation rows. */
int pgxgo_step_slots(pgxgo_t h, int32_t n, const int32_t* src_slots_dev, const int32_t* actions_dev, const int32_t* dst_slots_dev,
                     uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev);

/* state[dst_slots_dev[i]] = state[src_slots_dev[i]] for i in 0..n-1 (same constraints). */
int pgxgo_copy_slots(pgxgo_t h, int32_t n, const int32_t* src_slots_dev, const int32_t* dst_slots_dev);

/* Getters for the current state; each enqueues one kernel or copy into the caller's buffer. */
int pgxgo_legal_mask(pgxgo_t h, uint8_t* dst_dev /* [batch][mask_pitch] */);
int pgxgo_observe(pgxgo_t h, uint8_t* dst_dev /* [batch][obs_pitch] */);
int pgxgo_rewards(pgxgo_t h, float* dst_dev /* [batch][2], values of the last step call */);
int pgxgo_terminated(pgxgo_t h, uint8_t* dst_dev /* [batch], values of the last step call */);
int pgxgo_current_player(pgxgo_t h, uint8_t* dst_dev /* [batch] player id to move */);

/* Canonical state for tests, checkpoints and search: any pointer may be NULL on export.
 *   board [batch][N*N] int8 (0 empty, +1 black, -1 white); history [batch][8][N*N] int8,
 *   history[.][0] = current position, zero before the game started; ko int32 (-1 = none);
 *   to_play int8 (+1 black / -1 white); steps int32; passes int8; terminated uint8;
 *   black_player uint8; episode uint32; illegal uint32 (count of illegal actions received). */
int pgxgo_export_state(pgxgo_t h, int8_t* board_dev, int8_t* history_dev, int32_t* ko_dev, int8_t* to_play_dev,
                       int32_t* steps_dev, int8_t* passes_dev, uint8_t* terminated_dev, uint8_t* black_player_dev,
                       uint32_t* episode_dev, uint32_t* illegal_dev);
/* All pointers required.  Positions must be legal Go positions (every chain has a liberty). */
int pgxgo_import_state(pgxgo_t h, const int8_t* board_dev, const int8_t* history_dev, const int32_t* ko_dev,
                       const int8_t* to_play_dev, const int32_t* steps_dev, const int8_t* passes_dev,
                       const uint8_t* terminated_dev, const uint8_t* black_player_dev, const uint32_t* episode_dev);

/* Launch-shape knob: how many boards the step and rollout kernels put into one 64-lane wavefront, 1 up to
 * pgxgo_boards_per_wavefront(board_size).  0 restores the automatic choice made by pgxgo_init (fewer boards per
 * wavefront for small batches, where latency rather than throughput decides).  Results do not depend on it.
 * Returns the value now in use (> 0), or a negative error code. */
int pgxgo_set_boards_per_wavefront(pgxgo_t h, int32_t boards);

/* Positional superko (Appendix C "Go": Tromp-Taylor rules, whose repetition rule forbids a play that recreates an
 * earlier whole-board position of the game).  Off by default (simple ko only, as the benchmark configurations state).
 *   mode 2: the rule proper.  legal_action_mask leaves out every play that would recreate an earlier position of the
 *           game; playing one anyway is an illegal action like any other (game over, offender -1 / opponent +1,
 *           position unchanged).
 *   mode 1: the rule is looked at only when the move is played (same consequence for the offender), while the mask
 *           keeps showing the simple-ko set.
 *   mode 0 (table_dev ignored): off.
 * Positions are compared through two 32-bit Zobrist keys, one per colour (64 bits in all; probe chains are chosen by
 * the stone counts), kept in a per-game table inside table_dev.  pgxgo_superko_bytes: bytes of device memory the tables need (0 for invalid arguments); 256-byte aligned.
 * pgxgo_enable_superko switches the rule on with a caller-owned buffer that must outlive the handle.  The positions
 * known from then on are the ones the state still carries (the 8 history positions and the current one); the same
 * holds after pgxgo_import_state.  Needs max_steps <= 2*N*N.  Every entry point honours the rule: pgxgo_step /
 * pgxgo_step_sample, pgxgo_rollout, pgxgo_random_actions, the getters, and pgxgo_step_slots / pgxgo_copy_slots, where a
 * game that moves to another slot takes its table along (16 KB per 19x19 game, 4 KB per 9x9 game). */
size_t pgxgo_superko_bytes(int32_t batch, int32_t board_size);
int pgxgo_enable_superko(pgxgo_t h, int32_t mode, void* table_dev, size_t table_bytes);

/* Blocks the host until everything enqueued on the handle's stream has finished. */
int pgxgo_sync(pgxgo_t h);

/* Facts about the compiled kernels, for the harness. */
int32_t pgxgo_boards_per_wavefront(int32_t board_size); /* 3 for 19, 6 for 9, 0 otherwise */
int32_t pgxgo_num_actions(int32_t board_size);          /* N*N+1 (Table 1: 82 / 362) */
int32_t pgxgo_obs_bytes(int32_t board_size);            /* N*N*17 (Table 1: 9x9x17 / 19x19x17) */

const char* pgxgo_strerror(int code);
int pgxgo_last_hip_error(void); /* hipError_t of the most recent PGXGO_EHIP on this thread, else 0 */

/* Measurement helpers for the benchmark (no game logic).  pgxgo_fill_probe: one launch that fills nbytes (a multiple
 * of 16, dst_dev 16-byte aligned) with 16-byte vector stores of `value` -- the store-only ceiling the step kernel's
 * output rate is compared with.  kind: 0 ordinary stores, 1 with the non-temporal hint, 2 written through the L2 (what
 * the kernels use for whole 128-byte lines; the fastest fill: 15.5 against 16.8 us for 106 MB); anything else is
 * PGXGO_EINVAL.  pgxgo_empty_probe: `count` back-to-back launches of an empty kernel, enqueued from one host loop (the
 * time per launch is the gap between dependent launches on one stream). */
int pgxgo_fill_probe(void* dst_dev, size_t nbytes, uint32_t value, int32_t kind, void* stream);
int pgxgo_empty_probe(void* stream, int32_t count);

/* Harness helper: cross-lane shift semantics of the target (lane i reads lane i-1 / i+1, zero at
 * the wavefront ends).  Writes out_dev[0..63] = value seen from below, out_dev[64..127] = value
 * seen from above, for in_dev[0..63].  Used by the tests to check the lane layout the kernels rely on. */
int pgxgo_lane_shift_probe(const uint32_t* in_dev, uint32_t* out_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PGXGO_H_ */
