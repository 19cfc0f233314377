// hex_oracle.cpp -- TEST INFRASTRUCTURE, not product code.
//
// A plain, slow, single-threaded CPU implementation of the batched Hex environment of the Pgx paper
// (arXiv 2303.17503): Fig. 2 (init/step API, current_player, observation, legal_action_mask), Table 1
// (Hex: 11x11x4 observation, 122 actions) and Appendix C "Hex" (stones are placed in turn, a player wins
// by joining their two sides, no draw exists, the swap rule, planes = mover's stones, opponent's stones,
// colour, swap-is-legal; actions 0..N*N-1 place a stone, action N*N swaps and is available on the second
// turn only; rewards +1/-1).  Sec. 4.1: random policy and auto-reset.
//
// Where the paper is silent the readings are:
//   * Black moves first and joins the top row (row 0) with the bottom row (row N-1); White joins the
//     left column with the right column.
//   * Cell (r,c) touches (r,c-1) (r,c+1) (r-1,c) (r-1,c+1) (r+1,c) (r+1,c-1): the rhombic board whose
//     rows lean to the right going up.
//   * Swap: the lone black stone at (r,c) is taken off and a white stone is put at the mirrored cell
//     (c,r); the ply counts like any other and Black is to move next.
//   * Illegal action (occupied cell, swap when it is not offered, out of range): the game ends at once,
//     offender -1 / opponent +1, position and side to move unchanged, a per-game counter records it.
//   * Colour plane: all ones when Black is to move.  Swap plane: all ones when swap is legal.
//   * Seats: black_player = hash(seed, 1, env, episode) & 1; rewards are indexed by player id.
//   * A finished game that is stepped again (no auto-reset) is frozen: zero rewards, terminated stays 1.
//     Its mask and observation follow the ordinary rules on the final position.
//   * Auto-reset: the finishing ply returns its rewards/terminated with the fresh game's mask/observation.
//   * Action -1 (not in the paper) leaves the environment untouched.
//   * Sampler: the k-th legal action in ascending order, k = hash(seed,0,env,t) mod legal_count; action 0
//     when nothing is legal (a finished game on a full board, which ignores it).
//
// Only tests, the smoke check and the CPU-baseline leg of the benchmark may use this file.  It shares no
// code, header, table or helper with the HIP library.
//
// Everything is done on a plain int8 board (0 empty, +1 black, -1 white); the winner test is a whole-board
// search from one side after every ply, nothing is incremental, packed or fused.
//
// Parity pins (tests/test_hex_oracle.py): the paper's printed shapes and swap rule, hand-built winning and
// non-winning paths that tell the two diagonal directions apart, the no-draw theorem on random full
// boards, exhaustive play on 2x2 and 3x3 and random games on 2x2..11x11 against an independent Python
// implementation (union-find over cube coordinates), the half-turn and transpose-and-recolour symmetries,
// the shortest possible game, hash vectors.  Unpinned: agreement with the upstream Pgx library's own choices
// where the paper is silent (sides, lean of the board, illegal actions).

#include <cstdint>
#include <cstring>
#include <vector>

namespace {

constexpr int kMaxN = 11;
constexpr int kMaxP = kMaxN * kMaxN;
constexpr int kPlanes = 4;

struct Env {
  int8_t board[kMaxP];  // 0 empty, +1 black, -1 white; cell p = row*N + col
  int to_play;          // +1 black (moves first), -1 white
  int steps;            // plies played in this episode (the swap counts)
  int terminated;
  int black_player;     // player id (0/1) holding black this episode
  uint32_t episode;
  uint32_t env_id;
};

struct Oracle {
  int B, N, P;
  uint32_t seed;
  int auto_reset;
  std::vector<Env> env;
  std::vector<float> out_rew;     // [B][2] by player id
  std::vector<uint8_t> out_term;  // [B]
  std::vector<uint8_t> mask;      // [B][P+1]
  std::vector<uint8_t> obs;       // [B][P*4]
  std::vector<uint32_t> illegal;  // [B]
};

inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du;
  x ^= x >> 15; x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}
inline uint32_t hash4(uint32_t seed, uint32_t tag, uint32_t env, uint32_t t) {
  return mix32(mix32(mix32(seed + 0x9E3779B9u * (tag + 1u)) ^ env) ^ t);
}

// the (up to) six cells touching p
inline int neighbours(int N, int p, int out[6]) {
  static const int dr[6] = {0, 0, -1, -1, 1, 1};
  static const int dc[6] = {-1, 1, 0, 1, 0, -1};
  const int r = p / N, c = p % N;
  int k = 0;
  for (int i = 0; i < 6; ++i) {
    const int rr = r + dr[i], cc = c + dc[i];
    if (rr >= 0 && rr < N && cc >= 0 && cc < N) out[k++] = rr * N + cc;
  }
  return k;
}

// Appendix C "Hex", Rules: has `col` joined its two sides?  Search from every stone of that colour on the
// first side (top row for Black, left column for White) through touching stones of the same colour.
bool joined(const int8_t* board, int N, int col) {
  const int P = N * N;
  bool seen[kMaxP] = {false};
  int stack[kMaxP], sp = 0;
  for (int i = 0; i < N; ++i) {
    const int p = (col == 1) ? i : i * N;
    if (board[p] == col) { seen[p] = true; stack[sp++] = p; }
  }
  while (sp) {
    const int p = stack[--sp];
    const bool far_side = (col == 1) ? (p / N == N - 1) : (p % N == N - 1);
    if (far_side) return true;
    int nb[6], k = neighbours(N, p, nb);
    for (int i = 0; i < k; ++i)
      if (board[nb[i]] == col && !seen[nb[i]]) { seen[nb[i]] = true; stack[sp++] = nb[i]; }
  }
  (void)P;
  return false;
}

void env_reset(Oracle* o, Env& e) {
  std::memset(e.board, 0, sizeof e.board);
  e.to_play = 1; e.steps = 0; e.terminated = 0;
  e.black_player = (int)(hash4(o->seed, 1u, e.env_id, e.episode) & 1u);
}

void env_outputs(Oracle* o, int b) {
  Env& e = o->env[b];
  const int P = o->P;
  uint8_t* m = &o->mask[(size_t)b * (P + 1)];
  // Appendix C "Hex", Action: any empty cell; the swap only on the second turn.
  const int swap_ok = (e.steps == 1) ? 1 : 0;
  for (int p = 0; p < P; ++p) m[p] = (e.board[p] == 0) ? 1 : 0;
  m[P] = (uint8_t)swap_ok;
  // Observation of the player to move, layout [cell][plane]: own stones, opponent's stones, colour, swap.
  uint8_t* ob = &o->obs[(size_t)b * P * kPlanes];
  for (int p = 0; p < P; ++p) {
    ob[p * kPlanes + 0] = (e.board[p] == e.to_play) ? 1 : 0;
    ob[p * kPlanes + 1] = (e.board[p] == -e.to_play) ? 1 : 0;
    ob[p * kPlanes + 2] = (e.to_play == 1) ? 1 : 0;
    ob[p * kPlanes + 3] = (uint8_t)swap_ok;
  }
}

void env_step(Oracle* o, int b, int a) {
  Env& e = o->env[b];
  const int N = o->N, P = o->P;
  float* rew = &o->out_rew[(size_t)b * 2];
  if (a == -1) return;
  if (e.terminated) {
    rew[0] = rew[1] = 0.f; o->out_term[b] = 1;
    return;
  }
  rew[0] = rew[1] = 0.f;
  const int col = e.to_play;
  const int mover = (col == 1) ? e.black_player : 1 - e.black_player;
  const uint8_t* m = &o->mask[(size_t)b * (P + 1)];
  bool ended = false;
  if (a < 0 || a > P || !m[a]) {
    o->illegal[b] += 1;
    rew[mover] = -1.f; rew[1 - mover] = 1.f;
    ended = true;
  } else {
    if (a == P) {
      // swap rule: the first player's stone becomes the second player's, at the mirrored cell
      int at = -1;
      for (int p = 0; p < P; ++p) if (e.board[p] != 0) at = p;
      const int r = at / N, c = at % N;
      e.board[at] = 0;
      e.board[c * N + r] = (int8_t)col;
    } else {
      e.board[a] = (int8_t)col;
    }
    e.steps += 1;
    e.to_play = -col;
    if (joined(e.board, N, col)) {
      rew[mover] = 1.f; rew[1 - mover] = -1.f;
      ended = true;
    }
  }
  if (ended) {
    e.terminated = 1;
    o->out_term[b] = 1;
    if (o->auto_reset) {
      e.episode += 1;
      env_reset(o, e);
    }
  } else {
    o->out_term[b] = 0;
  }
  env_outputs(o, b);
}

}  // namespace

extern "C" {

void* hexo_create(int B, int N, uint32_t seed, int auto_reset, const int32_t* env_ids) {
  if (B <= 0 || N < 2 || N > kMaxN) return nullptr;
  Oracle* o = new Oracle;
  o->B = B; o->N = N; o->P = N * N; o->seed = seed; o->auto_reset = auto_reset;
  o->env.resize(B);
  o->out_rew.assign((size_t)B * 2, 0.f);
  o->out_term.assign(B, 0);
  o->mask.assign((size_t)B * (o->P + 1), 0);
  o->obs.assign((size_t)B * o->P * kPlanes, 0);
  o->illegal.assign(B, 0);
  for (int b = 0; b < B; ++b) {
    Env& e = o->env[b];
    e.env_id = env_ids ? (uint32_t)env_ids[b] : (uint32_t)b;
    e.episode = 0;
    env_reset(o, e);
    env_outputs(o, b);
  }
  return o;
}

void hexo_destroy(void* h) { delete (Oracle*)h; }

void hexo_reset(void* h) {
  Oracle* o = (Oracle*)h;
  for (int b = 0; b < o->B; ++b) {
    Env& e = o->env[b];
    e.episode += 1;
    env_reset(o, e);
    o->out_rew[2 * b] = o->out_rew[2 * b + 1] = 0.f; o->out_term[b] = 0;
    env_outputs(o, b);
  }
}

void hexo_step(void* h, const int32_t* actions) {
  Oracle* o = (Oracle*)h;
  for (int b = 0; b < o->B; ++b) env_step(o, b, actions[b]);
}

void hexo_random_actions(void* h, uint32_t seed, uint32_t t, const int32_t* start_t, int32_t* actions) {
  Oracle* o = (Oracle*)h;
  const int A = o->P + 1;
  for (int b = 0; b < o->B; ++b) {
    if (start_t && (int64_t)t < (int64_t)start_t[b]) { actions[b] = -1; continue; }
    const uint8_t* m = &o->mask[(size_t)b * A];
    int count = 0;
    for (int a = 0; a < A; ++a) count += m[a];
    if (count == 0) { actions[b] = 0; continue; }
    uint32_t k = hash4(seed, 0u, o->env[b].env_id, t) % (uint32_t)count;
    int pick = -1;
    for (int a = 0; a < A; ++a) if (m[a]) { if (k == 0) { pick = a; break; } --k; }
    actions[b] = pick;
  }
}

uint32_t hexo_hash(uint32_t seed, uint32_t tag, uint32_t env, uint32_t t) { return hash4(seed, tag, env, t); }

void hexo_legal_mask(void* h, uint8_t* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->mask.data(), o->mask.size()); }
void hexo_observe(void* h, uint8_t* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->obs.data(), o->obs.size()); }
void hexo_rewards(void* h, float* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->out_rew.data(), o->out_rew.size() * sizeof(float)); }
void hexo_terminated(void* h, uint8_t* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->out_term.data(), o->out_term.size()); }
void hexo_current_player(void* h, uint8_t* dst) {
  Oracle* o = (Oracle*)h;
  for (int b = 0; b < o->B; ++b) {
    const Env& e = o->env[b];
    dst[b] = (uint8_t)((e.to_play == 1) ? e.black_player : 1 - e.black_player);
  }
}
void hexo_illegal_count(void* h, uint32_t* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->illegal.data(), o->illegal.size() * 4); }

void hexo_export_state(void* h, int8_t* board /*[B][P]*/, int8_t* to_play, int32_t* steps, uint8_t* terminated, uint8_t* black_player,
                       uint32_t* episode) {
  Oracle* o = (Oracle*)h;
  for (int b = 0; b < o->B; ++b) {
    const Env& e = o->env[b];
    std::memcpy(board + (size_t)b * o->P, e.board, o->P);
    to_play[b] = (int8_t)e.to_play; steps[b] = e.steps; terminated[b] = (uint8_t)e.terminated;
    black_player[b] = (uint8_t)e.black_player; episode[b] = e.episode;
  }
}

void hexo_import_state(void* h, const int8_t* board, const int8_t* to_play, const int32_t* steps, const uint8_t* terminated,
                       const uint8_t* black_player, const uint32_t* episode) {
  Oracle* o = (Oracle*)h;
  for (int b = 0; b < o->B; ++b) {
    Env& e = o->env[b];
    std::memset(e.board, 0, sizeof e.board);
    std::memcpy(e.board, board + (size_t)b * o->P, o->P);
    e.to_play = to_play[b]; e.steps = steps[b]; e.terminated = terminated[b];
    e.black_player = black_player[b]; e.episode = episode[b];
    o->out_rew[2 * b] = o->out_rew[2 * b + 1] = 0.f; o->out_term[b] = (uint8_t)e.terminated;
    env_outputs(o, b);
  }
}

// stand-alone: has colour `col` (+1/-1) joined its sides on this board?
int hexo_joined(const int8_t* board, int N, int col) { return joined(board, N, col) ? 1 : 0; }

}  // extern "C"
