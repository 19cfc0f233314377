// go_oracle.cpp -- TEST INFRASTRUCTURE, not product code.
//
// A plain, slow, single-threaded CPU implementation of the batched Go environment
// of the Pgx paper (arXiv 2303.17503): Fig. 2 (init/step API, current_player,
// observation, legal_action_mask), Table 1 (Go 9x9: 9x9x17 obs, 82 actions;
// Go 19x19: 19x19x17 obs, 362 actions) and Appendix C "Go" (Tromp-Taylor rules,
// komi added to White's score, 2x8 history planes + one colour plane, the last
// action is pass, rewards +1/-1/0).  Where the paper is silent (simple ko,
// suicide illegal, ply cap 2*N*N, illegal action ends the game, counter-based
// action sampler, positional superko as an option in two readings: honoured by the
// legal mask, or enforced only when the move is played) each reading is stated next
// to the code that implements it.
//
// Only tests, the smoke check and the CPU-baseline leg of the benchmark may use
// this file.  It shares no code, header, table or helper with the HIP library.
//
// Everything is done on a plain int8 board (0 empty, +1 black, -1 white) with
// stack flood fills; nothing is packed, blocked or fused, so that each function
// can be checked against the rules by eye.
//
// Parity pins (tests/test_oracle_*.py): hand-built capture / ko / suicide /
// snapback / scoring positions, literal trial-placement legality, brute-force
// liberty recount by an independent Python implementation on tiny boards,
// per-ply invariants, board symmetries, closed forms on the empty board, hash
// vectors computed by an independent Python expression.
// Unpinned: agreement with the upstream Pgx library's own choices where the
// paper is silent (no upstream code or traces are available here).

#include <array>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

constexpr int kMaxN = 19;
constexpr int kMaxP = kMaxN * kMaxN;
constexpr int kHist = 8;     // Appendix C "Go", Observation: last 8 plies
constexpr int kPlanes = 17;  // 2*8 history planes + colour plane

struct Env {
  int8_t board[kMaxP];        // 0 empty, +1 black, -1 white; point p = row*N + col
  int8_t hist[kHist][kMaxP];  // hist[0] = current position, hist[i] = i plies ago; zero before game start
  int to_play;                // +1 black (moves first), -1 white
  int ko;                     // point forbidden by simple ko on the next ply, or -1
  int steps;                  // plies played in this episode (passes included)
  int passes;                 // consecutive passes so far (0,1,2)
  int terminated;             // state flag
  int black_player;           // player id (0/1) holding black this episode (Fig. 2: current_player independent of colour)
  uint32_t episode;           // number of resets so far
  uint32_t env_id;            // global environment index used by the hashes
  // positional superko (option): every whole-board position this episode has shown so far, the empty
  // starting board included, kept literally (with its two stone counts next to it)
  std::vector<std::array<int8_t, kMaxP>> seen;
  std::vector<std::array<int, 2>> seen_counts;   // {black stones, white stones} of seen[i]
};

struct Oracle {
  int B, N, P;
  uint32_t seed;
  int komi_x2, max_steps, auto_reset;
  // Positional superko (Tromp-Taylor: a play may not recreate an earlier whole-board position of the game).
  // 0: off (simple ko only).  2: the rule proper -- the legal mask leaves such plays out, so playing one is an
  // illegal action like any other.  1: the rule is looked at only when the move is played (the offender loses),
  // while the legal mask keeps showing the simple-ko set.
  int superko = 0;
  std::vector<Env> env;
  std::vector<float> out_rew;     // [B][2], by player id: values of the last step call
  std::vector<uint8_t> out_term;  // [B]
  std::vector<uint8_t> mask;      // [B][P+1]
  std::vector<uint8_t> obs;       // [B][P*17]
  std::vector<uint32_t> illegal;  // [B] count of illegal actions received
};

// ---- counter-based hash shared by definition (not by code) with the device sampler ----
inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du;
  x ^= x >> 15; x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}
inline uint32_t hash4(uint32_t seed, uint32_t tag, uint32_t env, uint32_t t) {
  return mix32(mix32(mix32(seed + 0x9E3779B9u * (tag + 1u)) ^ env) ^ t);
}

// ---- geometry ----
inline int neighbours(int N, int p, int out[4]) {
  int r = p / N, c = p % N, n = 0;
  if (r > 0) out[n++] = p - N;
  if (r < N - 1) out[n++] = p + N;
  if (c > 0) out[n++] = p - 1;
  if (c < N - 1) out[n++] = p + 1;
  return n;
}

// Chain (maximal 4-connected set of same-coloured stones) containing stone p.
// Returns its size, its cells in `cells`, and the number of distinct empty
// neighbour cells (liberties) in *libs, the first of them in *one_lib.
int chain_at(const int8_t* board, int N, int p, int* cells, int* libs, int* one_lib) {
  const int P = N * N;
  const int8_t col = board[p];
  bool seen[kMaxP], lib_seen[kMaxP];
  std::memset(seen, 0, P); std::memset(lib_seen, 0, P);
  int n = 0, head = 0, nl = 0, first = -1;
  cells[n++] = p; seen[p] = true;
  while (head < n) {
    int q = cells[head++], nb[4];
    int k = neighbours(N, q, nb);
    for (int i = 0; i < k; ++i) {
      int u = nb[i];
      if (board[u] == col) { if (!seen[u]) { seen[u] = true; cells[n++] = u; } }
      else if (board[u] == 0) { if (!lib_seen[u]) { lib_seen[u] = true; if (nl == 0) first = u; ++nl; } }
    }
  }
  if (libs) *libs = nl;
  if (one_lib) *one_lib = first;
  return n;
}

// Place a stone of colour `col` on empty point p and clear every opponent chain
// left without liberties (Tromp-Taylor: clear the opponent's colour first).
// Returns the number of captured stones; *cap_at = one captured point.
int place_and_capture(int8_t* board, int N, int p, int col, int* cap_at) {
  board[p] = (int8_t)col;
  int nb[4], cells[kMaxP], captured = 0;
  int k = neighbours(N, p, nb);
  for (int i = 0; i < k; ++i) {
    int q = nb[i];
    if (board[q] != -col) continue;  // may already have been cleared with an earlier neighbour
    int libs, n = chain_at(board, N, q, cells, &libs, nullptr);
    if (libs == 0) {
      for (int j = 0; j < n; ++j) board[cells[j]] = 0;
      captured += n;
      if (cap_at) *cap_at = cells[0];
    }
  }
  return captured;
}

// Legality by the literal definition: the point is empty, is not the ko point,
// and after placing the stone and clearing captured opponent chains the new
// stone's chain has a liberty (self-capture is not allowed).
bool legal_by_trial(const int8_t* board, int N, int col, int ko, int p) {
  if (board[p] != 0 || p == ko) return false;
  int8_t tmp[kMaxP];
  std::memcpy(tmp, board, N * N);
  place_and_capture(tmp, N, p, col, nullptr);
  int cells[kMaxP], libs;
  chain_at(tmp, N, p, cells, &libs, nullptr);
  return libs > 0;
}

// Legality through per-chain liberty counts (each chain flooded once): an empty
// non-ko point is playable iff it has an empty neighbour, or touches an own
// chain that keeps another liberty, or touches an opponent chain whose only
// liberty is this point (which is then captured).
void legal_by_chains(const int8_t* board, int N, int col, int ko, uint8_t* mask) {
  const int P = N * N;
  int chain_libs[kMaxP];
  bool labelled[kMaxP];
  std::memset(labelled, 0, P);
  int cells[kMaxP];
  for (int p = 0; p < P; ++p) {
    if (board[p] == 0 || labelled[p]) continue;
    int libs, n = chain_at(board, N, p, cells, &libs, nullptr);
    for (int j = 0; j < n; ++j) { labelled[cells[j]] = true; chain_libs[cells[j]] = libs; }
  }
  for (int p = 0; p < P; ++p) {
    bool ok = false;
    if (board[p] == 0 && p != ko) {
      int nb[4], k = neighbours(N, p, nb);
      for (int i = 0; i < k; ++i) {
        int q = nb[i];
        if (board[q] == 0) ok = true;
        else if (board[q] == col && chain_libs[q] >= 2) ok = true;
        else if (board[q] == -col && chain_libs[q] == 1) ok = true;
      }
    }
    mask[p] = ok ? 1 : 0;
  }
  mask[P] = 1;  // pass (the last action) is always available
}

// Tromp-Taylor area: a player's stones plus the empty regions that reach only
// that player's colour.
void area_score(const int8_t* board, int N, int* area_black, int* area_white) {
  const int P = N * N;
  bool seen[kMaxP];
  std::memset(seen, 0, P);
  int ab = 0, aw = 0, stack[kMaxP];
  for (int p = 0; p < P; ++p) {
    if (board[p] == 1) ++ab;
    else if (board[p] == -1) ++aw;
    else if (!seen[p]) {
      int n = 0, head = 0;
      bool tb = false, tw = false;
      stack[n++] = p; seen[p] = true;
      while (head < n) {
        int q = stack[head++], nb[4], k = neighbours(N, q, nb);
        for (int i = 0; i < k; ++i) {
          int u = nb[i];
          if (board[u] == 1) tb = true;
          else if (board[u] == -1) tw = true;
          else if (!seen[u]) { seen[u] = true; stack[n++] = u; }
        }
      }
      if (tb && !tw) ab += n;
      if (tw && !tb) aw += n;
    }
  }
  *area_black = ab; *area_white = aw;
}

// ---- positional superko (Appendix C "Go": Tromp-Taylor rules; their repetition rule forbids a play that
// recreates any earlier whole-board position of the game).
void stone_counts(const int8_t* board, int* nb, int* nw) {
  int b = 0, w = 0;
  for (int p = 0; p < kMaxP; ++p) { if (board[p] == 1) ++b; else if (board[p] == -1) ++w; }
  *nb = b; *nw = w;
}
void remember(Env& e) {
  std::array<int8_t, kMaxP> pos;
  std::memcpy(pos.data(), e.board, kMaxP);
  e.seen.push_back(pos);
  int nb, nw;
  stone_counts(e.board, &nb, &nw);
  e.seen_counts.push_back({nb, nw});
}
// the literal test: compare the whole board with every earlier position
bool seen_before(const Env& e, const int8_t* board) {
  for (const auto& pos : e.seen)
    if (std::memcmp(pos.data(), board, kMaxP) == 0) return true;
  return false;
}
// The same test, skipping the earlier positions whose stone counts differ from the board's (equal boards have
// equal counts); used where every legal point of every ply is tried.  Pinned against seen_before by the tests.
bool seen_before_counted(const Env& e, const int8_t* board) {
  int nb, nw;
  stone_counts(board, &nb, &nw);
  for (size_t i = 0; i < e.seen.size(); ++i)
    if (e.seen_counts[i][0] == nb && e.seen_counts[i][1] == nw && std::memcmp(e.seen[i].data(), board, kMaxP) == 0) return true;
  return false;
}
// would playing `col` on p (a move the simple rules allow) recreate an earlier position?
bool repeats_position(const Env& e, int N, int p, int col, bool literal) {
  int8_t tmp[kMaxP];
  std::memcpy(tmp, e.board, kMaxP);
  place_and_capture(tmp, N, p, col, nullptr);
  return literal ? seen_before(e, tmp) : seen_before_counted(e, tmp);
}

void env_reset(Oracle* o, Env& e) {
  std::memset(e.board, 0, sizeof e.board);
  std::memset(e.hist, 0, sizeof e.hist);
  e.to_play = 1; e.ko = -1; e.steps = 0; e.passes = 0; e.terminated = 0;
  // Fig. 2: which player acts first is drawn by a PRNG, independently of colour.
  e.black_player = (int)(hash4(o->seed, 1u, e.env_id, e.episode) & 1u);
  e.seen.clear(); e.seen_counts.clear();
  if (o->superko) remember(e);
}

void env_outputs(Oracle* o, int b) {
  Env& e = o->env[b];
  const int P = o->P;
  uint8_t* m = &o->mask[(size_t)b * (P + 1)];
  legal_by_chains(e.board, o->N, e.to_play, e.ko, m);
  if (o->superko == 2)   // the rule proper: try every point the simple rules allow; pass never repeats by a play
    for (int p = 0; p < P; ++p)
      if (m[p] && repeats_position(e, o->N, p, e.to_play, false)) m[p] = 0;
  // Observation of the player to move (Appendix C "Go", Observation): for each of
  // the last 8 positions, most recent first, one plane of the mover's stones and
  // one of the opponent's; the 17th plane is all ones when black is to move.
  // Layout [point][plane], one byte each.
  uint8_t* ob = &o->obs[(size_t)b * P * kPlanes];
  for (int p = 0; p < P; ++p) {
    for (int i = 0; i < kHist; ++i) {
      ob[p * kPlanes + 2 * i] = (e.hist[i][p] == e.to_play) ? 1 : 0;
      ob[p * kPlanes + 2 * i + 1] = (e.hist[i][p] == -e.to_play) ? 1 : 0;
    }
    ob[p * kPlanes + 16] = (e.to_play == 1) ? 1 : 0;
  }
}

void env_step(Oracle* o, int b, int a) {
  Env& e = o->env[b];
  const int N = o->N, P = o->P;
  float* rew = &o->out_rew[(size_t)b * 2];
  if (a == -1) return;  // skip: nothing about this environment changes
  if (e.terminated) {   // only reachable without auto-reset: frozen, zero rewards
    rew[0] = rew[1] = 0.f; o->out_term[b] = 1;
    return;
  }
  rew[0] = rew[1] = 0.f;
  const int col = e.to_play;
  const int mover = (col == 1) ? e.black_player : 1 - e.black_player;
  const uint8_t* m = &o->mask[(size_t)b * (P + 1)];
  bool ended = false;
  if (a < 0 || a > P || !m[a] || (o->superko == 1 && a < P && repeats_position(e, N, a, col, true))) {
    // Illegal action: the game ends at once, the offender loses; the position,
    // ply counter and side to move stay as they were.
    o->illegal[b] += 1;
    rew[mover] = -1.f; rew[1 - mover] = 1.f;
    ended = true;
  } else {
    if (a == P) {
      e.passes += 1;
      e.ko = -1;
    } else {
      int nb[4], k = neighbours(N, a, nb);
      bool lone = true;  // no own-colour neighbour before the move
      for (int i = 0; i < k; ++i) if (e.board[nb[i]] == col) lone = false;
      int cap_at = -1;
      int captured = place_and_capture(e.board, N, a, col, &cap_at);
      // Simple ko: exactly one stone was taken, the capturing stone stands alone
      // and its only liberty is the point just vacated.
      int cells[kMaxP], libs, one;
      int n = chain_at(e.board, N, a, cells, &libs, &one);
      e.ko = (captured == 1 && lone && n == 1 && libs == 1 && one == cap_at) ? cap_at : -1;
      e.passes = 0;
      if (o->superko) remember(e);
    }
    e.steps += 1;
    for (int i = kHist - 1; i > 0; --i) std::memcpy(e.hist[i], e.hist[i - 1], P);
    std::memcpy(e.hist[0], e.board, P);
    e.to_play = -col;
    if (e.passes >= 2 || e.steps >= o->max_steps) {
      int ab, aw;
      area_score(e.board, N, &ab, &aw);
      int d = 2 * (ab - aw) - o->komi_x2;  // komi counts for White
      float s = d > 0 ? 1.f : (d < 0 ? -1.f : 0.f);
      rew[e.black_player] = s; rew[1 - e.black_player] = -s;
      ended = true;
    }
  }
  if (ended) {
    e.terminated = 1;
    o->out_term[b] = 1;
    if (o->auto_reset) {  // Sec. 4.1: the environment resets to the initial state on termination
      e.episode += 1;
      env_reset(o, e);
    }
  } else {
    o->out_term[b] = 0;
  }
  env_outputs(o, b);
}

void rebuild_seen(Oracle* o, Env& e) {
  e.seen.clear(); e.seen_counts.clear();
  if (!o->superko) return;
  for (int i = kHist - 1; i >= 0; --i) {
    std::array<int8_t, kMaxP> pos;
    pos.fill(0);
    std::memcpy(pos.data(), e.hist[i], o->P);
    e.seen.push_back(pos);
    int nb, nw;
    stone_counts(pos.data(), &nb, &nw);
    e.seen_counts.push_back({nb, nw});
  }
  remember(e);
}

}  // namespace

extern "C" {

void* oracle_create(int B, int N, uint32_t seed, int komi_x2, int max_steps, int auto_reset,
                    const int32_t* env_ids /* nullable: env b has global index b */) {
  if (B <= 0 || N < 2 || N > kMaxN) return nullptr;
  Oracle* o = new Oracle;
  o->B = B; o->N = N; o->P = N * N; o->seed = seed;
  o->komi_x2 = komi_x2; o->max_steps = max_steps > 0 ? max_steps : 2 * N * N; o->auto_reset = auto_reset;
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

void oracle_destroy(void* h) { delete (Oracle*)h; }

void oracle_reset(void* h) {
  Oracle* o = (Oracle*)h;
  for (int b = 0; b < o->B; ++b) {
    Env& e = o->env[b];
    e.episode += 1;
    env_reset(o, e);
    o->out_rew[2 * b] = o->out_rew[2 * b + 1] = 0.f; o->out_term[b] = 0;
    env_outputs(o, b);
  }
}

void oracle_step(void* h, const int32_t* actions) {
  Oracle* o = (Oracle*)h;
  for (int b = 0; b < o->B; ++b) env_step(o, b, actions[b]);
}

// Uniform random legal action: the k-th set entry (ascending action index) of the
// legal mask, k = hash(seed, 0, env, t) mod legal_count.  Environments with
// t < start_t[env] get the skip action -1.
void oracle_random_actions(void* h, uint32_t seed, uint32_t t, const int32_t* start_t, int32_t* actions) {
  Oracle* o = (Oracle*)h;
  const int A = o->P + 1;
  for (int b = 0; b < o->B; ++b) {
    if (start_t && (int64_t)t < (int64_t)start_t[b]) { actions[b] = -1; continue; }
    const uint8_t* m = &o->mask[(size_t)b * A];
    int count = 0;
    for (int a = 0; a < A; ++a) count += m[a];
    uint32_t k = hash4(seed, 0u, o->env[b].env_id, t) % (uint32_t)count;
    int pick = -1;
    for (int a = 0; a < A; ++a) if (m[a]) { if (k == 0) { pick = a; break; } --k; }
    actions[b] = pick;
  }
}

uint32_t oracle_hash(uint32_t seed, uint32_t tag, uint32_t env, uint32_t t) { return hash4(seed, tag, env, t); }

// ---- outputs of the environment API ----
void oracle_legal_mask(void* h, uint8_t* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->mask.data(), o->mask.size()); }
void oracle_observe(void* h, uint8_t* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->obs.data(), o->obs.size()); }
void oracle_rewards(void* h, float* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->out_rew.data(), o->out_rew.size() * sizeof(float)); }
void oracle_terminated(void* h, uint8_t* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->out_term.data(), o->out_term.size()); }
void oracle_current_player(void* h, uint8_t* dst) {
  Oracle* o = (Oracle*)h;
  for (int b = 0; b < o->B; ++b) {
    const Env& e = o->env[b];
    dst[b] = (uint8_t)(e.to_play == 1 ? e.black_player : 1 - e.black_player);
  }
}
void oracle_illegal_count(void* h, uint32_t* dst) { Oracle* o = (Oracle*)h; std::memcpy(dst, o->illegal.data(), o->illegal.size() * 4); }

// ---- canonical state, for comparison and for setting up positions ----
void oracle_export_state(void* h, int8_t* board /*[B][P]*/, int8_t* history /*[B][8][P]*/, int32_t* ko, int8_t* to_play /*+1/-1*/,
                         int32_t* steps, int8_t* passes, uint8_t* terminated, uint8_t* black_player, uint32_t* episode) {
  Oracle* o = (Oracle*)h;
  const int P = o->P;
  for (int b = 0; b < o->B; ++b) {
    const Env& e = o->env[b];
    if (board) std::memcpy(board + (size_t)b * P, e.board, P);
    if (history) for (int i = 0; i < kHist; ++i) std::memcpy(history + ((size_t)b * kHist + i) * P, e.hist[i], P);
    if (ko) ko[b] = e.ko;
    if (to_play) to_play[b] = (int8_t)e.to_play;
    if (steps) steps[b] = e.steps;
    if (passes) passes[b] = (int8_t)e.passes;
    if (terminated) terminated[b] = (uint8_t)e.terminated;
    if (black_player) black_player[b] = (uint8_t)e.black_player;
    if (episode) episode[b] = e.episode;
  }
}

void oracle_import_state(void* h, const int8_t* board, const int8_t* history, const int32_t* ko, const int8_t* to_play,
                         const int32_t* steps, const int8_t* passes, const uint8_t* terminated, const uint8_t* black_player,
                         const uint32_t* episode) {
  Oracle* o = (Oracle*)h;
  const int P = o->P;
  for (int b = 0; b < o->B; ++b) {
    Env& e = o->env[b];
    std::memcpy(e.board, board + (size_t)b * P, P);
    for (int i = 0; i < kHist; ++i) std::memcpy(e.hist[i], history + ((size_t)b * kHist + i) * P, P);
    e.ko = ko[b]; e.to_play = to_play[b]; e.steps = steps[b]; e.passes = passes[b];
    e.terminated = terminated[b]; e.black_player = black_player[b]; e.episode = episode[b];
    o->out_rew[2 * b] = o->out_rew[2 * b + 1] = 0.f; o->out_term[b] = (uint8_t)e.terminated;
    rebuild_seen(o, e);
    env_outputs(o, b);
  }
}

// Switches positional superko on or off.  The positions known from then on are the ones the state still
// carries: the 8 history positions (entries from before the game started are the empty board) and the current one.
// mode 0: off; 1: looked at only when the move is played; 2: honoured by the legal mask (the rule proper).
void oracle_set_superko(void* h, int mode) {
  Oracle* o = (Oracle*)h;
  o->superko = (mode == 1 || mode == 2) ? mode : 0;
  for (int b = 0; b < o->B; ++b) { rebuild_seen(o, o->env[b]); env_outputs(o, b); }
}

// For the pins: would playing the mover's colour on p recreate an earlier position of environment b, by the literal
// whole-board comparison with every earlier position (no count shortcut)?  p must be empty.
int oracle_repeats_literal(void* h, int b, int p) {
  Oracle* o = (Oracle*)h;
  const Env& e = o->env[b];
  return repeats_position(e, o->N, p, e.to_play, true) ? 1 : 0;
}
int oracle_seen_count(void* h, int b) { return (int)((Oracle*)h)->env[b].seen.size(); }

// ---- stand-alone rule functions on a caller-supplied board (used by the pins) ----
void oracle_legal_trial(const int8_t* board, int N, int to_play, int ko, uint8_t* mask /*[P+1]*/) {
  for (int p = 0; p < N * N; ++p) mask[p] = legal_by_trial(board, N, to_play, ko, p) ? 1 : 0;
  mask[N * N] = 1;
}
void oracle_legal_chains(const int8_t* board, int N, int to_play, int ko, uint8_t* mask) { legal_by_chains(board, N, to_play, ko, mask); }
void oracle_area(const int8_t* board, int N, int32_t* area_black, int32_t* area_white) {
  int ab, aw; area_score(board, N, &ab, &aw); *area_black = ab; *area_white = aw;
}
// size and liberty count of the chain at p (0,0 on an empty point)
void oracle_chain(const int8_t* board, int N, int p, int32_t* size, int32_t* libs) {
  if (board[p] == 0) { *size = 0; *libs = 0; return; }
  int cells[kMaxP], l; *size = chain_at(board, N, p, cells, &l, nullptr); *libs = l;
}

}  // extern "C"
