// pgxhex.hip -- batched Hex environment step for AMD MI355X (gfx950, wave64), C ABI in include/pgxhex.h.
//
// What is computed: the Hex environment of the Pgx paper (arXiv 2303.17503): Fig. 2 (init/step API,
// legal_action_mask, observation, current_player), Table 1 (11x11x4 observation, 122 actions), Appendix C "Hex"
// (stones placed in turn, a player wins by joining their two sides, swap rule on the second turn, planes =
// mover's stones / opponent's stones / colour / swap-is-legal, rewards +1/-1), Sec. 4.1 (random policy,
// auto-reset on termination).
//
// Mapping (the same as the Go kernels of this library): one board row per lane, 5 boards per wavefront, board j
// in lanes 12j+1 .. 12j+11 with all-zero sentinel lanes between boards.  A row is one dword (black in bits 0-10,
// white in bits 16-26), so a board is 44 bytes of state plus one 16-byte scalar record.  The six neighbours of a
// cell are two register shifts plus the two DPP row shifts and their one-column offsets; the winner test floods
// the mover's stones from the stone just placed and asks by ballot whether the flood touches both of the mover's
// sides.  Mask and observation bytes are staged as a bit stream in LDS (4 bits per cell for the observation) and
// written as aligned 16-byte vectors; the boards of a wavefront form one contiguous run of bytes.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>
#include <stdlib.h>

#include "pgxhex.h"
#include "wave_common.hpp"

namespace {

using namespace pgxwave;

thread_local int g_last_hip = 0;

#define HIPCHK(expr)                                   \
  do {                                                 \
    hipError_t e_ = (expr);                            \
    if (e_ != hipSuccess) {                            \
      g_last_hip = (int)e_;                            \
      return PGXHEX_EHIP;                              \
    }                                                  \
  } while (0)

constexpr int N = PGXHEX_N;
constexpr int P = N * N;
constexpr int A = P + 1;                    // Table 1: 122 actions
constexpr int OBS = P * 4;                  // Table 1: 11 x 11 x 4
constexpr int STRIDE = N + 1;               // lanes per board, one of them the zero sentinel row
constexpr int W = 63 / STRIDE;              // boards per wavefront
constexpr uint32_t FULL = (1u << N) - 1u;
constexpr int kWavesPerBlock = 4;           // wavefronts never synchronise with each other after the table is filled
constexpr int OBS_DW = ((15 + W * OBS + 31) / 32 + 3) / 4 * 4;   // LDS dwords of a wavefront's observation bit stream
constexpr int MASK_DW = 64;                                      // the mask stream is cleared by one store per lane
static_assert(A == PGXHEX_ACTIONS && OBS == PGXHEX_OBS_BYTES, "header constants");
static_assert((15 + W * A + 31) / 32 <= MASK_DW, "mask stream fits its staging area");
static_assert(N <= 16, "a row holds both colours in one dword");
static_assert(N == 11, "the action decode divides by 11 with a multiply and a shift");

// per-board scalars, one 16-byte record: x = steps[0:8) | white_to_move[8] | terminated[9] | black_player[10],
// y = episode, z = illegal actions received
struct Meta {
  int steps, wtm, term, bp;
  uint32_t episode, illegal;
};
__device__ __forceinline__ Meta unpack_meta(uint4 v) {
  Meta m;
  m.steps = v.x & 0xFF; m.wtm = (v.x >> 8) & 1; m.term = (v.x >> 9) & 1; m.bp = (v.x >> 10) & 1;
  m.episode = v.y; m.illegal = v.z;
  return m;
}
__device__ __forceinline__ uint4 pack_meta(const Meta& m) {
  return make_uint4((uint32_t)m.steps | ((uint32_t)m.wtm << 8) | ((uint32_t)m.term << 9) | ((uint32_t)m.bp << 10), m.episode, m.illegal, 0u);
}

struct Lane {
  int lane, j, r, b;     // lane id, board slot in the wavefront, row, environment index
  bool valid;            // this lane holds a real row of a real board
  bool boardok;          // slot j holds a real board (also true for its sentinel lane)
  uint32_t seglo, seghi; // lanes of the rows of this lane's board
  uint32_t full;
  __device__ __forceinline__ Lane(int wave, int lane_, int B) {
    lane = lane_;
    j = lane / STRIDE;
    const int rr = lane - j * STRIDE;
    r = rr - 1;
    b = wave * W + j;
    boardok = (j < W) && (b < B);
    valid = boardok && rr >= 1;
    const uint64_t seg = (j < W) ? (((1ull << N) - 1ull) << (j * STRIDE + 1)) : 0ull;
    seglo = (uint32_t)seg; seghi = (uint32_t)(seg >> 32);
    full = valid ? FULL : 0u;
  }
};

// all cells touching the set x (Appendix C "Hex"; reading: (r,c) touches (r,c-1) (r,c+1) (r-1,c) (r-1,c+1) (r+1,c)
// (r+1,c-1)).  Bits beyond column N-1 may be set; callers intersect with on-board sets.
__device__ __forceinline__ uint32_t hex_dilate(uint32_t x) {
  const uint32_t up = from_lane_below(x), down = from_lane_above(x);   // rows r-1 and r+1
  return (x << 1) | (x >> 1) | up | (up >> 1) | down | (down << 1);
}

// bit i of x (x < 256) -> bit 4i
__device__ __forceinline__ uint32_t spread_every4(uint32_t x) {
  x = (x | (x << 12)) & 0x000F000Fu;
  x = (x | (x << 6)) & 0x03030303u;
  x = (x | (x << 3)) & 0x11111111u;
  return x;
}

// Legal mask [122] and observation [11][11][4] bytes of every board of the wavefront (Fig. 2, Table 1, Appendix C
// "Hex" Observation / Action) from the position after the ply.
__device__ __forceinline__ void emit_outputs(const Lane& L, uint32_t bk, uint32_t wt, const Meta& m, int wave, int B, uint8_t* mask, uint8_t* obs,
                                             uint32_t* lds_mask, uint32_t* lds_obs, const uint2* lut) {
  const int b0 = wave * W;
  const int nb = B - b0 < W ? B - b0 : W;
  const uint32_t E = L.full & ~(bk | wt);
  const bool swap = m.steps == 1;   // the swap is on offer on the second turn only
  if (mask) {
    lds_mask[L.lane] = 0u;
    wave_lds_fence();
    if (L.valid) {
      const uint32_t head = (uint32_t)((uintptr_t)(mask + (int64_t)b0 * A) & 15u) + (uint32_t)(L.j * A);
      const uint32_t o = head + (uint32_t)(N * L.r), q = o >> 5, s = o & 31u;
      atomicOr(&lds_mask[q], E << s);
      if (s + N > 32u) atomicOr(&lds_mask[q + 1], E >> (32u - s));
      if (L.r == 0 && swap) { const uint32_t o2 = head + P; atomicOr(&lds_mask[o2 >> 5], 1u << (o2 & 31u)); }
    }
    wave_lds_fence();
    emit_bytes<W * A, kStoreThrough>(lds_mask, lut, mask + (int64_t)b0 * A, (uint32_t)(nb * A), L.lane);
    wave_lds_fence();
  }
  if (obs) {
    // 4 bits per cell: mover's stone, opponent's stone, Black to move, swap legal; a row is N such nibbles
    const uint32_t mine = m.wtm ? wt : bk, theirs = m.wtm ? bk : wt;
    const uint32_t flags = (m.wtm ? 0u : 0x44444444u) | (swap ? 0x88888888u : 0u);
    const uint32_t lo = spread_every4(mine & 255u) | (spread_every4(theirs & 255u) << 1) | (L.valid ? flags : 0u);
    const uint32_t hi = (spread_every4(mine >> 8) | (spread_every4(theirs >> 8) << 1) | (L.valid ? flags : 0u)) & ((1u << (4 * (N - 8))) - 1u);
    if (L.lane < OBS_DW / 4) ((uint4*)lds_obs)[L.lane] = make_uint4(0u, 0u, 0u, 0u);
    wave_lds_fence();
    if (L.valid) {
      const uint32_t head = (uint32_t)((uintptr_t)(obs + (int64_t)b0 * OBS) & 15u) + (uint32_t)(L.j * OBS);
      const uint32_t o = head + (uint32_t)(4 * N * L.r), q = o >> 5, s = o & 31u;
      atomicOr(&lds_obs[q], lo << s);
      atomicOr(&lds_obs[q + 1], __funnelshift_l(lo, hi, s));
      const uint32_t t2 = __funnelshift_l(hi, 0u, s);
      if (t2) atomicOr(&lds_obs[q + 2], t2);
    }
    wave_lds_fence();
    emit_bytes<W * OBS, kStoreThrough>(lds_obs, lut, obs + (int64_t)b0 * OBS, (uint32_t)(nb * OBS), L.lane);
    wave_lds_fence();
  }
}

// Uniform random legal action (Sec. 4.1): the k-th legal action in ascending order, k = hash mod legal_count; the
// swap, when legal, is the last one; 0 when nothing is legal; -1 while the environment waits for its start time.
__device__ __forceinline__ int draw_action(const Lane& L, uint32_t E, bool swap, uint32_t seed, uint32_t t, bool wait) {
  const uint32_t cnt = __popc(E);
  uint32_t before = 0u, total = swap ? 1u : 0u;
#pragma unroll
  for (int k = 0; (1 << k) <= N; ++k) {
    const uint64_t m = __ballot((cnt >> k) & 1u);
    const uint32_t lo = (uint32_t)m & L.seglo, hi = (uint32_t)(m >> 32) & L.seghi;
    before += __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u)) << k;
    total += (uint32_t)(__popc(lo) + __popc(hi)) << k;
  }
  const uint32_t k = env_hash(seed, 0u, (uint32_t)L.b, t) % (total ? total : 1u);
  uint32_t n = k - before, w = E, pos = 0u;   // position of the (n+1)-th set bit of the row word by halving
#pragma unroll
  for (int width = 8; width >= 1; width >>= 1) {
    const uint32_t c = __popc(w & ((1u << width) - 1u));
    if (n >= c) { n -= c; w >>= width; pos += width; }
  }
  const bool mine = L.valid && k >= before && k < before + cnt;
  const uint64_t sel = __ballot(mine);
  const uint32_t slo = (uint32_t)sel & L.seglo, shi = (uint32_t)(sel >> 32) & L.seghi;
  const int src = slo ? __ffs(slo) - 1 : (shi ? 31 + __ffs(shi) : 0);
  const int pr = src - (L.j * STRIDE + 1);
  const int pc = __shfl((int)pos, src);
  if (wait) return -1;
  if (total == 0u) return 0;
  if (swap && k == total - 1u) return P;
  return pr * N + pc;
}

struct StepArgs {
  uint32_t* rows;            // [B][N] row words
  uint4* meta;               // [B]
  const int32_t* actions;    // [B]
  float* rew;                // [B][2]
  uint8_t* term;             // [B]
  uint8_t* mask;             // [B][A] or null
  uint8_t* obs;              // [B][OBS] or null
  int B;
  uint32_t seed;
  int auto_reset;
  uint32_t sample_seed, sample_t;
  const int32_t* start_t;    // nullable
  int32_t* next_actions;     // SAMPLE only
};

// What one ply did to a board (the same in every lane of the board)
struct Ply {
  bool skip, frozen, ended;
  float rew0, rew1;     // by player id; zero unless the ply ended the game
};

// One ply of every board of the wavefront, registers in, registers out (Fig. 2 "step"): a1 decode, a2 legality
// gate, a3 placement or swap, a4 winner test, a5 rewards / termination / auto-reset.
__device__ __forceinline__ Ply hex_ply(const Lane& L, uint32_t& bk, uint32_t& wt, Meta& m, int act, uint32_t seed, int auto_reset) {
  Ply out;
  const bool skip = act == -1 || !L.boardok;
  const bool frozen = !skip && m.term;        // finished earlier and not reset: nothing changes
  const bool live = !skip && !frozen;
  const uint32_t E = L.full & ~(bk | wt);
  const bool want_point = live && act >= 0 && act < P;
  const int row_of = (int)(__umul24((uint32_t)act & 127u, 745u) >> 13);   // act / 11 for 0 <= act < 128
  const int pr = want_point ? row_of : -100;
  const int pc = want_point ? act - row_of * N : 0;
  const uint32_t pbit = (L.valid && L.r == pr) ? (1u << pc) : 0u;
  const bool point_ok = want_point && board_any((E & pbit) != 0u, L.seglo, L.seghi);
  const bool swap_ok = live && act == P && m.steps == 1;
  const bool illegal_now = live && !point_ok && !swap_ok;
  const bool moved = point_ok || swap_ok;
  const int wtm = m.wtm;

  // swap rule: on the second turn the board holds Black's lone stone (r0,c0); it comes off and a white stone goes to (c0,r0)
  uint32_t swapped = 0u;
  if (__ballot(swap_ok) != 0ull) {   // once per game at most: keep it off the common path
    const uint64_t nz = __ballot(bk != 0u);
    const uint32_t zlo = (uint32_t)nz & L.seglo, zhi = (uint32_t)(nz >> 32) & L.seghi;
    const int src = zlo ? __ffs(zlo) - 1 : (zhi ? 31 + __ffs(zhi) : 0);
    const int r0 = src - (L.j * STRIDE + 1);
    const int c0 = __ffs(__shfl((int)bk, src)) - 1;
    swapped = (L.valid && L.r == c0 && r0 >= 0) ? (1u << (r0 & 15)) : 0u;
  }
  const uint32_t placed = swap_ok ? swapped : (point_ok ? pbit : 0u);
  if (swap_ok) { bk = 0u; wt = swapped; }
  else if (wtm) wt |= placed;
  else bk |= placed;

  // winner test: the chain of the new stone must touch both of the mover's sides
  const uint32_t S = wtm ? wt : bk;
  uint32_t F = placed;
  for (;;) {
    F |= hex_dilate(F) & S;
    F |= hex_dilate(F) & S;
    const uint32_t G = F | (hex_dilate(F) & S);
    const bool ch = G != F;
    F = G;
    if (__ballot(ch) == 0ull) break;
  }
  const bool side_a = wtm ? (F & 1u) != 0u : (F != 0u && L.r == 0);
  const bool side_b = wtm ? ((F >> (N - 1)) & 1u) != 0u : (F != 0u && L.r == N - 1);
  const bool hit_a = board_any(L.valid && side_a, L.seglo, L.seghi);
  const bool hit_b = board_any(L.valid && side_b, L.seglo, L.seghi);
  const bool won = moved && hit_a && hit_b;

  const int mover = wtm ? 1 - m.bp : m.bp;
  m.steps += moved ? 1 : 0;
  m.wtm = wtm ^ (moved ? 1 : 0);
  const bool ended = illegal_now || won;
  const float r_mover = won ? 1.f : (illegal_now ? -1.f : 0.f);
  const float r_other = won ? -1.f : (illegal_now ? 1.f : 0.f);
  m.illegal += illegal_now ? 1u : 0u;
  m.term = (m.term || ended) ? 1 : 0;
  if (ended && auto_reset) {   // Sec. 4.1: back to the initial state within the same ply
    m.episode += 1u;
    bk = 0u; wt = 0u;
    m.steps = 0; m.wtm = 0; m.term = 0;
    m.bp = (int)(env_hash(seed, 1u, (uint32_t)L.b, m.episode) & 1u);
  }
  out.skip = skip; out.frozen = frozen; out.ended = ended;
  out.rew0 = mover == 0 ? r_mover : r_other;
  out.rew1 = mover == 0 ? r_other : r_mover;
  return out;
}

// One launch = one ply of every game, then a6 legal mask, a7 observation, a8 state store, optionally the next draw.
template <bool SAMPLE>
__global__ void __launch_bounds__(64 * kWavesPerBlock) hex_step_kernel(StepArgs a) {
  __shared__ uint2 lut[256];
  __shared__ __align__(16) uint32_t lds_obs[kWavesPerBlock][OBS_DW];
  __shared__ uint32_t lds_mask[kWavesPerBlock][MASK_DW];
  const int wib = wave_in_block(), lane = threadIdx.x & 63;
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  const Lane L(wave, lane, a.B);
  const uint32_t word = L.valid ? a.rows[(size_t)L.b * N + L.r] : 0u;
  const uint4 mv = L.boardok ? a.meta[L.b] : make_uint4(0u, 0u, 0u, 0u);
  const int act = L.boardok ? a.actions[L.b] : -1;
  // loaded with the state: a load issued after the output stores would have to wait for them (one counter)
  const int32_t start_raw = (SAMPLE && a.start_t && L.boardok) ? a.start_t[L.b] : INT32_MIN;
  fill_spread_table(lut);
  if (wave * W >= a.B) return;
  const bool wait_start = (int64_t)a.sample_t < (int64_t)held_back(start_raw);

  uint32_t bk = word & 0xFFFFu, wt = word >> 16;
  Meta m = unpack_meta(mv);
  const Ply ply = hex_ply(L, bk, wt, m, act, a.seed, a.auto_reset);
  if (L.valid && L.r == 0 && !ply.skip) {
    *(float2*)(a.rew + 2 * (size_t)L.b) = make_float2(ply.rew0, ply.rew1);
    a.term[L.b] = (ply.ended || ply.frozen) ? 1 : 0;
    a.meta[L.b] = pack_meta(m);
  }
  const uint32_t word_new = bk | (wt << 16);
  if (L.valid && word_new != word) a.rows[(size_t)L.b * N + L.r] = word_new;

  emit_outputs(L, bk, wt, m, wave, a.B, a.mask, a.obs, lds_mask[wib], lds_obs[wib], lut);

  if (SAMPLE) {
    const int next = draw_action(L, L.full & ~(bk | wt), m.steps == 1, a.sample_seed, a.sample_t, wait_start);
    if (L.valid && L.r == 0) a.next_actions[L.b] = next;
  }
}

// ------------------------------------------------------------------------------------------------
// Board-per-lane mapping for very large batches: a lane holds a whole board as two 121-bit sets (cell p = 11*row + col
// is bit p of four dwords), a wavefront 64 boards.  Everything that the row-per-lane mapping pays once per 5 boards
// (decode, hash, draw, scalars, emission set-up) is paid once per 64; the flood runs until the slowest of the 64 boards
// has converged.  Same state layout, same outputs, same results; chosen by the launch code above a batch threshold.
// ------------------------------------------------------------------------------------------------
struct B128 {
  uint32_t w[4];
};
constexpr bool cell_in(int kind, int p) {   // 0: the board, 1: column 0, 2: column 10, 3: row 0, 4: row 10
  return kind == 0 ? true : kind == 1 ? p % N == 0 : kind == 2 ? p % N == N - 1 : kind == 3 ? p / N == 0 : p / N == N - 1;
}
constexpr uint32_t set_word(int kind, int i) {
  uint32_t v = 0u;
  for (int p = 32 * i; p < 32 * i + 32 && p < P; ++p)
    if (cell_in(kind, p)) v |= 1u << (p - 32 * i);
  return v;
}
template <int KIND>
__device__ __forceinline__ B128 set_of() { return B128{{set_word(KIND, 0), set_word(KIND, 1), set_word(KIND, 2), set_word(KIND, 3)}}; }

__device__ __forceinline__ B128 b_or(B128 a, B128 b) { return B128{{a.w[0] | b.w[0], a.w[1] | b.w[1], a.w[2] | b.w[2], a.w[3] | b.w[3]}}; }
__device__ __forceinline__ B128 b_and(B128 a, B128 b) { return B128{{a.w[0] & b.w[0], a.w[1] & b.w[1], a.w[2] & b.w[2], a.w[3] & b.w[3]}}; }
__device__ __forceinline__ B128 b_andn(B128 a, B128 b) { return B128{{a.w[0] & ~b.w[0], a.w[1] & ~b.w[1], a.w[2] & ~b.w[2], a.w[3] & ~b.w[3]}}; }
__device__ __forceinline__ bool b_any(B128 a) { return (a.w[0] | a.w[1] | a.w[2] | a.w[3]) != 0u; }
__device__ __forceinline__ bool b_ne(B128 a, B128 b) { return ((a.w[0] ^ b.w[0]) | (a.w[1] ^ b.w[1]) | (a.w[2] ^ b.w[2]) | (a.w[3] ^ b.w[3])) != 0u; }
__device__ __forceinline__ B128 b_bit(int p, bool on) {   // the set {p} (empty when !on)
  const uint32_t bit = on ? 1u << (p & 31) : 0u;
  const int i = p >> 5;
  return B128{{i == 0 ? bit : 0u, i == 1 ? bit : 0u, i == 2 ? bit : 0u, i == 3 ? bit : 0u}};
}
template <int K>
__device__ __forceinline__ B128 b_up(B128 x) {     // cell p -> p + K
  return B128{{x.w[0] << K, __builtin_amdgcn_alignbit(x.w[1], x.w[0], 32 - K), __builtin_amdgcn_alignbit(x.w[2], x.w[1], 32 - K),
               __builtin_amdgcn_alignbit(x.w[3], x.w[2], 32 - K)}};
}
template <int K>
__device__ __forceinline__ B128 b_down(B128 x) {   // cell p -> p - K
  return B128{{__builtin_amdgcn_alignbit(x.w[1], x.w[0], K), __builtin_amdgcn_alignbit(x.w[2], x.w[1], K), __builtin_amdgcn_alignbit(x.w[3], x.w[2], K),
               x.w[3] >> K}};
}
// all cells touching the set x (the same six neighbours as hex_dilate); bits beyond cell 120 may be set
__device__ __forceinline__ B128 dilate128(B128 x) {
  const B128 not_last = b_andn(x, set_of<2>()), not_first = b_andn(x, set_of<1>());
  return b_or(b_or(b_or(b_up<1>(not_last), b_down<N - 1>(not_last)), b_or(b_down<1>(not_first), b_up<N - 1>(not_first))), b_or(b_down<N>(x), b_up<N>(x)));
}

// bit i of x (x < 256) -> bit 4i, from a table in LDS
__device__ __forceinline__ void fill_spread4_table(uint32_t* lut4) {
  for (uint32_t x = threadIdx.x; x < 256u; x += blockDim.x) lut4[x] = spread_every4(x);
}

// Puts the ND-dword bit string S at bit offset o of an LDS bit stream: a left shift by 1..32 from dword (o-1)/32 on, so
// that every stream dword is one funnel shift of two neighbours of S.  Stream dwords OWN_LO..OWN_HI (relative to the
// first) hold bits of this string only whatever o is and are stored plainly; the others are OR-ed in.
template <int ND, int OWN_LO, int OWN_HI>
__device__ __forceinline__ void stream_put(uint32_t* stream, const uint32_t (&S)[ND], uint32_t o) {
  const uint32_t u1 = (o + 31u) & 31u;
  uint32_t* reg = stream + ((int32_t)(o - 1u - u1) >> 5);   // dword -1 only when o = 0, and then nothing is written there
  const uint32_t sh = 31u - u1;
  const uint32_t t0 = __builtin_amdgcn_alignbit(S[0], 0u, sh);
  if (t0) atomicOr(&reg[0], t0);
#pragma unroll
  for (int i = 1; i <= ND; ++i) {
    const uint32_t t = __builtin_amdgcn_alignbit(i < ND ? S[i] : 0u, S[i - 1], sh);
    if (i >= OWN_LO && i <= OWN_HI) reg[i] = t;
    else if (t) atomicOr(&reg[i], t);
  }
}

constexpr int LANE_MASK_DW = ((15 + 64 * A + 31) / 32 + 3) / 4 * 4;   // LDS dwords of a wavefront's streams: 64 boards
constexpr int LANE_OBS_DW = ((15 + 64 * OBS + 31) / 32 + 3) / 4 * 4;

// rows (black bits 0-10, white bits 16-26 of one dword per row) <-> the two sets of a board
__device__ __forceinline__ void rows_to_sets(const uint32_t (&row)[N], B128& bk, B128& wt) {
  bk = B128{{0u, 0u, 0u, 0u}}; wt = bk;
#pragma unroll
  for (int r = 0; r < N; ++r) {
    const int i = (N * r) >> 5, s = (N * r) & 31;
    const uint32_t kb = row[r] & FULL, kw = (row[r] >> 16) & FULL;
    bk.w[i] |= kb << s; wt.w[i] |= kw << s;
    if (s + N > 32) { bk.w[i + 1] |= kb >> (32 - s); wt.w[i + 1] |= kw >> (32 - s); }
  }
}
__device__ __forceinline__ void store_sets_as_rows(uint32_t* rows_of_board, const B128& bk, const B128& wt) {
#pragma unroll
  for (int r = 0; r < N; ++r) {
    const int i = (N * r) >> 5, s = (N * r) & 31;
    uint32_t kb = bk.w[i] >> s, kw = wt.w[i] >> s;
    if (s + N > 32) { kb |= bk.w[i + 1] << (32 - s); kw |= wt.w[i + 1] << (32 - s); }
    rows_of_board[r] = (kb & FULL) | ((kw & FULL) << 16);
  }
}

struct LanePly {          // what one ply did to this lane's board
  bool skip, frozen, ended, point_ok, swap_ok, reset;
  float rew0, rew1;       // by player id; zero unless the ply ended the game
};

// a1-a5 for this lane's board (Fig. 2 "step"): decode, legality gate, placement or swap, winner test, rewards /
// termination / auto-reset.  Every lane of the wavefront must call it (the flood's convergence test is a ballot).
__device__ __forceinline__ LanePly lane_ply(B128& bk, B128& wt, Meta& m, int act, bool ok, int b, uint32_t seed, int auto_reset) {
  LanePly out;
  const bool skip = act == -1 || !ok;
  const bool frozen = !skip && m.term;
  const bool live = !skip && !frozen;
  const B128 E0 = b_andn(set_of<0>(), b_or(bk, wt));
  const bool want_point = live && act >= 0 && act < P;
  const B128 pbit = b_bit(want_point ? act : 0, want_point);
  const bool point_ok = want_point && b_any(b_and(E0, pbit));
  const bool swap_ok = live && act == P && m.steps == 1;
  const bool illegal_now = live && !point_ok && !swap_ok;
  const bool moved = point_ok || swap_ok;
  const int wtm = m.wtm;
  B128 placed = pbit;
  if (!point_ok) placed = B128{{0u, 0u, 0u, 0u}};
  if (swap_ok) {   // Black's lone stone (r0,c0) comes off, a white stone goes to (c0,r0); once per game at most
    const int p0 = bk.w[0] ? __ffs(bk.w[0]) - 1 : bk.w[1] ? 31 + __ffs(bk.w[1]) : bk.w[2] ? 63 + __ffs(bk.w[2]) : 95 + __ffs(bk.w[3]);
    const int r0 = p0 / N, c0 = p0 - r0 * N;
    placed = b_bit(c0 * N + r0, true);
    bk = B128{{0u, 0u, 0u, 0u}}; wt = placed;
  } else if (wtm) {
    wt = b_or(wt, placed);
  } else {
    bk = b_or(bk, placed);
  }
  // winner test: the chain of the new stone must touch both of the mover's sides
  const B128 S = wtm ? wt : bk;
  B128 F = placed;
  for (;;) {
    F = b_or(F, b_and(dilate128(F), S));
    const B128 G = b_or(F, b_and(dilate128(F), S));
    const bool ch = b_ne(G, F);
    F = G;
    if (__ballot(ch) == 0ull) break;
  }
  const bool hit_a = b_any(b_and(F, wtm ? set_of<1>() : set_of<3>()));
  const bool hit_b = b_any(b_and(F, wtm ? set_of<2>() : set_of<4>()));
  const bool won = moved && hit_a && hit_b;

  const int mover = wtm ? 1 - m.bp : m.bp;
  m.steps += moved ? 1 : 0;
  m.wtm = wtm ^ (moved ? 1 : 0);
  const bool ended = illegal_now || won;
  const float r_mover = won ? 1.f : (illegal_now ? -1.f : 0.f);
  const float r_other = won ? -1.f : (illegal_now ? 1.f : 0.f);
  m.illegal += illegal_now ? 1u : 0u;
  m.term = (m.term || ended) ? 1 : 0;
  const bool reset = ended && auto_reset;
  if (reset) {   // Sec. 4.1: back to the initial state within the same ply
    m.episode += 1u;
    bk = B128{{0u, 0u, 0u, 0u}}; wt = bk;
    m.steps = 0; m.wtm = 0; m.term = 0;
    m.bp = (int)(env_hash(seed, 1u, (uint32_t)b, m.episode) & 1u);
  }
  out.skip = skip; out.frozen = frozen; out.ended = ended; out.point_ok = point_ok; out.swap_ok = swap_ok; out.reset = reset;
  out.rew0 = mover == 0 ? r_mover : r_other;
  out.rew1 = mover == 0 ? r_other : r_mover;
  return out;
}

// the legal actions of the position as a 122-bit set (bit 121 = the swap)
__device__ __forceinline__ B128 lane_legal(const B128& bk, const B128& wt, const Meta& m) {
  B128 legal = b_andn(set_of<0>(), b_or(bk, wt));
  if (m.steps == 1) legal.w[3] |= 1u << (P - 96);
  return legal;
}

// a6 / a7: legal mask [122] and observation [11][11][4] of the 64 boards of the wavefront (nb real ones from board b0 on)
__device__ __forceinline__ void lane_emit(const B128& bk, const B128& wt, const Meta& m, const B128& legal, bool ok, int lane, int b0, int nb,
                                          uint8_t* mask, uint8_t* obs, uint32_t* lds_mask, uint32_t* lds_obs, const uint2* lut, const uint32_t* lut4) {
  {
    uint4* z = (uint4*)lds_obs;
#pragma unroll
    for (int i = 0; i < (LANE_OBS_DW / 4 + 63) / 64; ++i)
      if (i * 64 + lane < LANE_OBS_DW / 4) z[i * 64 + lane] = make_uint4(0u, 0u, 0u, 0u);
    if (lane < LANE_MASK_DW / 4) ((uint4*)lds_mask)[lane] = make_uint4(0u, 0u, 0u, 0u);
    static_assert(LANE_MASK_DW / 4 <= 64, "the mask stream is cleared by one store per lane");
  }
  wave_lds_fence();
  if (mask && ok) {
    const uint32_t head = (uint32_t)((uintptr_t)(mask + (size_t)b0 * A) & 15u);
    stream_put<4, 1, 2>(lds_mask, legal.w, head + (uint32_t)(A * lane));
  }
  if (obs && ok) {
    // 4 bits per cell: mover's stone, opponent's stone, Black to move, swap legal
    const B128 mine = m.wtm ? wt : bk, theirs = m.wtm ? bk : wt;
    const uint32_t flags = (m.wtm ? 0u : 0x44444444u) | (m.steps == 1 ? 0x88888888u : 0u);
    uint32_t O[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const uint32_t mb = (mine.w[k >> 2] >> (8 * (k & 3))) & 255u, tb = (theirs.w[k >> 2] >> (8 * (k & 3))) & 255u;
      O[k] = lut4[mb] | (lut4[tb] << 1) | (k < 15 ? flags : (flags & 0xFu));
    }
    const uint32_t head = (uint32_t)((uintptr_t)(obs + (size_t)b0 * OBS) & 15u);
    stream_put<16, 1, 14>(lds_obs, O, head + (uint32_t)(OBS * lane));
  }
  wave_lds_fence();
  if (mask) emit_bytes<64 * A, kStoreThrough>(lds_mask, lut, mask + (size_t)b0 * A, (uint32_t)(nb * A), lane);
  if (obs) emit_bytes<64 * OBS, kStoreThrough>(lds_obs, lut, obs + (size_t)b0 * OBS, (uint32_t)(nb * OBS), lane);
  wave_lds_fence();
}

// the uniform random legal action of this lane's board: the k-th set bit of the legal set, k = hash mod count
__device__ __forceinline__ int lane_draw(const B128& legal, uint32_t seed, uint32_t b, uint32_t t, bool wait) {
  const uint32_t c0 = __popc(legal.w[0]), c1 = __popc(legal.w[1]), c2 = __popc(legal.w[2]), c3 = __popc(legal.w[3]);
  const uint32_t total = c0 + c1 + c2 + c3;
  uint32_t k = env_hash(seed, 0u, b, t) % (total ? total : 1u);
  uint32_t w = legal.w[0], base = 0u;
  if (k >= c0) { k -= c0; w = legal.w[1]; base = 32u;
    if (k >= c1) { k -= c1; w = legal.w[2]; base = 64u;
      if (k >= c2) { k -= c2; w = legal.w[3]; base = 96u; } } }
  uint32_t pos = 0u;
#pragma unroll
  for (int width = 16; width >= 1; width >>= 1) {
    const uint32_t c = __popc(w & ((1u << width) - 1u));
    if (k >= c) { k -= c; w >>= width; pos += width; }
  }
  return wait ? -1 : (total == 0u ? 0 : (int)(base + pos));
}

template <bool SAMPLE>
__global__ void __launch_bounds__(64 * kWavesPerBlock) hex_step_lane_kernel(StepArgs a) {
  __shared__ uint2 lut[256];
  __shared__ uint32_t lut4[256];
  __shared__ __align__(16) uint32_t lds_obs[kWavesPerBlock][LANE_OBS_DW];
  __shared__ __align__(16) uint32_t lds_mask[kWavesPerBlock][LANE_MASK_DW];
  const int wib = wave_in_block(), lane = threadIdx.x & 63;
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  const int b0 = wave * 64;                 // first board of the wavefront
  const int b = b0 + lane;
  const bool ok = b < a.B;
  // state: 11 row words, the scalar record, the action
  uint32_t row[N];
#pragma unroll
  for (int r = 0; r < N; ++r) row[r] = ok ? a.rows[(size_t)b * N + r] : 0u;
  const uint4 mv = ok ? a.meta[b] : make_uint4(0u, 0u, 0u, 0u);
  const int act = ok ? a.actions[b] : -1;
  // loaded with the state: a load issued after the output stores would have to wait for them (one counter)
  const int32_t start_raw = (SAMPLE && a.start_t && ok) ? a.start_t[b] : INT32_MIN;
  fill_spread4_table(lut4);
  fill_spread_table(lut);                   // ends with the block's only barrier (nothing loaded above is looked at before it)
  if (b0 >= a.B) return;
  const bool wait_start = (int64_t)a.sample_t < (int64_t)held_back(start_raw);
  const int nb = a.B - b0 < 64 ? a.B - b0 : 64;
  Meta m = unpack_meta(mv);
  B128 bk, wt;
  rows_to_sets(row, bk, wt);
  const int wtm = m.wtm;
  const LanePly ply = lane_ply(bk, wt, m, act, ok, b, a.seed, a.auto_reset);
  if (!ply.skip) {
    *(float2*)(a.rew + 2 * (size_t)b) = make_float2(ply.rew0, ply.rew1);
    a.term[b] = (ply.ended || ply.frozen) ? 1 : 0;
    a.meta[b] = pack_meta(m);
    // a8: state store.  A placed stone changes one bit of one row word; a swap or a reset rewrites the board.
    if (ply.swap_ok || ply.reset) {
      store_sets_as_rows(a.rows + (size_t)b * N, bk, wt);
    } else if (ply.point_ok) {
      const int pr = (int)(__umul24((uint32_t)act, 745u) >> 13);   // act / 11 for 0 <= act < 128
      atomicOr(&a.rows[(size_t)b * N + pr], (1u << (act - pr * N)) << (wtm ? 16 : 0));
    }
  }
  const B128 legal = lane_legal(bk, wt, m);
  lane_emit(bk, wt, m, legal, ok, lane, b0, nb, a.mask, a.obs, lds_mask[wib], lds_obs[wib], lut, lut4);
  if (SAMPLE) {
    const int next = lane_draw(legal, a.sample_seed, (uint32_t)b, a.sample_t, wait_start);
    if (ok) a.next_actions[b] = next;
  }
}

// `steps` plies of uniform random legal play in one launch (Sec. 2: all-on-device loops; Sec. 4.1: random policy with
// auto-reset).  The state stays in registers; the outputs of ply i go to slice (i mod slices) of the caller's buffers.
struct RolloutArgs {
  uint32_t* rows;
  uint4* meta;
  int B;
  uint32_t seed_env;       // the handle's seed (seat draws)
  int auto_reset;
  int steps, slices;
  uint32_t seed, t0;       // sampler
  const int32_t* start_t;  // nullable
  int32_t* actions;        // [slices][B] or null
  float* rew;              // [slices][B][2] or null
  uint8_t* term;           // [slices][B] or null
  uint8_t* mask;           // [slices][B][A] or null
  uint8_t* obs;            // [slices][B][OBS] or null
};

__global__ void __launch_bounds__(64 * kWavesPerBlock) hex_rollout_kernel(RolloutArgs a) {
  __shared__ uint2 lut[256];
  __shared__ __align__(16) uint32_t lds_obs[kWavesPerBlock][OBS_DW];
  __shared__ uint32_t lds_mask[kWavesPerBlock][MASK_DW];
  fill_spread_table(lut);
  const int wib = wave_in_block(), lane = threadIdx.x & 63;
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  if (wave * W >= a.B) return;
  const Lane L(wave, lane, a.B);
  const uint32_t word = L.valid ? a.rows[(size_t)L.b * N + L.r] : 0u;
  uint32_t bk = word & 0xFFFFu, wt = word >> 16;
  Meta m = unpack_meta(L.boardok ? a.meta[L.b] : make_uint4(0u, 0u, 0u, 0u));
  const int64_t start = (L.boardok && a.start_t) ? (int64_t)a.start_t[L.b] : INT64_MIN;
  int slice = 0;
  for (int i = 0; i < a.steps; ++i) {   // the same trip count for every wavefront
    const uint32_t t = a.t0 + (uint32_t)i;
    const bool wait = (int64_t)t < start;
    const int act = draw_action(L, L.full & ~(bk | wt), m.steps == 1, a.seed, t, wait);
    const Ply ply = hex_ply(L, bk, wt, m, L.boardok ? act : -1, a.seed_env, a.auto_reset);
    const size_t sb = (size_t)slice * a.B;
    if (L.valid && L.r == 0) {
      const size_t e = sb + L.b;
      if (a.actions) a.actions[e] = act;
      // a waiting environment reports what a skipped step leaves behind at the start: zeros
      if (a.rew) *(float2*)(a.rew + 2 * e) = ply.skip ? make_float2(0.f, 0.f) : make_float2(ply.rew0, ply.rew1);
      if (a.term) a.term[e] = (uint8_t)((!ply.skip && (ply.ended || ply.frozen)) ? 1 : 0);
    }
    emit_outputs(L, bk, wt, m, wave, a.B, a.mask ? a.mask + sb * A : nullptr, a.obs ? a.obs + sb * OBS : nullptr, lds_mask[wib], lds_obs[wib], lut);
    slice = slice + 1 == a.slices ? 0 : slice + 1;
  }
  if (L.valid) a.rows[(size_t)L.b * N + L.r] = bk | (wt << 16);
  if (L.valid && L.r == 0) a.meta[L.b] = pack_meta(m);
}

// the same with a board per lane (very large batches): state of 64 boards in the registers of one wavefront
__global__ void __launch_bounds__(64 * kWavesPerBlock) hex_rollout_lane_kernel(RolloutArgs a) {
  __shared__ uint2 lut[256];
  __shared__ uint32_t lut4[256];
  __shared__ __align__(16) uint32_t lds_obs[kWavesPerBlock][LANE_OBS_DW];
  __shared__ __align__(16) uint32_t lds_mask[kWavesPerBlock][LANE_MASK_DW];
  fill_spread4_table(lut4);
  fill_spread_table(lut);
  const int wib = wave_in_block(), lane = threadIdx.x & 63;
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  const int b0 = wave * 64;
  if (b0 >= a.B) return;
  const int b = b0 + lane;
  const bool ok = b < a.B;
  const int nb = a.B - b0 < 64 ? a.B - b0 : 64;
  uint32_t row[N];
#pragma unroll
  for (int r = 0; r < N; ++r) row[r] = ok ? a.rows[(size_t)b * N + r] : 0u;
  Meta m = unpack_meta(ok ? a.meta[b] : make_uint4(0u, 0u, 0u, 0u));
  const int64_t start = (ok && a.start_t) ? (int64_t)a.start_t[b] : INT64_MIN;
  B128 bk, wt;
  rows_to_sets(row, bk, wt);
  B128 legal = lane_legal(bk, wt, m);
  int slice = 0;
  for (int i = 0; i < a.steps; ++i) {   // the same trip count for every wavefront
    const uint32_t t = a.t0 + (uint32_t)i;
    const bool wait = (int64_t)t < start;
    const int act = ok ? lane_draw(legal, a.seed, (uint32_t)b, t, wait) : -1;
    const LanePly ply = lane_ply(bk, wt, m, act, ok, b, a.seed_env, a.auto_reset);
    legal = lane_legal(bk, wt, m);
    const size_t sb = (size_t)slice * a.B;
    if (ok) {
      const size_t e = sb + b;
      if (a.actions) a.actions[e] = act;
      if (a.rew) *(float2*)(a.rew + 2 * e) = ply.skip ? make_float2(0.f, 0.f) : make_float2(ply.rew0, ply.rew1);
      if (a.term) a.term[e] = (uint8_t)((!ply.skip && (ply.ended || ply.frozen)) ? 1 : 0);
    }
    lane_emit(bk, wt, m, legal, ok, lane, b0, nb, a.mask ? a.mask + sb * A : nullptr, a.obs ? a.obs + sb * OBS : nullptr, lds_mask[wib], lds_obs[wib], lut,
              lut4);
    slice = slice + 1 == a.slices ? 0 : slice + 1;
  }
  if (ok) {
    store_sets_as_rows(a.rows + (size_t)b * N, bk, wt);
    a.meta[b] = pack_meta(m);
  }
}

__global__ void __launch_bounds__(64 * kWavesPerBlock) hex_emit_kernel(const uint32_t* rows, const uint4* meta, int B, uint8_t* mask, uint8_t* obs) {
  __shared__ uint2 lut[256];
  __shared__ __align__(16) uint32_t lds_obs[kWavesPerBlock][OBS_DW];
  __shared__ uint32_t lds_mask[kWavesPerBlock][MASK_DW];
  const int wib = wave_in_block(), lane = threadIdx.x & 63;
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  const Lane L(wave, lane, B);
  const uint32_t word = L.valid ? rows[(size_t)L.b * N + L.r] : 0u;
  const Meta m = unpack_meta(L.boardok ? meta[L.b] : make_uint4(0u, 0u, 0u, 0u));
  fill_spread_table(lut);
  if (wave * W >= B) return;
  emit_outputs(L, word & 0xFFFFu, word >> 16, m, wave, B, mask, obs, lds_mask[wib], lds_obs[wib], lut);
}

__global__ void __launch_bounds__(64 * kWavesPerBlock) hex_random_actions_kernel(const uint32_t* rows, const uint4* meta, int B, uint32_t seed, uint32_t t,
                                                                                const int32_t* start_t, int32_t* actions) {
  const int wib = wave_in_block(), lane = threadIdx.x & 63;
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  if (wave * W >= B) return;
  const Lane L(wave, lane, B);
  const uint32_t word = L.valid ? rows[(size_t)L.b * N + L.r] : 0u;
  const Meta m = unpack_meta(L.boardok ? meta[L.b] : make_uint4(0u, 0u, 0u, 0u));
  const bool wait = start_t && L.boardok && (int64_t)t < (int64_t)start_t[L.b];
  const int next = draw_action(L, L.full & ~((word & 0xFFFFu) | (word >> 16)), m.steps == 1, seed, t, wait);
  if (L.valid && L.r == 0) actions[L.b] = next;
}

// first = 1: episode 0 (init); first = 0: the next episode of every game
__global__ void hex_reset_kernel(uint32_t* rows, uint4* meta, float* rew, uint8_t* term, int B, uint32_t seed, int first) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)B * N) return;
  rows[i] = 0u;
  if (i < (size_t)B) {
    Meta m;
    m.steps = 0; m.wtm = 0; m.term = 0;
    m.episode = first ? 0u : meta[i].y + 1u;
    m.illegal = first ? 0u : meta[i].z;
    m.bp = (int)(env_hash(seed, 1u, (uint32_t)i, m.episode) & 1u);
    meta[i] = pack_meta(m);
    rew[2 * i] = 0.f; rew[2 * i + 1] = 0.f;
    term[i] = 0;
  }
}

__global__ void hex_current_player_kernel(const uint4* meta, int B, uint8_t* dst) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const Meta m = unpack_meta(meta[b]);
  dst[b] = (uint8_t)(m.wtm ? 1 - m.bp : m.bp);
}

struct Canon {
  int8_t* board; int8_t* to_play; int32_t* steps; uint8_t* terminated; uint8_t* black_player; uint32_t* episode; uint32_t* illegal;
};

__global__ void hex_export_kernel(const uint32_t* rows, const uint4* meta, int B, Canon c) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one thread per row
  if (i >= (size_t)B * N) return;
  if (c.board) {
    const uint32_t w = rows[i];
    for (int col = 0; col < N; ++col) c.board[i * N + col] = (int8_t)(((w >> col) & 1u) ? 1 : (((w >> (16 + col)) & 1u) ? -1 : 0));
  }
  if (i < (size_t)B) {
    const Meta m = unpack_meta(meta[i]);
    if (c.to_play) c.to_play[i] = (int8_t)(m.wtm ? -1 : 1);
    if (c.steps) c.steps[i] = m.steps;
    if (c.terminated) c.terminated[i] = (uint8_t)m.term;
    if (c.black_player) c.black_player[i] = (uint8_t)m.bp;
    if (c.episode) c.episode[i] = m.episode;
    if (c.illegal) c.illegal[i] = m.illegal;
  }
}

__global__ void hex_import_kernel(uint32_t* rows, uint4* meta, float* rew, uint8_t* term, int B, Canon c) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)B * N) return;
  uint32_t w = 0u;
  for (int col = 0; col < N; ++col) {
    const int8_t v = c.board[i * N + col];
    w |= (v > 0 ? 1u : 0u) << col;
    w |= (v < 0 ? 1u : 0u) << (16 + col);
  }
  rows[i] = w;
  if (i < (size_t)B) {
    Meta m;
    m.steps = c.steps[i] & 0xFF; m.wtm = c.to_play[i] < 0 ? 1 : 0; m.term = c.terminated[i] ? 1 : 0; m.bp = c.black_player[i] & 1;
    m.episode = c.episode[i]; m.illegal = meta[i].z;
    meta[i] = pack_meta(m);
    rew[2 * i] = 0.f; rew[2 * i + 1] = 0.f;
    term[i] = (uint8_t)m.term;
  }
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t state_layout(int B, size_t* off_meta, size_t* off_rew, size_t* off_term) {
  size_t o = align_up((size_t)B * N * sizeof(uint32_t), 256);
  if (off_meta) *off_meta = o;
  o += align_up((size_t)B * sizeof(uint4), 256);
  if (off_rew) *off_rew = o;
  o += align_up((size_t)B * 2 * sizeof(float), 256);
  if (off_term) *off_term = o;
  o += align_up((size_t)B, 256);
  return o;
}

}  // namespace

struct pgxhex_ctx {
  int B;
  uint32_t seed;
  int auto_reset;
  hipStream_t stream;
  uint32_t* rows;
  uint4* meta;
  float* rew_int;
  uint8_t* term_int;
  uint8_t* mask_out;
  uint8_t* obs_out;
  float* rew_out;
  uint8_t* term_out;
  int mapping;   // 0: automatic, 1: a board row per lane, 2: a board per lane
};

namespace {

// From this many games on the kernels hold a board per lane; below, a board row per lane, which needs far fewer games
// to fill the machine.  Measured per ply, a board row per lane against a board per lane: one launch per ply 6.7 / 8.2 us
// at 16384 games, 9.4 / 8.5 us at 32768, 14.1 / 11.0 us at 65536, 38.5 / 29.4 us at 262144; the rollout kernel
// 4.4 / 4.95 us at 16384 games, 7.0 / 5.0 us at 32768, 12.5 / 5.5 us at 65536.
constexpr int kLaneMappingFromStep = 28672, kLaneMappingFromRollout = 20480;
bool board_per_lane(const pgxhex_ctx* h, bool rollout = false) {
  return h->mapping == 2 || (h->mapping == 0 && h->B >= (rollout ? kLaneMappingFromRollout : kLaneMappingFromStep));
}

// grids of the board kernels: a multiple of 8 blocks (piece_of_block)
unsigned blocks_for(int B) {
  const unsigned waves = (unsigned)((B + W - 1) / W);
  return ((waves + kWavesPerBlock - 1) / kWavesPerBlock + 7u) & ~7u;
}
unsigned lane_blocks_for(int B) { return ((unsigned)((B + 64 * kWavesPerBlock - 1) / (64 * kWavesPerBlock)) + 7u) & ~7u; }
unsigned row_blocks(int B) { return (unsigned)(((size_t)B * N + 255) / 256); }

int launch_emit(pgxhex_ctx* h, uint8_t* mask, uint8_t* obs) {
  hipLaunchKernelGGL(hex_emit_kernel, dim3(blocks_for(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, h->rows, h->meta, h->B, mask, obs);
  HIPCHK(hipGetLastError());
  return PGXHEX_OK;
}

int launch_reset(pgxhex_ctx* h, int first) {
  hipLaunchKernelGGL(hex_reset_kernel, dim3(row_blocks(h->B)), dim3(256), 0, h->stream, h->rows, h->meta, h->rew_out, h->term_out, h->B, h->seed, first);
  HIPCHK(hipGetLastError());
  return PGXHEX_OK;
}

int launch_step(pgxhex_ctx* h, const int32_t* actions, bool sample, uint32_t seed, uint32_t t, const int32_t* start_t, int32_t* next) {
  StepArgs a;
  a.rows = h->rows; a.meta = h->meta; a.actions = actions; a.rew = h->rew_out; a.term = h->term_out; a.mask = h->mask_out; a.obs = h->obs_out;
  a.B = h->B; a.seed = h->seed; a.auto_reset = h->auto_reset;
  a.sample_seed = seed; a.sample_t = t; a.start_t = start_t; a.next_actions = next;
  if (board_per_lane(h)) {
    const dim3 grid(lane_blocks_for(h->B));
    if (sample) hipLaunchKernelGGL(hex_step_lane_kernel<true>, grid, dim3(64 * kWavesPerBlock), 0, h->stream, a);
    else hipLaunchKernelGGL(hex_step_lane_kernel<false>, grid, dim3(64 * kWavesPerBlock), 0, h->stream, a);
  } else if (sample) hipLaunchKernelGGL(hex_step_kernel<true>, dim3(blocks_for(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, a);
  else hipLaunchKernelGGL(hex_step_kernel<false>, dim3(blocks_for(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, a);
  HIPCHK(hipGetLastError());
  return PGXHEX_OK;
}

}  // namespace

extern "C" {

size_t pgxhex_state_bytes(int32_t batch) { return batch > 0 ? state_layout(batch, nullptr, nullptr, nullptr) : 0; }

int32_t pgxhex_boards_per_wavefront(void) { return W; }

int pgxhex_init(pgxhex_t* out, int32_t batch, uint32_t seed, const pgxhex_opts* opts, void* state_dev, size_t state_bytes) {
  if (!out) return PGXHEX_EINVAL;
  *out = nullptr;
  if (batch <= 0 || !state_dev || ((uintptr_t)state_dev & 255u) != 0) return PGXHEX_EINVAL;
  size_t off_meta, off_rew, off_term;
  if (state_bytes < state_layout(batch, &off_meta, &off_rew, &off_term)) return PGXHEX_EINVAL;
  pgxhex_ctx* h = (pgxhex_ctx*)calloc(1, sizeof(pgxhex_ctx));
  if (!h) return PGXHEX_ENOMEM;
  h->B = batch; h->seed = seed;
  h->auto_reset = (opts && opts->auto_reset) ? 1 : 0;
  h->stream = opts ? (hipStream_t)opts->stream : nullptr;
  uint8_t* base = (uint8_t*)state_dev;
  h->rows = (uint32_t*)base;
  h->meta = (uint4*)(base + off_meta);
  h->rew_int = (float*)(base + off_rew);
  h->term_int = base + off_term;
  h->rew_out = h->rew_int; h->term_out = h->term_int;
  int rc = launch_reset(h, 1);
  if (rc == PGXHEX_OK) {
    hipError_t e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) { g_last_hip = (int)e; rc = PGXHEX_EHIP; }
  }
  if (rc != PGXHEX_OK) { free(h); return rc; }
  *out = h;
  return PGXHEX_OK;
}

int pgxhex_destroy(pgxhex_t h) {
  if (!h) return PGXHEX_EINVAL;
  free(h);
  return PGXHEX_OK;
}

int pgxhex_reset(pgxhex_t h) {
  if (!h) return PGXHEX_EINVAL;
  int rc = launch_reset(h, 0);
  if (rc != PGXHEX_OK) return rc;
  if (h->mask_out || h->obs_out) return launch_emit(h, h->mask_out, h->obs_out);
  return PGXHEX_OK;
}

int pgxhex_bind_outputs(pgxhex_t h, uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev) {
  if (!h) return PGXHEX_EINVAL;
  float* new_rew = rewards_dev ? rewards_dev : h->rew_int;
  uint8_t* new_term = terminated_dev ? terminated_dev : h->term_int;
  if (new_rew != h->rew_out) HIPCHK(hipMemcpyAsync(new_rew, h->rew_out, (size_t)h->B * 2 * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
  if (new_term != h->term_out) HIPCHK(hipMemcpyAsync(new_term, h->term_out, (size_t)h->B, hipMemcpyDeviceToDevice, h->stream));
  h->rew_out = new_rew; h->term_out = new_term;
  h->mask_out = mask_dev; h->obs_out = obs_dev;
  if (mask_dev || obs_dev) return launch_emit(h, mask_dev, obs_dev);
  return PGXHEX_OK;
}

int pgxhex_set_output_buffers(pgxhex_t h, uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev) {
  if (!h) return PGXHEX_EINVAL;
  h->mask_out = mask_dev; h->obs_out = obs_dev;
  h->rew_out = rewards_dev ? rewards_dev : h->rew_int;
  h->term_out = terminated_dev ? terminated_dev : h->term_int;
  return PGXHEX_OK;
}

int pgxhex_step(pgxhex_t h, const int32_t* actions_dev) {
  if (!h || !actions_dev) return PGXHEX_EINVAL;
  return launch_step(h, actions_dev, false, 0u, 0u, nullptr, nullptr);
}

int pgxhex_step_sample(pgxhex_t h, const int32_t* actions_dev, uint32_t seed, uint32_t t, const int32_t* start_t_dev, int32_t* next_actions_dev) {
  if (!h || !actions_dev || !next_actions_dev || next_actions_dev == actions_dev) return PGXHEX_EINVAL;
  return launch_step(h, actions_dev, true, seed, t, start_t_dev, next_actions_dev);
}

int pgxhex_rollout(pgxhex_t h, int32_t steps, int32_t slices, uint32_t seed, uint32_t t0, const int32_t* start_t_dev, int32_t* actions_dev,
                   float* rewards_dev, uint8_t* terminated_dev, uint8_t* mask_dev, uint8_t* obs_dev) {
  if (!h || steps < 0 || slices < 1) return PGXHEX_EINVAL;
  if (steps == 0) return PGXHEX_OK;
  RolloutArgs a;
  a.rows = h->rows; a.meta = h->meta; a.B = h->B; a.seed_env = h->seed; a.auto_reset = h->auto_reset;
  a.steps = steps; a.slices = slices; a.seed = seed; a.t0 = t0; a.start_t = start_t_dev;
  a.actions = actions_dev; a.rew = rewards_dev; a.term = terminated_dev; a.mask = mask_dev; a.obs = obs_dev;
  if (board_per_lane(h, true))
    hipLaunchKernelGGL(hex_rollout_lane_kernel, dim3(lane_blocks_for(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, a);
  else hipLaunchKernelGGL(hex_rollout_kernel, dim3(blocks_for(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, a);
  HIPCHK(hipGetLastError());
  return PGXHEX_OK;
}

int pgxhex_random_actions(pgxhex_t h, uint32_t seed, uint32_t t, const int32_t* start_t_dev, int32_t* actions_dev) {
  if (!h || !actions_dev) return PGXHEX_EINVAL;
  hipLaunchKernelGGL(hex_random_actions_kernel, dim3(blocks_for(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, h->rows, h->meta, h->B, seed, t,
                     start_t_dev, actions_dev);
  HIPCHK(hipGetLastError());
  return PGXHEX_OK;
}

int pgxhex_legal_mask(pgxhex_t h, uint8_t* dst_dev) {
  if (!h || !dst_dev) return PGXHEX_EINVAL;
  return launch_emit(h, dst_dev, nullptr);
}

int pgxhex_observe(pgxhex_t h, uint8_t* dst_dev) {
  if (!h || !dst_dev) return PGXHEX_EINVAL;
  return launch_emit(h, nullptr, dst_dev);
}

int pgxhex_rewards(pgxhex_t h, float* dst_dev) {
  if (!h || !dst_dev) return PGXHEX_EINVAL;
  if (dst_dev != h->rew_out) HIPCHK(hipMemcpyAsync(dst_dev, h->rew_out, (size_t)h->B * 2 * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
  return PGXHEX_OK;
}

int pgxhex_terminated(pgxhex_t h, uint8_t* dst_dev) {
  if (!h || !dst_dev) return PGXHEX_EINVAL;
  if (dst_dev != h->term_out) HIPCHK(hipMemcpyAsync(dst_dev, h->term_out, (size_t)h->B, hipMemcpyDeviceToDevice, h->stream));
  return PGXHEX_OK;
}

int pgxhex_current_player(pgxhex_t h, uint8_t* dst_dev) {
  if (!h || !dst_dev) return PGXHEX_EINVAL;
  hipLaunchKernelGGL(hex_current_player_kernel, dim3((unsigned)((h->B + 255) / 256)), dim3(256), 0, h->stream, h->meta, h->B, dst_dev);
  HIPCHK(hipGetLastError());
  return PGXHEX_OK;
}

int pgxhex_export_state(pgxhex_t h, int8_t* board_dev, int8_t* to_play_dev, int32_t* steps_dev, uint8_t* terminated_dev, uint8_t* black_player_dev,
                        uint32_t* episode_dev, uint32_t* illegal_dev) {
  if (!h) return PGXHEX_EINVAL;
  Canon c{board_dev, to_play_dev, steps_dev, terminated_dev, black_player_dev, episode_dev, illegal_dev};
  hipLaunchKernelGGL(hex_export_kernel, dim3(row_blocks(h->B)), dim3(256), 0, h->stream, h->rows, h->meta, h->B, c);
  HIPCHK(hipGetLastError());
  return PGXHEX_OK;
}

int pgxhex_import_state(pgxhex_t h, const int8_t* board_dev, const int8_t* to_play_dev, const int32_t* steps_dev, const uint8_t* terminated_dev,
                        const uint8_t* black_player_dev, const uint32_t* episode_dev) {
  if (!h || !board_dev || !to_play_dev || !steps_dev || !terminated_dev || !black_player_dev || !episode_dev) return PGXHEX_EINVAL;
  Canon c{(int8_t*)board_dev, (int8_t*)to_play_dev, (int32_t*)steps_dev, (uint8_t*)terminated_dev, (uint8_t*)black_player_dev, (uint32_t*)episode_dev,
          nullptr};
  hipLaunchKernelGGL(hex_import_kernel, dim3(row_blocks(h->B)), dim3(256), 0, h->stream, h->rows, h->meta, h->rew_out, h->term_out, h->B, c);
  HIPCHK(hipGetLastError());
  if (h->mask_out || h->obs_out) return launch_emit(h, h->mask_out, h->obs_out);
  return PGXHEX_OK;
}

int pgxhex_set_mapping(pgxhex_t h, int32_t mapping) {
  if (!h || mapping < 0 || mapping > 2) return PGXHEX_EINVAL;
  h->mapping = mapping;
  return board_per_lane(h) ? 2 : 1;
}

int pgxhex_sync(pgxhex_t h) {
  if (!h) return PGXHEX_EINVAL;
  HIPCHK(hipStreamSynchronize(h->stream));
  return PGXHEX_OK;
}

const char* pgxhex_strerror(int code) {
  switch (code) {
    case PGXHEX_OK: return "ok";
    case PGXHEX_EINVAL: return "invalid argument";
    case PGXHEX_EHIP: return "HIP runtime error";
    case PGXHEX_ENOMEM: return "out of host memory";
    default: return "unknown error";
  }
}

int pgxhex_last_hip_error(void) { return g_last_hip; }

}  // extern "C"
