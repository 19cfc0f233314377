// pgxgo.hip -- batched Go environment step for AMD MI355X (gfx950, wave64), C ABI in include/pgxgo.h.
//
// What is computed: the Go environment of the Pgx paper (arXiv 2303.17503): Fig. 2 (init/step API,
// legal_action_mask, observation, current_player), Table 1 (9x9x17 / 82 actions, 19x19x17 / 362 actions),
// Appendix C "Go" (Tromp-Taylor area scoring, komi for White, 8x2 history planes + colour plane, pass is
// the last action, rewards +1/-1/0), Sec. 4.1 (random policy, auto-reset on termination).
//
// How it is mapped to the machine (nothing of this is in the paper, whose implementation is XLA-generated):
//   * One board row per lane.  A wavefront holds W = 63/(N+1) boards (3 at 19x19, 6 at 9x9): board j owns
//     lanes j*(N+1)+1 .. j*(N+1)+N, and lanes j*(N+1) stay all-zero "sentinel rows", so a one-lane DPP
//     wave shift moves every row to its north/south neighbour and brings zeros in from off the board.
//   * Stones are row bitboards (bit c = column c).  East/west neighbours are register shifts, north/south
//     neighbours are DPP shifts; a flood-fill step is a handful of VALU instructions for all W boards at once.
//   * Facts about a whole board (a move is legal, a chain has one liberty, ...) come from a ballot masked with
//     the lane segment of the board; every lane of the board then holds the same answer.
//   * The state keeps, besides the stones, the set of stones whose chain has exactly one liberty
//     ("atari sets").  With them captures, the ko test and the whole legal mask are stencils; only the
//     chains touched by the move are re-flooded (the merged chain and at most four opposing neighbours),
//     a flood stops as soon as two liberties have been seen, and several growth steps are taken per
//     (comparatively expensive) look at the liberties.
//   * History is stored point-major: 16 bits per point = 8 plies x (black, white), two points per dword,
//     so a ply is one shift-and-insert per dword and the [N][N][17] byte observation is produced by
//     building the 17-bit-per-point bit stream of a board in LDS and expanding 16 bits -> 16 bytes per
//     lane through a 256-entry LDS table, stored as aligned 16-byte vectors.
//   * HBM layout: struct of arrays of 16-byte vectors, plane k holds dwords 4k..4k+3 of every row record,
//     indexed [env*N + row], so every load/store instruction of a wavefront touches one contiguous run.
//     Only the planes of a row that changed are written back (absolute colours make unchanged points
//     keep their history word).
//   * Kernels: go_step_kernel (one ply per launch, optionally drawing the next random action),
//     go_rollout_kernel (T plies per launch, state in registers), go_step_slots_kernel (tree search: step
//     from and to arbitrary state slots), go_step_superko_kernel (one ply with the positional-superko rule:
//     Zobrist keys in per-game open-addressing tables), plus small set-up / export / import kernels.
//   * How many boards a launch puts into a wavefront (1 .. W) is chosen per launch: W for throughput at large
//     batches, fewer at small batches where the slowest board of a wavefront and its serial output rounds
//     decide the latency.
//   * Output stores: every store instruction of a wavefront covers whole 128-byte lines (wave_common.hpp), and
//     the kind of store -- through the L2, with the non-temporal hint, ordinary -- is chosen per launch from the
//     bytes it writes and from whether it overwrites the previous launch's buffers (store_kind_for).  The
//     line-padded output pitches make a wavefront's stream consist of whole lines only.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <type_traits>

#include "pgxgo.h"
#include "wave_common.hpp"

namespace {

using namespace pgxwave;

thread_local int g_last_hip = 0;

#define HIPCHK(expr)                                   \
  do {                                                 \
    hipError_t e_ = (expr);                            \
    if (e_ != hipSuccess) {                            \
      g_last_hip = (int)e_;                            \
      return PGXGO_EHIP;                               \
    }                                                  \
  } while (0)

#ifndef PGXGO_WAVES_PER_BLOCK
#define PGXGO_WAVES_PER_BLOCK 4
#endif
constexpr int kWavesPerBlock = PGXGO_WAVES_PER_BLOCK;   // wavefronts never synchronise with each other; this only shapes the launch


// ------------------------------------------------------------------------------------------------
// geometry
// ------------------------------------------------------------------------------------------------
template <int N>
struct Geo {
  static constexpr int P = N * N;
  static constexpr int A = P + 1;
  static constexpr int STRIDE = N + 1;        // lanes per board, one of them the zero sentinel row
  static constexpr int W = 63 / STRIDE;       // boards per wavefront
  static constexpr int HD = (N + 1) / 2;      // history dwords per row, two points per dword
  static constexpr int REC = HD + 4;          // + black, white, atari-black, atari-white
  static constexpr int NQ = REC / 4;          // full 16-byte planes per row record
  static constexpr int REM = REC % 4;         // dwords of the last, narrower plane
  static constexpr uint32_t FULL = (1u << N) - 1u;
  static constexpr int OBS = P * 17;          // observation bytes per board
  static constexpr int ROWBITS = N * 17;      // observation bits contributed by one row
  static constexpr int NR = (ROWBITS + 31) / 32;       // dwords of one row's bit string
  static constexpr int NI = ROWBITS / 32 - 1;          // dwords 1..NI of the shifted string are never shared with another row
  static constexpr int OBS_PAD = (OBS + 127) / 128 * 128;   // the pitches at which every board starts on a 128-byte line
  static constexpr int A_PAD = (A + 127) / 128 * 128;
  static constexpr int OBS_DW = ((OBS_PAD + 15 + 31) / 32 + 3) / 4 * 4;   // LDS dwords of one board's bit stream (+ up to 15 lead bits)
  static constexpr int MASK_DW = ((A + 15 + 31) / 32 + 3) / 4 * 4;
  static constexpr size_t row_bytes = (size_t)REC * 4;
  // lanes holding the rows of board slot j
  static constexpr uint64_t seg(int j) { return ((1ull << N) - 1ull) << (j * STRIDE + 1); }
};

// per-board scalars, one 16-byte record per environment
//   x: ko point or -1     y: steps[0:16) | passes[16:18) | white_to_move[18] | terminated[19] | black_player[20]
//   z: episode            w: illegal actions received
struct Meta {
  int ko, steps, passes, wtm, term, bp;
  uint32_t episode, illegal;
};
__device__ __forceinline__ Meta unpack_meta(uint4 v) {
  Meta m;
  m.ko = (int)v.x;
  m.steps = v.y & 0xFFFF; m.passes = (v.y >> 16) & 3; m.wtm = (v.y >> 18) & 1; m.term = (v.y >> 19) & 1; m.bp = (v.y >> 20) & 1;
  m.episode = v.z; m.illegal = v.w;
  return m;
}
__device__ __forceinline__ uint4 pack_meta(const Meta& m) {
  uint4 v;
  v.x = (uint32_t)m.ko;
  v.y = (uint32_t)m.steps | ((uint32_t)m.passes << 16) | ((uint32_t)m.wtm << 18) | ((uint32_t)m.term << 19) | ((uint32_t)m.bp << 20);
  v.z = m.episode; v.w = m.illegal;
  return v;
}

// all 4-neighbours of the set x (bits beyond column N-1 may be set; callers intersect with on-board sets)
__device__ __forceinline__ uint32_t dilate(uint32_t x) { return (x << 1) | (x >> 1) | from_lane_below(x) | from_lane_above(x); }

// Size class of a board-wide set given by its row words: exactly one element / two or more.
__device__ __forceinline__ void board_count(uint32_t w, uint32_t seglo, uint32_t seghi, bool& one, bool& two) {
  const uint64_t nz = __ballot(w != 0u), mu = __ballot((w & (w - 1u)) != 0u);
  const int c = __popc((uint32_t)nz & seglo) + __popc((uint32_t)(nz >> 32) & seghi);
  two = (((uint32_t)mu & seglo) | ((uint32_t)(mu >> 32) & seghi)) != 0u || c >= 2;
  one = !two && c == 1;
}

// connected component(s) of `seed` inside S
__device__ __forceinline__ uint32_t flood_plain(uint32_t seed, uint32_t S) {
  uint32_t F = seed;
  for (;;) {   // three growth steps per convergence test: the test (ballot, scalar branch) costs as much as a step
    F |= dilate(F) & S;
    F |= dilate(F) & S;
    uint32_t G = F | (dilate(F) & S);
    bool ch = G != F;
    F = G;
    if (__ballot(ch) == 0ull) break;
  }
  return F;
}

// ------------------------------------------------------------------------------------------------
// lane bookkeeping
// ------------------------------------------------------------------------------------------------
template <int N>
struct Lane {
  int lane, j, r, b;     // lane id, board slot in the wavefront, row, index of the board in the call (outputs, actions)
  int slot;              // index of the environment whose state this board is (= b except in the slot kernels)
  bool valid;            // this lane holds a real row of a real board
  bool boardok;          // slot j holds a real board (also true for its sentinel lane)
  uint32_t seglo, seghi; // lanes of the rows of this lane's board
  uint32_t full;         // FULL on valid lanes, else 0
  // wb: boards this launch puts into a wavefront (1 .. W; fewer than W trades lanes for latency at small batches)
  __device__ __forceinline__ Lane(int wave, int lane_, int B, int wb = Geo<N>::W) {
    using G = Geo<N>;
    lane = lane_;
    j = lane / G::STRIDE;
    int rr = lane - j * G::STRIDE;
    r = rr - 1;
    b = wave * wb + j;
    slot = b;
    boardok = (j < wb) && (b < B);
    valid = boardok && rr >= 1;
    uint64_t seg = (j < wb) ? (((1ull << N) - 1ull) << (j * G::STRIDE + 1)) : 0ull;
    seglo = (uint32_t)seg; seghi = (uint32_t)(seg >> 32);
    full = valid ? G::FULL : 0u;
  }
};

template <int N>
struct Row {                      // per-lane registers: one row of one board
  uint32_t h[Geo<N>::HD];         // history halfwords, bit 2i = black i plies ago, bit 2i+1 = white
  uint32_t bk, wt, ab, aw;        // stones and atari sets (stones of chains with exactly one liberty)
};

// record dword k of row idx lives in plane k/4 (16-byte planes first, then one narrower plane)
template <int N>
__device__ __forceinline__ void load_row(const uint4* __restrict__ planes, size_t rows_total, const Lane<N>& L, Row<N>& R) {
  using G = Geo<N>;
  uint32_t rec[G::NQ * 4 + 4];
#pragma unroll
  for (int k = 0; k < G::NQ * 4 + 4; ++k) rec[k] = 0u;
  if (L.valid) {
    const size_t idx = (size_t)L.slot * N + L.r;
#pragma unroll
    for (int k = 0; k < G::NQ; ++k) {
      uint4 v = planes[(size_t)k * rows_total + idx];
      rec[4 * k] = v.x; rec[4 * k + 1] = v.y; rec[4 * k + 2] = v.z; rec[4 * k + 3] = v.w;
    }
    const uint32_t* tail = (const uint32_t*)(planes + (size_t)G::NQ * rows_total);
    if constexpr (G::REM == 2) { uint2 v = *(const uint2*)(tail + idx * 2); rec[4 * G::NQ] = v.x; rec[4 * G::NQ + 1] = v.y; }
    if constexpr (G::REM == 1) { rec[4 * G::NQ] = tail[idx]; }
  }
#pragma unroll
  for (int k = 0; k < G::HD; ++k) R.h[k] = rec[k];
  R.bk = rec[G::HD]; R.wt = rec[G::HD + 1]; R.ab = rec[G::HD + 2]; R.aw = rec[G::HD + 3];
}

// ST: kind of the 16-byte stores (wave_common.hpp)
template <int N, int ST = kStorePlain>
__device__ __forceinline__ void store_row(uint4* __restrict__ planes, size_t rows_total, const Lane<N>& L, const Row<N>& R) {
  using G = Geo<N>;
  uint32_t rec[G::NQ * 4 + 4];
#pragma unroll
  for (int k = 0; k < G::HD; ++k) rec[k] = R.h[k];
  rec[G::HD] = R.bk; rec[G::HD + 1] = R.wt; rec[G::HD + 2] = R.ab; rec[G::HD + 3] = R.aw;
  if (L.valid) {
    const size_t idx = (size_t)L.slot * N + L.r;
#pragma unroll
    for (int k = 0; k < G::NQ; ++k)
      store16<ST>(&planes[(size_t)k * rows_total + idx], make_uint2(rec[4 * k], rec[4 * k + 1]), make_uint2(rec[4 * k + 2], rec[4 * k + 3]));
    uint32_t* tail = (uint32_t*)(planes + (size_t)G::NQ * rows_total);
    if constexpr (G::REM == 2) *(uint2*)(tail + idx * 2) = make_uint2(rec[4 * G::NQ], rec[4 * G::NQ + 1]);
    if constexpr (G::REM == 1) tail[idx] = rec[4 * G::NQ];
  }
}

// The four row words as loaded, kept to tell at store time which of them changed.
struct RowWords {
  uint32_t bk, wt, ab, aw;
};
template <int N>
__device__ __forceinline__ RowWords row_words(const Row<N>& R) { return RowWords{R.bk, R.wt, R.ab, R.aw}; }

// Stores only the 16-byte planes of this row whose content differs from what the kernel loaded.  With colours
// stored absolutely, a history word changes only while its point changed within the last 8 plies, so most
// rows of most planes are unchanged from ply to ply.  hdirty: bit k set = a history dword of plane k changed (from
// push_history; all ones after a reset); Old: the row words as loaded.
template <int N>
__device__ __forceinline__ void store_row_changed(uint4* __restrict__ planes, size_t rows_total, const Lane<N>& L, const Row<N>& R, uint32_t hdirty,
                                                  const RowWords& Old) {
  using G = Geo<N>;
  uint32_t rec[G::NQ * 4 + 4], dif[G::NQ * 4 + 4];
#pragma unroll
  for (int k = 0; k < G::NQ * 4 + 4; ++k) { rec[k] = 0u; dif[k] = 0u; }
#pragma unroll
  for (int k = 0; k < G::HD; ++k) rec[k] = R.h[k];
  rec[G::HD] = R.bk; rec[G::HD + 1] = R.wt; rec[G::HD + 2] = R.ab; rec[G::HD + 3] = R.aw;
  dif[G::HD] = R.bk ^ Old.bk; dif[G::HD + 1] = R.wt ^ Old.wt; dif[G::HD + 2] = R.ab ^ Old.ab; dif[G::HD + 3] = R.aw ^ Old.aw;
  if (L.valid) {
    const size_t idx = (size_t)L.slot * N + L.r;
#pragma unroll
    for (int k = 0; k <= G::NQ; ++k) {   // k = NQ: the narrower last plane
      const uint32_t diff = ((hdirty >> k) & 1u) | dif[4 * k] | dif[4 * k + 1] | dif[4 * k + 2] | dif[4 * k + 3];
      if (k < G::NQ) {
        if (diff) planes[(size_t)k * rows_total + idx] = make_uint4(rec[4 * k], rec[4 * k + 1], rec[4 * k + 2], rec[4 * k + 3]);
      } else {
        uint32_t* tail = (uint32_t*)(planes + (size_t)G::NQ * rows_total);
        if constexpr (G::REM == 2) { if (diff) *(uint2*)(tail + idx * 2) = make_uint2(rec[4 * G::NQ], rec[4 * G::NQ + 1]); }
        if constexpr (G::REM == 1) { if (diff) tail[idx] = rec[4 * G::NQ]; }
      }
    }
  }
}

// legal points of the player to move (Fig. 2 legal_action_mask, pass excluded): empty, not the ko point, and
// next to an empty point, or to an own chain that is not in atari, or to an opposing chain that is
template <int N>
__device__ __forceinline__ uint32_t legal_row(const Lane<N>& L, const Row<N>& R, int wtm, int ko) {
  uint32_t E = L.full & ~(R.bk | R.wt);
  uint32_t own = wtm ? R.wt : R.bk, opp = wtm ? R.bk : R.wt;
  uint32_t aown = wtm ? R.aw : R.ab, aopp = wtm ? R.ab : R.aw;
  uint32_t support = E | (own & ~aown) | (opp & aopp);
  int kr = ko / N, kc = ko - kr * N;
  uint32_t kobit = (ko >= 0 && L.r == kr) ? (1u << kc) : 0u;
  return E & ~kobit & dilate(support);
}

// Legal mask bytes [N*N+1] of every board of the wavefront.  TIGHT: the pitch is the dense one (N*N+1) or the
// line-padded one (A_PAD); the boards of a wavefront are then one contiguous run of bytes, pad bytes included, and
// are staged and written as one stream (the pad bytes as zeros); otherwise board by board, pad bytes untouched.
template <int N, bool TIGHT, int ST = kStorePlain>
__device__ __forceinline__ void emit_mask(const Lane<N>& L, uint32_t legal, int wave, int B, uint8_t* mask, int64_t mask_pitch,
                                          uint32_t* lds_mask, const uint2* lut, int wb = Geo<N>::W) {
  using G = Geo<N>;
  static_assert(G::W * G::MASK_DW <= 64 && (15 + G::W * G::A_PAD + 31) / 32 <= 64, "mask staging is cleared by one store per lane");
  constexpr bool tight = TIGHT;   // the caller guarantees mask_pitch == N*N+1 or A_PAD
  const uint32_t stride = (uint32_t)mask_pitch;
  const int b0 = wave * wb;
  const int nb = B - b0 < wb ? B - b0 : wb;   // boards of this wavefront
  lds_mask[L.lane] = 0u;
  wave_lds_fence();
  if (L.valid) {
    uint32_t* reg;
    uint32_t head;
    if constexpr (tight) { head = (uint32_t)((uintptr_t)(mask + (int64_t)b0 * mask_pitch) & 15u) + __umul24((uint32_t)L.j, stride); reg = lds_mask; }
    else { head = (uint32_t)((uintptr_t)(mask + (int64_t)L.b * mask_pitch) & 15u); reg = lds_mask + L.j * G::MASK_DW; }
    const uint32_t o = head + (uint32_t)(N * L.r), q = o >> 5, s = o & 31u;
    atomicOr(&reg[q], legal << s);
    if (s + N > 32u) atomicOr(&reg[q + 1], legal >> (32u - s));
    if (L.r == 0) { const uint32_t o2 = head + G::P; atomicOr(&reg[o2 >> 5], 1u << (o2 & 31u)); }   // pass is always legal
  }
  wave_lds_fence();
  if constexpr (tight) {
    emit_bytes<G::W * G::A_PAD, ST>(lds_mask, lut, mask + (int64_t)b0 * mask_pitch, (uint32_t)nb * stride, L.lane);
  } else {
#pragma unroll
    for (int jj = 0; jj < G::W; ++jj)
      if (jj < nb) emit_bytes<G::A, ST>(lds_mask + jj * G::MASK_DW, lut, mask + (int64_t)(b0 + jj) * mask_pitch, G::A, L.lane);
  }
  wave_lds_fence();
}

// Observation bytes [N][N][17] of every board of the wavefront from the history words h of its rows.
template <int N, bool TIGHT, int ST = kStorePlain>
__device__ __forceinline__ void emit_obs(const Lane<N>& L, const uint32_t (&h)[Geo<N>::HD], int wtm, int wave, int B, uint8_t* obs,
                                         int64_t obs_pitch, uint32_t* lds_obs, const uint2* lut, int wb = Geo<N>::W) {
  using G = Geo<N>;
  static_assert((15 + G::W * G::OBS_PAD + 31) / 32 <= G::W * G::OBS_DW, "one stream for all boards fits the staging area");
  constexpr bool tight = TIGHT;   // the caller guarantees obs_pitch == N*N*17 or OBS_PAD (see emit_mask)
  const uint32_t stride = (uint32_t)obs_pitch;
  const int b0 = wave * wb;
  const int nb = B - b0 < wb ? B - b0 : wb;
  // 17 bits per point: the point's history halfword seen by the mover (pairs swapped when White moves),
  // then the colour bit (Appendix C "Go", Observation); a row is N such pieces back to back.
  uint32_t S[G::NR];
#pragma unroll
  for (int k = 0; k < G::NR; ++k) S[k] = 0u;
  const uint32_t cb = wtm ? 0u : 1u;
  const uint32_t swapmask = wtm ? 0x55555555u : 0u;
#pragma unroll
  for (int jd = 0; jd < G::HD; ++jd) {
    uint32_t w = h[jd];
    uint32_t x = (w ^ (w >> 1)) & swapmask;
    w ^= x | (x << 1);
    uint32_t lo17 = (w & 0xFFFFu) | (cb << 16);
    uint32_t hi17 = (2 * jd + 1 < N) ? ((w >> 16) | (cb << 16)) : 0u;
    uint32_t low32 = lo17 | (hi17 << 17), high2 = hi17 >> 15;
    const int pos = 34 * jd, k = pos >> 5, sh = pos & 31;
    S[k] |= low32 << sh;
    if (k + 1 < G::NR) S[k + 1] |= sh ? ((low32 >> (32 - sh)) | (high2 << sh)) : high2;
  }
  {
    uint4* z = (uint4*)lds_obs;
    constexpr int NZ = G::W * G::OBS_DW / 4;
#pragma unroll
    for (int i = 0; i < (NZ + 63) / 64; ++i)
      if (i * 64 + 63 < NZ || i * 64 + L.lane < NZ) z[i * 64 + L.lane] = make_uint4(0u, 0u, 0u, 0u);
  }
  wave_lds_fence();
  if (L.valid) {
    uint32_t* reg;
    uint32_t head;
    if constexpr (tight) { head = (uint32_t)((uintptr_t)(obs + (int64_t)b0 * obs_pitch) & 15u) + __umul24((uint32_t)L.j, stride); reg = lds_obs; }
    else { head = (uint32_t)((uintptr_t)(obs + (int64_t)L.b * obs_pitch) & 15u); reg = lds_obs + L.j * G::OBS_DW; }
    // The row's string goes to bit offset o of the stream.  Written as a left shift by u = 1..32 from dword (o-u)/32
    // on, every shifted dword is one funnel shift of two neighbours of S (a shift by 0 would need a special case):
    // T[i] = bits of dword q+i; T[0] and T[NI+1..NR] may share their dword with the rows next door.
    const uint32_t o = head + (uint32_t)(G::ROWBITS * L.r);
    const uint32_t u1 = (o + 31u) & 31u;            // u - 1
    reg += (int32_t)(o - 1u - u1) >> 5;             // dword -1 only when o = 0, and then T[0] = 0 is not written
    const uint32_t sh = 31u - u1;                   // right shift of the (S[i], S[i-1]) pair that equals the left shift by u
    {
      const uint32_t t0 = __builtin_amdgcn_alignbit(S[0], 0u, sh);
      if (t0) atomicOr(&reg[0], t0);
    }
#pragma unroll
    for (int i = 1; i <= G::NR; ++i) {
      const uint32_t hi = (i < G::NR) ? S[i] : 0u;
      const uint32_t t = __builtin_amdgcn_alignbit(hi, S[i - 1], sh);
      if (i <= G::NI) reg[i] = t;
      else if (t) atomicOr(&reg[i], t);
    }
  }
  wave_lds_fence();
  if constexpr (tight) {
    emit_bytes<G::W * G::OBS_PAD, ST>(lds_obs, lut, obs + (int64_t)b0 * obs_pitch, (uint32_t)nb * stride, L.lane);
  } else {
#pragma unroll
    for (int jj = 0; jj < G::W; ++jj)
      if (jj < nb) emit_bytes<G::OBS, ST>(lds_obs + jj * G::OBS_DW, lut, obs + (int64_t)(b0 + jj) * obs_pitch, G::OBS, L.lane);
  }
  wave_lds_fence();
}

template <int N, bool TIGHT, int ST = kStorePlain>
__device__ __forceinline__ void emit_outputs(const Lane<N>& L, const Row<N>& R, uint32_t legal, int wtm, int wave, int B,
                                             uint8_t* mask, int64_t mask_pitch, uint8_t* obs, int64_t obs_pitch,
                                             uint32_t* lds_mask, uint32_t* lds_obs, const uint2* lut, int wb = Geo<N>::W) {
  if (mask) emit_mask<N, TIGHT, ST>(L, legal, wave, B, mask, mask_pitch, lds_mask, lut, wb);
  if (obs) emit_obs<N, TIGHT, ST>(L, R.h, wtm, wave, B, obs, obs_pitch, lds_obs, lut, wb);
}

// ------------------------------------------------------------------------------------------------
// uniform random legal action: the k-th legal action in ascending order, k = hash mod legal_count
// ------------------------------------------------------------------------------------------------
template <int N>
struct Draw {          // the drawn action as every lane of the board sees it
  bool pass, point;    // neither = the environment is still waiting for its start time (action -1)
  int pr, pc;          // row and column when `point`
  __device__ __forceinline__ int action() const { return pass ? Geo<N>::P : point ? pr * N + pc : -1; }
};

template <int N>
__device__ __forceinline__ Draw<N> draw_action(const Lane<N>& L, uint32_t legal, uint32_t seed, uint32_t t, bool wait) {
  using G = Geo<N>;
  const uint32_t cnt = __popc(legal);
  // legal points in the rows above this one, and on the whole board, from ballots of the bits of cnt
  uint32_t before = 0u, total = 1u;   // pass is always legal
#pragma unroll
  for (int k = 0; (1 << k) <= N; ++k) {
    const uint64_t m = __ballot((cnt >> k) & 1u);
    const uint32_t lo = (uint32_t)m & L.seglo, hi = (uint32_t)(m >> 32) & L.seghi;
    before += __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u)) << k;
    total += (uint32_t)(__popc(lo) + __popc(hi)) << k;
  }
  const uint32_t k = env_hash(seed, 0u, (uint32_t)L.b, t) % total;
  // position of the (n+1)-th set bit of the row word by halving (meaningful in the row that holds it)
  uint32_t n = k - before, w = legal, pos = 0u;
#pragma unroll
  for (int width = 16; width >= 1; width >>= 1) {
    const uint32_t c = __popc(w & ((1u << width) - 1u));
    if (n >= c) { n -= c; w >>= width; pos += width; }
  }
  const bool mine = L.valid && k >= before && k < before + cnt;
  const uint64_t sel = __ballot(mine);
  const uint32_t slo = (uint32_t)sel & L.seglo, shi = (uint32_t)(sel >> 32) & L.seghi;
  const int src = slo ? __ffs(slo) - 1 : 31 + __ffs(shi);   // lane of the chosen row (any lane when pass is drawn)
  Draw<N> d;
  d.pass = !wait && k == total - 1u;
  d.point = !wait && k != total - 1u;
  d.pr = (src & 63) - (L.j * G::STRIDE + 1);
  d.pc = (int)__shfl((int)pos, src & 63);
  return d;
}

// ------------------------------------------------------------------------------------------------
// one ply for every board of the wavefront (steps a2-a8); registers in, registers out
// ------------------------------------------------------------------------------------------------
struct Rules {
  uint32_t seed;
  int komi_x2, max_steps, auto_reset;
};

// What a requested action amounts to for a board (the same in every lane of the board).
struct Move {
  bool skip;      // leave the board alone
  bool frozen;    // the game had ended before (no auto-reset): nothing changes, terminated is reported
  bool is_pass, playing, illegal;
  int pr, pc;     // the point when `playing`
};

// a1/a2.  want_pass / want_point(pr,pc): the requested action; anything else is illegal.
// GATE: check the point against the mover's legal set (not needed for actions drawn from that set).
template <int N, bool GATE>
__device__ __forceinline__ Move gate_move(const Lane<N>& L, const Row<N>& R, const Meta& m, bool skip, bool want_pass, bool want_point,
                                          int pr_in, int pc_in) {
  Move mv;
  mv.skip = skip;
  mv.frozen = !skip && m.term;
  const bool live = !skip && !mv.frozen;
  mv.is_pass = live && want_pass;
  const bool on_board = live && want_point;
  mv.playing = on_board;
  if (GATE) {
    const uint32_t pbit = (L.valid && on_board && L.r == pr_in) ? (1u << pc_in) : 0u;
    const uint32_t legal_now = legal_row<N>(L, R, m.wtm, m.ko);
    mv.playing = on_board && board_any((legal_now & pbit) != 0u, L.seglo, L.seghi);
  }
  mv.illegal = live && !mv.is_pass && !mv.playing;
  mv.pr = mv.playing ? pr_in : -100;
  mv.pc = mv.playing ? pc_in : 0;
  return mv;
}

// history push: every halfword shifts by one ply and takes the position (bk, wt) in its low bits
// hdirty: bit k is set when a history dword of the row record's 16-byte plane k changed
template <int N>
__device__ __forceinline__ void push_history(uint32_t (&h)[Geo<N>::HD], uint32_t bk, uint32_t wt, bool moved, uint32_t& hdirty) {
  const uint32_t lo = (bk & 0x55555555u) | ((wt & 0x55555555u) << 1);   // bit 2j / 2j+1: black / white at column 2j
  const uint32_t hi = ((bk >> 1) & 0x55555555u) | (wt & 0xAAAAAAAAu);   // the same for column 2j+1
  uint32_t acc[(Geo<N>::HD + 3) / 4];
#pragma unroll
  for (int k = 0; k < (Geo<N>::HD + 3) / 4; ++k) acc[k] = 0u;
#pragma unroll
  for (int jd = 0; jd < Geo<N>::HD; ++jd) {
    const uint32_t cur = ((lo >> (2 * jd)) & 3u) | (((hi >> (2 * jd)) & 3u) << 16);
    const uint32_t pushed = ((h[jd] << 2) & 0xFFFCFFFCu) | cur;
    acc[jd / 4] |= moved ? (pushed ^ h[jd]) : 0u;
    h[jd] = moved ? pushed : h[jd];
  }
  hdirty = 0u;
#pragma unroll
  for (int k = 0; k < (Geo<N>::HD + 3) / 4; ++k) hdirty |= acc[k] ? (1u << k) : 0u;
}

// a8: back to the initial state of the next episode (Sec. 4.1); the seat is drawn anew
template <int N>
__device__ __forceinline__ void reset_board(const Lane<N>& L, Row<N>& R, Meta& m, uint32_t seed) {
#pragma unroll
  for (int jd = 0; jd < Geo<N>::HD; ++jd) R.h[jd] = 0u;
  R.bk = R.wt = R.ab = R.aw = 0u;
  m.ko = -1; m.steps = 0; m.passes = 0; m.wtm = 0; m.term = 0;
  m.episode += 1;
  m.bp = (int)(env_hash(seed, 1u, (uint32_t)L.slot, m.episode) & 1u);
}

// a3-a8 for every board of the wavefront; registers in, registers out.
// Out: rewards by player id, `flag` = the terminated output (game ended in this ply, or had ended before),
// `captured` = the stones this ply removed, `reset` = the board was re-initialised by auto-reset.
// `hdirty` = which planes of the row record hold a changed history dword (see push_history; all ones after a reset).
template <int N>
__device__ __forceinline__ void apply_move(const Lane<N>& L, Row<N>& R, Meta& m, const Rules& cfg, const Move& mv, float& rew0, float& rew1,
                                           bool& flag, uint32_t& captured, bool& reset, uint32_t& hdirty) {
  using G = Geo<N>;
  const bool playing = mv.playing, is_pass = mv.is_pass, illegal = mv.illegal, frozen = mv.frozen;
  const int pr = mv.pr, pc = mv.pc;
  const uint32_t pbit = (L.valid && L.r == pr) ? (1u << pc) : 0u;
  const int wtm0 = m.wtm;
  rew0 = 0.f; rew1 = 0.f;
  captured = 0u;

  // ---- a3-a5: place the stone, capture, update the atari sets, ko ----------------------------------------
  if (__ballot(playing) != 0ull) {
    uint32_t own = wtm0 ? R.wt : R.bk, opp = wtm0 ? R.bk : R.wt;
    uint32_t aown = wtm0 ? R.aw : R.ab, aopp = wtm0 ? R.ab : R.aw;
    const uint32_t nbN = (L.valid && L.r == pr - 1) ? (1u << pc) : 0u;
    const uint32_t nbS = (L.valid && L.r == pr + 1) ? (1u << pc) : 0u;
    const uint32_t nbW = (L.valid && L.r == pr) ? ((1u << pc) >> 1) : 0u;
    const uint32_t nbE = (L.valid && L.r == pr) ? ((2u << pc) & G::FULL) : 0u;
    const uint32_t nb = nbN | nbS | nbW | nbE;
    const uint32_t friends = nb & own;   // own stones next to the new one
    own |= pbit;
    // opposing chains in atari that touch the new stone lose their last liberty
    int ko_new = -1;
    const uint32_t capseed = nb & aopp;
    if (__ballot(capseed != 0u) != 0ull) {
      const uint32_t cap = flood_plain(capseed, aopp);
      if (playing) captured = cap;
      opp &= ~cap; aopp &= ~cap;
      // own chains in atari next to the vacated points gain a liberty
      const uint32_t un = flood_plain(aown & dilate(cap), aown);
      aown &= ~un;
      // simple ko: exactly one stone taken by a stone without friends whose only liberty is the vacated point
      bool cap1, cap2, lib1, lib2;
      board_count(cap, L.seglo, L.seghi, cap1, cap2);
      board_count(nb & L.full & ~(own | opp), L.seglo, L.seghi, lib1, lib2);
      const bool lone = !board_any(friends != 0u, L.seglo, L.seghi);
      const bool cN = board_any((cap & nbN) != 0u, L.seglo, L.seghi), cS = board_any((cap & nbS) != 0u, L.seglo, L.seghi);
      const bool cW = board_any((cap & nbW) != 0u, L.seglo, L.seghi);
      const int p = pr * N + pc;
      if (cap1 && lib1 && lone) ko_new = cN ? p - N : cS ? p + N : cW ? p - 1 : p + 1;
    }
    const uint32_t E = L.full & ~(own | opp);
    // own chains in atari that the new stone joins stop being chains of their own
    const uint32_t clrseed = friends & aown;
    if (__ballot(clrseed != 0u) != 0ull) aown &= ~flood_plain(clrseed, aown);
    // Liberty class of the new stone's chain (flood 0, through own stones) and of the surviving opposing
    // neighbour chains, which lost the liberty just filled (floods 1-4, through opposing stones).  A flood
    // leaves the race as soon as two liberties are known; one that converges with a single liberty has
    // found a whole chain in atari.
    uint32_t F0 = pbit, F1 = nbN & opp, F2 = nbS & opp, F3 = nbW & opp, F4 = nbE & opp;
    bool run0 = board_any(F0 != 0u, L.seglo, L.seghi), run1 = board_any(F1 != 0u, L.seglo, L.seghi);
    bool run2 = board_any(F2 != 0u, L.seglo, L.seghi), run3 = board_any(F3 != 0u, L.seglo, L.seghi);
    bool run4 = board_any(F4 != 0u, L.seglo, L.seghi);
    bool at0 = false, at1 = false, at2 = false, at3 = false, at4 = false;
    auto flood_step = [&](uint32_t& F, uint32_t S, bool& run, bool& at, bool first) {
      if (!first) {   // after the first look, unexamined growth steps precede each examined one
#ifndef PGXGO_BLIND
#define PGXGO_BLIND 4
#endif
#pragma unroll
        for (int b_ = 0; b_ < PGXGO_BLIND; ++b_) F |= dilate(F) & S;
      }
      const uint32_t D = dilate(F);
      const uint32_t Gn = F | (D & S);
      bool one, two;
      board_count(D & E, L.seglo, L.seghi, one, two);
      const bool grew = board_any(Gn != F, L.seglo, L.seghi);
      const bool conv = run && !two && !grew;
      at = at || (conv && one);
      run = run && !two && !conv;
      F = Gn;
    };
    bool first = true;
    for (;;) {
      const uint64_t r0 = __ballot(run0), r1 = __ballot(run1), r2 = __ballot(run2), r3 = __ballot(run3), r4 = __ballot(run4);
      if ((r0 | r1 | r2 | r3 | r4) == 0ull) break;
      if (r0 != 0ull) flood_step(F0, own, run0, at0, first);
      if (r1 != 0ull) flood_step(F1, opp, run1, at1, first);
      if (r2 != 0ull) flood_step(F2, opp, run2, at2, first);
      if (r3 != 0ull) flood_step(F3, opp, run3, at3, first);
      if (r4 != 0ull) flood_step(F4, opp, run4, at4, first);
      first = false;
    }
    aown |= at0 ? F0 : 0u;
    aopp |= (at1 ? F1 : 0u) | (at2 ? F2 : 0u) | (at3 ? F3 : 0u) | (at4 ? F4 : 0u);
    if (playing) {
      m.ko = ko_new;
      R.bk = wtm0 ? opp : own; R.wt = wtm0 ? own : opp;
      R.ab = wtm0 ? aopp : aown; R.aw = wtm0 ? aown : aopp;
    }
  }
  const bool moved = playing || is_pass;
  if (is_pass) { m.ko = -1; m.passes += 1; }
  if (playing) m.passes = 0;
  if (moved) {
    m.steps += 1;
    m.wtm ^= 1;
  }
  // ---- a6: history push ---------------------------------------------------------------------------------
  push_history<N>(R.h, R.bk, R.wt, moved, hdirty);

  // ---- a7: termination and Tromp-Taylor area score ------------------------------------------------------
  const bool score = moved && (m.passes >= 2 || m.steps >= cfg.max_steps);
  if (__ballot(score) != 0ull) {
    const uint32_t E = L.full & ~(R.bk | R.wt);
    const uint32_t rb = flood_plain(E & dilate(R.bk), E);
    const uint32_t rw = flood_plain(E & dilate(R.wt), E);
    // per-board sum of (black area - white area) of the rows, from ballots of the bits of a biased row value
    const uint32_t v = (uint32_t)(__popc(R.bk | (rb & ~rw)) - __popc(R.wt | (rw & ~rb)) + N);   // 0 .. 2N
    int sum = -N * N;
#pragma unroll
    for (int k = 0; (1 << k) <= 2 * N; ++k) {
      const uint64_t mk = __ballot((v >> k) & 1u);
      sum += (__popc((uint32_t)mk & L.seglo) + __popc((uint32_t)(mk >> 32) & L.seghi)) << k;
    }
    if (score) {
      int d = 2 * sum - cfg.komi_x2;   // komi counts for White
      float s = d > 0 ? 1.f : (d < 0 ? -1.f : 0.f);
      rew0 = m.bp == 0 ? s : -s;
      rew1 = -rew0;
    }
  }
  if (illegal) {  // the offender loses at once, the position stays
    const int mover = wtm0 ? 1 - m.bp : m.bp;
    rew0 = mover == 0 ? -1.f : 1.f;
    rew1 = -rew0;
    m.illegal += 1;
  }
  const bool ended = score || illegal;
  reset = ended && cfg.auto_reset != 0;
  if (ended) {
    m.term = 1;
    // ---- a8: auto-reset (Sec. 4.1) -------------------------------------------------------------------------
    if (cfg.auto_reset) { reset_board<N>(L, R, m, cfg.seed); hdirty = ~0u; }
  }
  flag = ended || frozen;
}
template <int N>
__device__ __forceinline__ void apply_move(const Lane<N>& L, Row<N>& R, Meta& m, const Rules& cfg, const Move& mv, float& rew0, float& rew1,
                                           bool& flag, uint32_t& captured, bool& reset) {
  uint32_t hdirty;
  apply_move<N>(L, R, m, cfg, mv, rew0, rew1, flag, captured, reset, hdirty);
}

template <int N, bool GATE>
__device__ __forceinline__ void step_core(const Lane<N>& L, Row<N>& R, Meta& m, const Rules& cfg, bool skip, bool want_pass, bool want_point,
                                          int pr_in, int pc_in, float& rew0, float& rew1, bool& flag) {
  const Move mv = gate_move<N, GATE>(L, R, m, skip, want_pass, want_point, pr_in, pc_in);
  uint32_t captured;
  bool reset;
  apply_move<N>(L, R, m, cfg, mv, rew0, rew1, flag, captured, reset);
}

// ------------------------------------------------------------------------------------------------
// the step kernel: one launch = one ply of every environment
// ------------------------------------------------------------------------------------------------
struct StepArgs {
  uint4* planes;
  uint4* meta;
  const int32_t* actions;
  float* rew;
  uint8_t* term;
  uint8_t* mask;
  uint8_t* obs;
  int64_t mask_pitch, obs_pitch;
  int B;
  int wb;                    // boards per wavefront of this launch
  int store_kind;            // kind of the output stores, by the bytes the launch writes (store_kind_for)
  int sparse_store;
  Rules rules;
  // fused sampler
  uint32_t sample_seed, sample_t;
  const int32_t* start_t;
  int32_t* next_actions;
};

template <int N, bool SAMPLE, bool TIGHT, int ST>
__global__ void __launch_bounds__(64 * kWavesPerBlock, 6) go_step_kernel(StepArgs a) {
  using G = Geo<N>;
  __shared__ __attribute__((aligned(16))) uint32_t lds_obs_all[kWavesPerBlock][G::W * G::OBS_DW];
  __shared__ __attribute__((aligned(16))) uint32_t lds_mask_all[kWavesPerBlock][64];
  __shared__ uint2 lut[256];
  const int wib = wave_in_block();
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  const Lane<N> L(wave, threadIdx.x & 63, a.B, a.wb);   // in a wavefront beyond the batch no lane is valid
  const size_t rows_total = (size_t)a.B * N;

  // the loads are issued first and fly while the block fills its lookup table
  Row<N> R;
  load_row<N>(a.planes, rows_total, L, R);
  const uint4 meta_raw = L.boardok ? a.meta[L.b] : make_uint4(0xFFFFFFFFu, 0u, 0u, 0u);
  const int act = L.boardok ? a.actions[L.b] : -1;
  // loaded here and not where it is used: a load after the output stores would have to wait for them (one counter);
  // looked at only after the table is filled, so that no wait for a load comes before the barrier
  const int32_t start_raw = (SAMPLE && L.boardok && a.start_t) ? a.start_t[L.b] : INT32_MIN;
  fill_spread_table(lut);
  if (wave * a.wb >= a.B) return;   // whole wavefront idle; there is no block-wide barrier anywhere below
  const bool wait_start = (int64_t)a.sample_t < (int64_t)held_back(start_raw);
  const RowWords W_loaded = row_words<N>(R);
  Meta m = unpack_meta(meta_raw);

  // a1/a2: decode the action and gate it
  const bool skip = !L.boardok || act == -1;
  const bool in_range = act >= 0 && act < G::P;
  const int pr = in_range ? act / N : 0, pc = in_range ? act - (act / N) * N : 0;
  const Move mv = gate_move<N, true>(L, R, m, skip, act == G::P, in_range, pr, pc);

  // a3-a8
  float rew0, rew1;
  bool flag, reset;
  uint32_t captured, hdirty;
  apply_move<N>(L, R, m, a.rules, mv, rew0, rew1, flag, captured, reset, hdirty);
  if (!skip && L.valid && L.r == 0) {
    *(float2*)(a.rew + 2 * (size_t)L.b) = make_float2(rew0, rew1);
    a.term[L.b] = (uint8_t)(flag ? 1 : 0);
  }

  // ---- a10 / a9: observation and legal mask of the player now to move ---------------------------------------
  if (a.obs) emit_obs<N, TIGHT, ST>(L, R.h, m.wtm, wave, a.B, a.obs, a.obs_pitch, lds_obs_all[wib], lut, a.wb);
  const uint32_t legal = legal_row<N>(L, R, m.wtm, m.ko);
  if (a.mask) emit_mask<N, TIGHT, ST>(L, legal, wave, a.B, a.mask, a.mask_pitch, lds_mask_all[wib], lut, a.wb);

  // ---- a11: store the state --------------------------------------------------------------------------------
  if (!skip) {
    // Writing only the changed planes pays while state and outputs stay resident in the memory-side cache
    // (partial lines merge there); beyond it partial lines cost a read-modify-write in DRAM and whole rows win.
    // (whole rows written through the L2: 65536 games 87.9 -> 85.5 us per ply; with the non-temporal hint they are slower)
    if (a.sparse_store) store_row_changed<N>(a.planes, rows_total, L, R, hdirty, W_loaded);
    else store_row<N, kStoreThrough>(a.planes, rows_total, L, R);
    if (L.valid && L.r == 0) a.meta[L.b] = pack_meta(m);
  }
  if (SAMPLE) {
    const Draw<N> d = draw_action<N>(L, legal, a.sample_seed, a.sample_t, wait_start);
    if (L.valid && L.r == 0) a.next_actions[L.b] = d.action();
  }
}

// ------------------------------------------------------------------------------------------------
// positional superko (Appendix C "Go": Tromp-Taylor rules, whose repetition rule forbids a play that recreates
// an earlier whole-board position of the game).  Two readings, chosen by `mode`: 2 = the rule proper, the legal mask
// leaves such plays out; 1 = looked at only when the move is played (the offender loses like for any illegal
// action) while the mask keeps showing the simple-ko set.
//
// Every position is summarised by two 32-bit Zobrist keys, one per colour (XOR of one key per stone of that colour,
// updated from the stones that changed), and its two stone counts.  A play by colour c always gives a position with
// exactly one more stone of colour c, so the earlier positions a play can recreate are those whose count of c is
// (current count + 1): the per-game table (open addressing, linear probing, 8-byte entries = the two keys) holds
// every position twice, once on the probe chain of (black, its black count) and once on that of (white, its white
// count).  Per ply that costs one chain walk to find where the new position goes and one for the next mover's
// forbidden plays.  The latter needs no loop over the legal points: an earlier position q can be recreated by the
// mover's play on p only if q's key of the mover's colour differs from the current one by exactly the key of a stone
// on p, and the stone keys come from an invertible mixer, so every lane inverts the difference of the entry it holds
// and sees at once whether it is a stone key at all (a random 32-bit value is one with probability 2^-22).  Only for
// such an entry -- a genuine near-repetition -- is the rest checked: the other colour's keys must differ by nothing
// (a play that takes nothing) or by exactly the keys of the chains the play takes.  The forbidden plays found when a
// position arises are kept with the game (two points, or a marker to look again), so the next ply's legality gate
// and the getters need no table access.
// Equality of positions = equality of the 64 key bits; the empty board (keys 0,0 = an empty slot) is never stored
// and can never be recreated.
// ------------------------------------------------------------------------------------------------
template <int N>
struct Zt {
  static constexpr int LOG2 = N == 19 ? 11 : 9;
  static constexpr uint32_t SLOTS = 1u << LOG2;
  static constexpr uint32_t MASK = SLOTS - 1u;
  static constexpr uint32_t WIN = N >= 16 ? 16u : 8u;   // slots a board's row lanes look at per round: one aligned 128- or 64-byte piece of the table
  static_assert(SLOTS > 2u * (2u * N * N + 9u), "two entries per position (ply cap + the imported history window) always leave empty slots");
};

// key of a stone: an invertible function of 2*point + colour + 1 (colour 0 black / 1 white)
__device__ __forceinline__ uint32_t zkey(uint32_t point, uint32_t colour) { return mixer(0x9E3779B9u * (2u * point + colour + 1u)); }
// 2*point + colour + 1 for a stone key, anything else for other values
__device__ __forceinline__ uint32_t zkey_inverse(uint32_t x) {
  x ^= x >> 16; x *= 0x43021123u;               // the mixer's steps undone in reverse order (odd multipliers are invertible mod 2^32)
  x ^= (x >> 15) ^ (x >> 30); x *= 0x1d69e2a5u;
  x ^= x >> 16;
  return x * 0x144cbc89u;                        // 0x9E3779B9^-1
}

// Keys (x: black stones, y: white stones) and stone counts of a game's current position, and the plays that would
// recreate an earlier position (fw: two points in 16 bits each, kNoPoint = none; kLookAgain in the low half = more than
// two, to be found by walking the table again).  The same in every lane of the board.
struct SkGame {
  uint2 key;
  int nb, nw;
  uint32_t fw;
};
constexpr uint32_t kNoPoint = 0xFFFFu, kLookAgain = 0xFFFEu;
__device__ __forceinline__ SkGame sk_unpack(uint4 v) {
  SkGame g;
  g.key = make_uint2(v.x, v.y); g.nb = (int)(v.z & 0xFFFFu); g.nw = (int)(v.z >> 16); g.fw = v.w;
  return g;
}
__device__ __forceinline__ uint4 sk_pack(const SkGame& g) { return make_uint4(g.key.x, g.key.y, (uint32_t)g.nb | ((uint32_t)g.nw << 16), g.fw); }
__device__ __forceinline__ SkGame sk_fresh() {   // a game on the empty board
  SkGame g;
  g.key = make_uint2(0u, 0u); g.nb = 0; g.nw = 0; g.fw = kNoPoint | (kNoPoint << 16);
  return g;
}

// a table entry is the position's two keys; (0,0) is an empty slot
__device__ __forceinline__ bool sk_real(uint2 e) { return (e.x | e.y) != 0u; }
// start of the probe chain of the positions whose count of `colour` stones is `count`
template <int N>
__device__ __forceinline__ uint32_t sk_home(int colour, int count) {
  return (((uint32_t)(2 * count + colour + 1) * 0x9E3779B1u) >> (32 - Zt<N>::LOG2)) & ~(Zt<N>::WIN - 1u);
}
// the same for the play-time reading (mode 1), where a position has one entry, on the chain of its two stone counts
template <int N>
__device__ __forceinline__ uint32_t sk_home_counts(int nb, int nw) {
  return (((uint32_t)((nb << 10) + nw + 1) * 0x9E3779B1u) >> (32 - Zt<N>::LOG2)) & ~(Zt<N>::WIN - 1u);
}
// Table accesses go to the device-coherent level: a wavefront of the rollout kernel reads in a later ply what its own
// lanes wrote in an earlier one.
__device__ __forceinline__ uint2 tab_load(const uint2* p) {
  const unsigned long long v = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
__device__ __forceinline__ void tab_store(uint2* p, uint2 e) {
  __hip_atomic_store((unsigned long long*)p, (unsigned long long)e.x | ((unsigned long long)e.y << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// orders a wavefront's earlier global-memory accesses before its later ones as seen by its own lanes
__device__ __forceinline__ void wave_mem_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// XOR of the keys of the stones of row r: x over the black bits, y over the white bits
template <int N>
__device__ __forceinline__ uint2 row_keys(int r, uint32_t black, uint32_t white) {
  uint2 acc = make_uint2(0u, 0u);
  for (uint32_t d = black; d; d &= d - 1u) acc.x ^= zkey((uint32_t)(r * N + __ffs(d) - 1), 0u);
  for (uint32_t d = white; d; d &= d - 1u) acc.y ^= zkey((uint32_t)(r * N + __ffs(d) - 1), 1u);
  return acc;
}

// every lane of a board receives the XOR of v over the board's rows; scratch = 2*W dwords of the wavefront's LDS
template <int N>
__device__ __forceinline__ uint2 board_xor(const Lane<N>& L, uint2 v, uint32_t* scratch) {
  using G = Geo<N>;
  if (L.lane < 2 * G::W) scratch[L.lane] = 0u;
  wave_lds_fence();
  if (L.valid && (v.x | v.y) != 0u) { atomicXor(&scratch[2 * L.j], v.x); atomicXor(&scratch[2 * L.j + 1], v.y); }
  wave_lds_fence();
  uint2 out = make_uint2(0u, 0u);
  if (L.j < G::W) out = make_uint2(scratch[2 * L.j], scratch[2 * L.j + 1]);
  wave_lds_fence();
  return out;
}

// number of set bits of a board-wide set given by its row words, known to every lane of the board
template <int N>
__device__ __forceinline__ int board_popcount(const Lane<N>& L, uint32_t w) {
  const uint32_t v = __popc(w);
  int sum = 0;
#pragma unroll
  for (int k = 0; (1 << k) <= N; ++k) {
    const uint64_t mk = __ballot((v >> k) & 1u);
    sum += (__popc((uint32_t)mk & L.seglo) + __popc((uint32_t)(mk >> 32) & L.seghi)) << k;
  }
  return sum;
}

// The WIN table slots from `home` on, one per row lane, loaded ahead of their use (home = ~0u: nothing loaded)
struct SkWin {
  uint32_t home;
  uint2 e;
};
template <int N>
__device__ __forceinline__ SkWin sk_window(const Lane<N>& L, const uint2* tab, uint32_t home, bool want) {
  SkWin w;
  w.home = want ? home : ~0u;
  w.e = make_uint2(1u, 0u);   // neither empty nor a real entry
  if (L.valid && want && (uint32_t)L.r < Zt<N>::WIN) w.e = tab_load(&tab[(home + (uint32_t)L.r) & Zt<N>::MASK]);
  return w;
}

// Walks the probe chain that starts at `home` (the same for every lane of a board; active = this board takes part),
// WIN slots per round, one per row lane, until the chain's first empty slot.  visit(e, look) is called once per round
// by every lane of the wavefront with the lane's entry (look = the lane holds a slot of an active board's chain).
// free_slot = the first empty slot other than `taken` (a slot this ply has filled already; ~0u = none); ok = found,
// which is always the case since the table is never full.  pre: a window loaded earlier, used when it starts at `home`.
template <int N, class V>
__device__ __forceinline__ void sk_walk(const Lane<N>& L, const uint2* tab, uint32_t home, bool active, const SkWin& pre, uint32_t taken, V&& visit,
                                        bool& ok, uint32_t& free_slot) {
  using G = Geo<N>;
  constexpr uint32_t WIN = Zt<N>::WIN;
  const uint64_t seg = ((uint64_t)L.seghi << 32) | L.seglo;
  ok = false; free_slot = 0u;
  bool done = !active;
  uint32_t base = home;
  for (uint32_t round = 0; round < Zt<N>::SLOTS / WIN + 1u; ++round) {
    if (__ballot(!done) == 0ull) break;
    const bool look = L.valid && (uint32_t)L.r < WIN && !done;
    uint2 e = make_uint2(1u, 0u);
    const uint32_t slot = (base + (uint32_t)L.r) & Zt<N>::MASK;
    const bool from_pre = round == 0u && pre.home == base;
    if (look && from_pre) e = pre.e;
    if (__ballot(look && !from_pre) != 0ull) {   // a branch of the whole wavefront: most walks end in the window loaded ahead
      if (look && !from_pre) e = tab_load(&tab[slot]);
      // the wait for this load stays inside the branch: after it, it would also be a wait for the caller's output stores
      asm volatile("" : "+v"(e.x), "+v"(e.y));
    }
    if (look && slot == taken && (e.x | e.y) == 0u) e = make_uint2(1u, 0u);
    visit(e, look);
    const uint64_t em = __ballot(look && (e.x | e.y) == 0u) & seg;
    if (!done) {
      if (em) { free_slot = (base + (uint32_t)(__ffsll((long long)em) - 1 - (L.j * G::STRIDE + 1))) & Zt<N>::MASK; ok = true; done = true; }
      else base += WIN;
    }
  }
}

// What placing a stone does to the game's key set (the same in every lane of the board).
struct SkPly {
  uint2 key;        // keys and counts of the position after the ply (meaningful for a board that placed a stone)
  int nb, nw;
  bool ok;          // free_a is valid
  uint32_t free_a;  // where the position goes on the chain of the mover's colour
};

// After the rules have been applied to a board that placed a stone (colour c, stones `captured` taken): the new
// position's keys and counts, and the free slot on its first chain.
template <int N>
__device__ __forceinline__ SkPly sk_look(const Lane<N>& L, const uint2* tab, const SkGame& g, int c, const Move& mv, uint32_t captured,
                                         const SkWin& pre, uint32_t* scratch) {
  SkPly s;
  const bool played = mv.playing;
  const uint32_t kp = zkey((uint32_t)(played ? mv.pr * N + mv.pc : 0), (uint32_t)c);
  int ncap = 0;
  uint2 dk = make_uint2(0u, 0u);
  if (__ballot(captured != 0u) != 0ull) {   // the captured stones have the other colour
    ncap = board_popcount<N>(L, captured);
    dk = board_xor<N>(L, row_keys<N>(L.r, c ? captured : 0u, c ? 0u : captured), scratch);
  }
  const int own1 = (c ? g.nw : g.nb) + 1, opp1 = (c ? g.nb : g.nw) - ncap;
  s.key = make_uint2(g.key.x ^ (c ? 0u : kp) ^ dk.x, g.key.y ^ (c ? kp : 0u) ^ dk.y);
  s.nb = c ? opp1 : own1; s.nw = c ? own1 : opp1;
  sk_walk<N>(L, tab, sk_home<N>(c, own1), played, pre, ~0u, [](uint2, bool) {}, s.ok, s.free_a);
  return s;
}

// Writes the position of a board that placed a stone into the table (both chains) and makes it the game's current one.
// tab_r: the table the chains are read from; tab_w: the one the entries go to (they differ only while the slot kernel
// copies a game from one slot to another).
template <int N>
__device__ __forceinline__ void sk_insert(const Lane<N>& L, const uint2* tab_r, uint2* tab_w, SkGame& g, const SkPly& s, bool insert, int c,
                                          const SkWin& pre) {
  if (__ballot(insert) == 0ull) return;
  bool ok_c;
  uint32_t free_c;
  const int opp1 = c ? s.nb : s.nw;   // count of the colour that did not move
  sk_walk<N>(L, tab_r, sk_home<N>(c ^ 1, opp1), insert, pre, s.ok ? s.free_a : ~0u, [](uint2, bool) {}, ok_c, free_c);
  if (insert) { g.key = s.key; g.nb = s.nb; g.nw = s.nw; }
  if (insert && L.valid && L.r == 0 && sk_real(s.key)) {
    if (s.ok) tab_store(&tab_w[s.free_a], s.key);
    if (ok_c) tab_store(&tab_w[free_c], s.key);
  }
  wave_mem_fence();
}

// Whether the mover's (colour c2) play on point p would recreate the earlier position whose keys differ from the
// current ones by d_other in the other colour (on = this board has such a candidate); returns the play as row words.
template <int N>
__device__ __forceinline__ uint32_t sk_forbidden_play(const Lane<N>& L, const Row<N>& R, int c2, int p, uint32_t d_other, bool on, uint32_t legal_s,
                                                      uint32_t* scratch) {
  const int pr = on ? p / N : -100, pc = on ? p - (p / N) * N : 0;
  const uint32_t pb = (L.valid && L.r == pr) ? (1u << pc) : 0u;
  const bool legal = on && board_any((legal_s & pb) != 0u, L.seglo, L.seghi);   // an occupied, suicidal or ko point is out anyway
  const uint32_t aopp = c2 ? R.ab : R.aw;
  const uint32_t seed = legal ? (dilate(pb) & aopp) : 0u;    // the opposing chains in atari next to the play are what it takes
  const bool takes = board_any(seed != 0u, L.seglo, L.seghi);
  uint32_t kt = 0u;
  if (__ballot(takes) != 0ull) {
    const uint32_t taken = flood_plain(seed, aopp);
    const uint2 k = board_xor<N>(L, row_keys<N>(L.r, c2 ? taken : 0u, c2 ? 0u : taken), scratch);
    kt = c2 ? k.x : k.y;
  }
  return (legal && kt == d_other) ? pb : 0u;
}

// The plays of the player to move that would recreate an earlier position of the game (row words): one walk of the
// chain of the positions with one more stone of the mover's colour than now.
template <int N>
__device__ __forceinline__ uint32_t sk_forbidden(const Lane<N>& L, const uint2* tab, const SkGame& g, const Row<N>& R, const Meta& m, bool active,
                                                 const SkWin& pre, uint32_t* scratch) {
  uint32_t forb = 0u;
  if (__ballot(active) == 0ull) return forb;
  const uint64_t seg = ((uint64_t)L.seghi << 32) | L.seglo;
  const int c2 = m.wtm, n2 = c2 ? g.nw : g.nb;
  bool ok;
  uint32_t fs;
  sk_walk<N>(L, tab, sk_home<N>(c2, n2 + 1), active, pre, ~0u,
             [&](uint2 e, bool look) {
               // is (entry xor current) in the mover's colour the key of one stone of that colour?
               const uint32_t u = zkey_inverse(c2 ? e.y ^ g.key.y : e.x ^ g.key.x) - 1u;   // 2*point + colour for a stone key
               const uint32_t d_other = c2 ? e.x ^ g.key.x : e.y ^ g.key.y;
               uint64_t pend = __ballot(look && sk_real(e) && u < 2u * N * N && (int)(u & 1u) == c2);
               if (pend == 0ull) return;          // nearly always: no earlier position is one stone of the mover's away
               const uint32_t legal_s = legal_row<N>(L, R, m.wtm, m.ko);
               while (pend != 0ull) {             // one candidate per board per turn
                 const uint64_t mine = pend & seg;
                 const bool on = mine != 0ull;
                 const int src = on ? (__ffsll((long long)mine) - 1) : L.lane;
                 const int p = __shfl((int)(u >> 1), src);
                 const uint32_t dq = (uint32_t)__shfl((int)d_other, src);
                 pend &= ~__ballot(on && L.lane == src);
                 forb |= sk_forbidden_play<N>(L, R, c2, p, dq, on, legal_s, scratch);
               }
             },
             ok, fs);
  return forb;
}

// the forbidden plays kept with a game -> row words of this lane's board
template <int N>
__device__ __forceinline__ uint32_t sk_forb_rows(const Lane<N>& L, uint32_t fw) {
  const uint32_t p1 = fw & 0xFFFFu, p2 = fw >> 16;
  uint32_t out = 0u;
  if (L.valid && p1 < (uint32_t)(N * N) && (int)(p1 / N) == L.r) out |= 1u << (p1 % N);
  if (L.valid && p2 < (uint32_t)(N * N) && (int)(p2 / N) == L.r) out |= 1u << (p2 % N);
  return out;
}
// row words -> the form kept with the game (the same in every lane of the board)
template <int N>
__device__ __forceinline__ uint32_t sk_forb_word(const Lane<N>& L, uint32_t forb) {
  using G = Geo<N>;
  uint32_t fw = kNoPoint | (kNoPoint << 16);
  if (__ballot(forb != 0u) == 0ull) return fw;   // nearly always
  const uint64_t seg = ((uint64_t)L.seghi << 32) | L.seglo;
  const int cnt = board_popcount<N>(L, forb);
  uint32_t rest = forb;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const uint64_t mine = __ballot(rest != 0u) & seg;
    const int src = mine ? (__ffsll((long long)mine) - 1) : L.lane;
    const int col = __shfl((int)(__ffs(rest) - 1), src);
    const uint32_t p = mine ? (uint32_t)((src - (L.j * G::STRIDE + 1)) * N + col) : kNoPoint;
    fw = k == 0 ? ((fw & 0xFFFF0000u) | p) : ((fw & 0xFFFFu) | (p << 16));
    if (L.lane == src) rest &= rest - 1u;
  }
  if (cnt > 2) fw = kLookAgain | (kNoPoint << 16);
  return fw;
}
// The forbidden plays of the position the kernel has just loaded: from the game's record, or (more than two of them
// were found when the position arose) by walking the table again.
template <int N>
__device__ __forceinline__ uint32_t sk_forb_loaded(const Lane<N>& L, const uint2* tab, const SkGame& g, const Row<N>& R, const Meta& m, const SkWin& pre,
                                                   uint32_t* scratch) {
  uint32_t forb = sk_forb_rows<N>(L, g.fw);
  const bool again = L.boardok && (g.fw & 0xFFFFu) == kLookAgain;
  if (__ballot(again) != 0ull) {
    const uint32_t f2 = sk_forbidden<N>(L, tab, g, R, m, again, pre, scratch);
    if (again) forb = f2;
  }
  return forb;
}

// all lanes of the wavefront clear the tables of the boards flagged by their row-0 lane (auto-reset); `game` = the
// index of this lane's board among the handle's tables
template <int N>
__device__ __forceinline__ void sk_clear_tables(const Lane<N>& L, bool flagged, uint2* zt, int game) {
  for (uint64_t q = __ballot(flagged && L.valid && L.r == 0); q; q &= q - 1ull) {
    const size_t bb = (size_t)__shfl(game, __ffsll((long long)q) - 1);
    uint4* t4 = (uint4*)(zt + bb * Zt<N>::SLOTS);
    for (uint32_t i = L.lane; i < Zt<N>::SLOTS / 2u; i += 64u) t4[i] = make_uint4(0u, 0u, 0u, 0u);
  }
  wave_mem_fence();
}

// Steps a2-a8 of one ply with the repetition rule for every board of the wavefront: the requested move passes the
// legality gate only if it is not one of the position's forbidden plays (`forb`, updated to those of the new position),
// the new position goes into the table, an auto-reset clears it.  tab_r / tab_w / game: see sk_insert, sk_clear_tables.
// GATE as in gate_move.  Out: as apply_move.
// board_final(hdirty) is called once the rows and scalars of the new position (an auto-reset included) are final: the
// caller emits the observation and may store the state there.  EARLY: before the table work, so that those stores are
// under way while the walks go on (measured: 25.1 -> 23.8 us per ply in the rollout kernel; in the one-launch-per-ply
// kernel it is 1 us slower than calling it afterwards, hence the choice).
template <int N, bool GATE, bool EARLY, class Hook>
__device__ __forceinline__ void sk_step_core(const Lane<N>& L, Row<N>& R, Meta& m, SkGame& g, uint32_t& forb, const Rules& rules, bool skip, bool want_pass,
                                             bool want_point, int pr_in, int pc_in, const uint2* tab_r, uint2* tab_w, uint2* zt, int game,
                                             uint32_t* scratch, float& rew0, float& rew1, bool& flag, bool pre_a_loaded, const SkWin& pre_a,
                                             Hook&& board_final) {   // board_final(hdirty): hdirty as from apply_move
  const int c = m.wtm, own = c ? g.nw : g.nb, opp = c ? g.nb : g.nw;
  Move mv = gate_move<N, GATE>(L, R, m, skip, want_pass, want_point, pr_in, pc_in);
  // a play the simple rules allow but the repetition rule forbids is an illegal action
  const uint32_t pbit = (L.valid && mv.playing && L.r == mv.pr) ? (1u << mv.pc) : 0u;
  const bool repeats = mv.playing && board_any((pbit & forb) != 0u, L.seglo, L.seghi);
  if (repeats) { mv.playing = false; mv.illegal = true; mv.pr = -100; mv.pc = 0; }
  // The chains this ply needs start at slots known before the rules run when the move takes nothing (most do): the
  // loads fly while the rules run.  pre[0]: one more stone of the mover's colour (where the new position goes);
  // pre[1]: one more stone of the other colour (the next mover's forbidden plays); pre[2]: as many stones of the
  // other colour as now (the new position's second entry).
  SkWin pre[3];
  if (pre_a_loaded) pre[0] = pre_a;
  else pre[0] = sk_window<N>(L, tab_r, sk_home<N>(c, own + 1), mv.playing);
  pre[1] = sk_window<N>(L, tab_r, sk_home<N>(c ^ 1, opp + 1), mv.playing || mv.is_pass);
  pre[2] = sk_window<N>(L, tab_r, sk_home<N>(c ^ 1, opp), mv.playing);
  Rules r0 = rules;
  r0.auto_reset = 0;   // the reset happens below, after the table work
  bool reset;
  uint32_t captured;
  uint32_t hdirty;
  apply_move<N>(L, R, m, r0, mv, rew0, rew1, flag, captured, reset, hdirty);
  const bool do_reset = !skip && !mv.frozen && m.term && rules.auto_reset != 0;
  if (do_reset) { reset_board<N>(L, R, m, rules.seed); hdirty = ~0u; }   // a board that is reset takes no part in the table work below
  if constexpr (EARLY) {
    // The windows have to be in registers before the caller's stores are issued: loads and stores share one counter,
    // and a wait for these loads placed after the stores would wait for the stores as well.
    asm volatile("" ::"v"(pre[0].e.x), "v"(pre[0].e.y), "v"(pre[1].e.x), "v"(pre[1].e.y), "v"(pre[2].e.x), "v"(pre[2].e.y));
    board_final(hdirty);
  }
  const SkPly s = sk_look<N>(L, tab_r, g, c, mv, captured, pre[0], scratch);
  sk_insert<N>(L, tab_r, tab_w, g, s, mv.playing && !do_reset, c, pre[2]);
  // the forbidden plays change with the position and with the player to move; otherwise they stay
  const bool moved = (mv.playing || mv.is_pass) && !do_reset;
  const uint32_t fresh = sk_forbidden<N>(L, tab_r, g, R, m, moved, pre[1], scratch);
  if (moved) forb = fresh;
  if (do_reset) { g = sk_fresh(); forb = 0u; }
  sk_clear_tables<N>(L, do_reset, zt, game);
  if constexpr (!EARLY) board_final(hdirty);
}

// The same for the reading in which the rule is looked at only for the move that is played (mode 1): no sets of
// forbidden plays are kept, and a position has ONE table entry, on the chain of its two stone counts (so that it is
// found whoever recreates it).  One table window read and one 8-byte store per game-ply instead of three and two.
// pre: the chain's first window for a play that takes nothing, loaded by the caller as early as it can (home = ~0u:
// not loaded).  Two orders:
//   POST = false (the rollout kernel, whose state lives in registers): the position the requested play would give is
//     known before the rules run -- it takes exactly the opposing chains in atari next to it -- so its keys are looked
//     up first; a hit turns the play into an illegal action.
//   POST = true (one launch per ply, where every wavefront would wait for the window before it can do anything else):
//     the rules run first, on the assumption that the play repeats nothing, board_final() is called (the observation is
//     under way), and the look-up follows; after a hit (rare) restore(R, m, which) brings back the state as loaded for
//     the boards flagged, the ply is applied again as an illegal action and board_final() is called once more: the
//     same wavefront overwrites what it stored the first time.
template <int N, bool GATE, bool POST, class Hook, class Restore>
__device__ __forceinline__ void sk_step_core_play(const Lane<N>& L, Row<N>& R, Meta& m, SkGame& g, const Rules& rules, bool skip, bool want_pass,
                                                  bool want_point, int pr_in, int pc_in, const uint2* tab_r, uint2* tab_w, uint2* zt, int game,
                                                  uint32_t* scratch, float& rew0, float& rew1, bool& flag, const SkWin& pre, Hook&& board_final,
                                                  Restore&& restore) {
  const int c = m.wtm, own1 = (c ? g.nw : g.nb) + 1;
  const uint64_t seg = ((uint64_t)L.seghi << 32) | L.seglo;
  Move mv = gate_move<N, GATE>(L, R, m, skip, want_pass, want_point, pr_in, pc_in);
  Rules r0 = rules;
  r0.auto_reset = 0;   // the reset happens below, together with the table's
  bool reset, do_reset = false;
  uint32_t captured = 0u, hdirty = 0u;
  if constexpr (POST) {
    apply_move<N>(L, R, m, r0, mv, rew0, rew1, flag, captured, reset, hdirty);
    do_reset = !skip && !mv.frozen && m.term && rules.auto_reset != 0;
    if (do_reset) { reset_board<N>(L, R, m, rules.seed); hdirty = ~0u; }
    // The window has to be in registers before the caller's stores are issued: loads and stores share one counter.
    asm volatile("" ::"v"(pre.e.x), "v"(pre.e.y));
    board_final(hdirty);   // on the assumption that nothing repeats; done again below if something does
  }
  // the stones the play takes: known from the rules (POST), else the opposing chains in atari next to it
  uint32_t taken = captured;
  if constexpr (!POST) {
    const uint32_t pbit = (L.valid && mv.playing && L.r == mv.pr) ? (1u << mv.pc) : 0u;
    const uint32_t aopp = c ? R.ab : R.aw;
    const uint32_t seed = dilate(pbit) & aopp;
    if (__ballot(seed != 0u) != 0ull) taken = flood_plain(seed, aopp);
  }
  int ncap = 0;
  uint2 dk = make_uint2(0u, 0u);
  if (__ballot(taken != 0u) != 0ull) {   // about one ply in ten
    ncap = board_popcount<N>(L, taken);
    dk = board_xor<N>(L, row_keys<N>(L.r, c ? taken : 0u, c ? 0u : taken), scratch);
  }
  const int opp1 = (c ? g.nb : g.nw) - ncap;
  const int nb1 = c ? opp1 : own1, nw1 = c ? own1 : opp1;
  const uint32_t kp = zkey((uint32_t)(mv.playing ? mv.pr * N + mv.pc : 0), (uint32_t)c);
  const uint2 key = make_uint2(g.key.x ^ (c ? 0u : kp) ^ dk.x, g.key.y ^ (c ? kp : 0u) ^ dk.y);
  bool hit = false, ok;
  uint32_t free_slot;
  sk_walk<N>(L, tab_r, sk_home_counts<N>(nb1, nw1), mv.playing, pre, ~0u,
             [&](uint2 e, bool look) { if ((__ballot(look && e.x == key.x && e.y == key.y) & seg) != 0ull) hit = true; }, ok, free_slot);
  const bool repeats = mv.playing && hit;
  if (repeats) { mv.playing = false; mv.illegal = true; mv.pr = -100; mv.pc = 0; }
  if constexpr (!POST) {
    apply_move<N>(L, R, m, r0, mv, rew0, rew1, flag, captured, reset, hdirty);
    do_reset = !skip && !mv.frozen && m.term && rules.auto_reset != 0;
    if (do_reset) { reset_board<N>(L, R, m, rules.seed); hdirty = ~0u; }
    board_final(hdirty);
  } else if (__ballot(repeats) != 0ull) {
    restore(R, m, repeats);   // the boards that repeat get the state as loaded back
    Move again = mv;          // the other boards of the wavefront keep what the first pass gave them: for them, a skipped ply
    if (!repeats) { again.skip = true; again.frozen = false; again.is_pass = false; again.playing = false; again.illegal = false; again.pr = -100; again.pc = 0; }
    float a0, a1;
    bool f2, rs2;
    uint32_t cap2, hd2;
    apply_move<N>(L, R, m, r0, again, a0, a1, f2, cap2, rs2, hd2);
    if (repeats) {
      rew0 = a0; rew1 = a1; flag = f2;
      do_reset = rules.auto_reset != 0;   // the illegal action has ended the game
      if (do_reset) reset_board<N>(L, R, m, rules.seed);
    }
    board_final(~0u);
  }
  if (mv.playing && !do_reset) {
    if (L.valid && L.r == 0 && ok && sk_real(key)) tab_store(&tab_w[free_slot], key);
    g.key = key; g.nb = nb1; g.nw = nw1;
  }
  if (do_reset) g = sk_fresh();
  wave_mem_fence();
  sk_clear_tables<N>(L, do_reset, zt, game);
}
// the window the next play of the game looks at first (mode 1), if that play takes nothing
template <int N>
__device__ __forceinline__ SkWin sk_window_play(const Lane<N>& L, const uint2* tab, const SkGame& g, const Meta& m, bool want) {
  return sk_window<N>(L, tab, sk_home_counts<N>(g.nb + (m.wtm ? 0 : 1), g.nw + (m.wtm ? 1 : 0)), want);
}

// One ply with the repetition rule.  Same steps as go_step_kernel.
// MODE: 1 = the rule is looked at when the move is played, 2 = honoured by the legal mask
template <int N, bool TIGHT, int ST, int MODE>
__global__ void __launch_bounds__(64 * kWavesPerBlock, 6) go_step_superko_kernel(StepArgs a, uint2* zt, uint4* zcur) {
  using G = Geo<N>;
  __shared__ __attribute__((aligned(16))) uint32_t lds_obs_all[kWavesPerBlock][G::W * G::OBS_DW];
  __shared__ __attribute__((aligned(16))) uint32_t lds_mask_all[kWavesPerBlock][64];
  __shared__ uint2 lut[256];
  const int wib = wave_in_block();
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  const Lane<N> L(wave, threadIdx.x & 63, a.B, a.wb);
  const size_t rows_total = (size_t)a.B * N;
  Row<N> R;
  load_row<N>(a.planes, rows_total, L, R);
  const uint4 meta_raw = L.boardok ? a.meta[L.b] : make_uint4(0xFFFFFFFFu, 0u, 0u, 0u);
  const int act = L.boardok ? a.actions[L.b] : -1;
  const uint4 g_raw = zcur[L.boardok ? L.b : 0];   // (an unconditional load: a conditional one is waited for on the spot)
  const int32_t start_raw = (a.next_actions && L.boardok && a.start_t) ? a.start_t[L.b] : INT32_MIN;
  fill_spread_table(lut);   // (nothing loaded above is looked at before this barrier)
  if (wave * a.wb >= a.B) return;
  const bool wait_start = (int64_t)a.sample_t < (int64_t)held_back(start_raw);
  SkGame g = L.boardok ? sk_unpack(g_raw) : sk_fresh();
  Meta m = unpack_meta(meta_raw);
  uint2* tab = zt + (size_t)(L.boardok ? L.b : 0) * Zt<N>::SLOTS;

  const bool skip = !L.boardok || act == -1;
  const bool in_range = act >= 0 && act < G::P;
  const int pr = in_range ? act / N : 0, pc = in_range ? act - (act / N) * N : 0;
  SkWin none;
  none.home = ~0u; none.e = make_uint2(1u, 0u);
  uint32_t forb = 0u;
  float rew0, rew1;
  bool flag;
  auto store_state = [&]() {   // a11 (whole rows: writing only the changed planes gains nothing here)
    if (!skip) {
      store_row<N>(a.planes, rows_total, L, R);
      if (L.valid && L.r == 0) a.meta[L.b] = pack_meta(m);
    }
  };
  auto board_final = [&](uint32_t) {   // a10, a11
    if (a.obs) emit_obs<N, TIGHT, ST>(L, R.h, m.wtm, wave, a.B, a.obs, a.obs_pitch, lds_obs_all[wib], lut, a.wb);
    if constexpr (MODE != 1) store_state();
  };
  if constexpr (MODE == 1) {
    const SkWin pre = sk_window_play<N>(L, tab, g, m, !skip);
    sk_step_core_play<N, true, true>(L, R, m, g, a.rules, skip, act == G::P, in_range, pr, pc, tab, tab, zt, L.b, lds_mask_all[wib], rew0, rew1, flag, pre,
                                     board_final, [&](Row<N>& Rr, Meta& mr, bool which) {   // the state is stored below: memory still holds it as loaded
                                       Row<N> T;
                                       load_row<N>(a.planes, rows_total, L, T);
                                       if (which) { Rr = T; mr = unpack_meta(meta_raw); }
                                     });
    store_state();
  } else {
    forb = sk_forb_loaded<N>(L, tab, g, R, m, none, lds_mask_all[wib]);
    sk_step_core<N, true, false>(L, R, m, g, forb, a.rules, skip, act == G::P, in_range, pr, pc, tab, tab, zt, L.b, lds_mask_all[wib], rew0, rew1, flag,
                                 false, none, board_final);
    g.fw = sk_forb_word<N>(L, forb);
  }
  if (!skip && L.valid && L.r == 0) {
    *(float2*)(a.rew + 2 * (size_t)L.b) = make_float2(rew0, rew1);
    a.term[L.b] = (uint8_t)(flag ? 1 : 0);
  }

  const uint32_t legal = legal_row<N>(L, R, m.wtm, m.ko) & ~(MODE == 2 ? forb : 0u);
  if (a.mask) emit_mask<N, TIGHT, ST>(L, legal, wave, a.B, a.mask, a.mask_pitch, lds_mask_all[wib], lut, a.wb);
  if (!skip && L.valid && L.r == 0) zcur[L.b] = sk_pack(g);
  if (a.next_actions) {
    const Draw<N> dr = draw_action<N>(L, legal, a.sample_seed, a.sample_t, wait_start);
    if (L.valid && L.r == 0) a.next_actions[L.b] = dr.action();
  }
}

// Fills the tables from what the state still carries: the 8 history positions and the current one (set-up, import),
// and finds the current position's forbidden plays.  The tables must have been cleared by an earlier launch.
template <int N>
__global__ void __launch_bounds__(64) go_superko_rebuild_kernel(const uint4* planes, const uint4* meta, int B, uint2* zt, uint4* zcur, int mode) {
  __shared__ uint32_t scratch[64];
  const Lane<N> L(blockIdx.x, threadIdx.x, B);
  Row<N> R;
  load_row<N>(planes, (size_t)B * N, L, R);
  const Meta m = unpack_meta(L.boardok ? meta[L.b] : make_uint4(0xFFFFFFFFu, 0u, 0u, 0u));
  uint2* tab = zt + (size_t)(L.boardok ? L.b : 0) * Zt<N>::SLOTS;
  SkWin none;
  none.home = ~0u; none.e = make_uint2(1u, 0u);
  SkGame g = sk_fresh();
  for (int i = 8; i >= 0; --i) {   // history position i-1 (oldest first), then i = 0: the current stones
    uint32_t black = R.bk, white = R.wt;
    if (i > 0) {
      black = 0u; white = 0u;
#pragma unroll
      for (int col = 0; col < N; ++col) {
        const uint32_t hw = (R.h[col >> 1] >> ((col & 1) * 16)) & 0xFFFFu;
        black |= ((hw >> (2 * (i - 1))) & 1u) << col;
        white |= ((hw >> (2 * (i - 1) + 1)) & 1u) << col;
      }
    }
    uint2 k = make_uint2(0u, 0u);
    if (L.valid) k = row_keys<N>(L.r, black, white);
    g.key = board_xor<N>(L, k, scratch);
    g.nb = board_popcount<N>(L, black); g.nw = board_popcount<N>(L, white);
    const uint2 entry = g.key;
    bool hit = false, ok_a, ok_b = false;
    uint32_t free_a, free_b = 0u;
    // mode 1: one entry on the chain of the two counts; mode 2: one on the chain of each colour's count
    sk_walk<N>(L, tab, mode == 1 ? sk_home_counts<N>(g.nb, g.nw) : sk_home<N>(0, g.nb), L.boardok, none, ~0u,
               [&](uint2 e, bool look) { hit = hit || (look && e.x == entry.x && e.y == entry.y); }, ok_a, free_a);
    const bool found = board_any(hit, L.seglo, L.seghi) || !sk_real(entry);   // the empty board is never stored
    if (mode != 1) sk_walk<N>(L, tab, sk_home<N>(1, g.nw), L.boardok && !found, none, ok_a ? free_a : ~0u, [](uint2, bool) {}, ok_b, free_b);
    if (L.valid && L.r == 0) {
      if (!found && ok_a) tab_store(&tab[free_a], entry);
      if (!found && ok_b) tab_store(&tab[free_b], entry);
    }
    __threadfence();   // the next round's look-ups must see these inserts
  }
  if (mode != 1) g.fw = sk_forb_word<N>(L, sk_forbidden<N>(L, tab, g, R, m, L.boardok, none, scratch));
  if (L.valid && L.r == 0) zcur[L.b] = sk_pack(g);
}

__global__ void go_zero_kernel(uint4* p, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// ------------------------------------------------------------------------------------------------
// the slot kernel (tree search): entry i reads the state of slot src[i], applies actions[i] (all -1 when
// actions is null: a plain copy) and writes the result to slot dst[i]; outputs go to row i.
// ------------------------------------------------------------------------------------------------
struct SlotArgs {
  uint4* planes;
  uint4* meta;
  int pool;             // number of state slots (the handle's batch)
  int n;                // entries of this call
  const int32_t* src;
  const int32_t* dst;
  const int32_t* actions;
  float* rew;           // [n][2] or null
  uint8_t* term;        // [n] or null; 255 marks an entry whose slot index was out of range
  uint8_t* mask;        // [n][mask_pitch] or null
  uint8_t* obs;         // [n][obs_pitch] or null
  int64_t mask_pitch, obs_pitch;
  Rules rules;
  uint2* zt;            // positional superko (SK kernels): per-slot tables, per-slot current keys, mode 1 / 2
  uint4* zcur;
  int sk_mode;
};

// SK: the positional-superko rule is on; a game that moves to another slot takes its key table along.
template <int N, bool TIGHT, int SK, int ST = kStorePlain>
__global__ void __launch_bounds__(64 * kWavesPerBlock, SK ? 4 : 6) go_step_slots_kernel(SlotArgs a) {
  using G = Geo<N>;
  __shared__ __attribute__((aligned(16))) uint32_t lds_obs_all[kWavesPerBlock][G::W * G::OBS_DW];
  __shared__ __attribute__((aligned(16))) uint32_t lds_mask_all[kWavesPerBlock][64];
  __shared__ uint2 lut[256];
  const int wib = wave_in_block();
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  Lane<N> L(wave, threadIdx.x & 63, a.n);
  const size_t rows_total = (size_t)a.pool * N;
  const int src = L.boardok ? a.src[L.b] : 0, dst = L.boardok ? a.dst[L.b] : 0;
  const bool in_pool = src >= 0 && src < a.pool && dst >= 0 && dst < a.pool;
  const bool bad = L.boardok && !in_pool;
  if (bad) { L.boardok = false; L.valid = false; L.full = 0u; }   // the entry becomes inert: no state access, no outputs
  L.slot = src;
  Row<N> R;
  load_row<N>(a.planes, rows_total, L, R);
  const uint4 meta_raw = L.boardok ? a.meta[src] : make_uint4(0xFFFFFFFFu, 0u, 0u, 0u);
  const int act = (L.boardok && a.actions) ? a.actions[L.b] : -1;
  fill_spread_table(lut);
  if (wave * G::W >= a.n) return;
  Meta m = unpack_meta(meta_raw);
  L.slot = dst;   // from here on the board is environment dst (seat draw on reset, state store)

  const bool skip = !L.boardok || act == -1;
  const bool in_range = act >= 0 && act < G::P;
  const int pr = in_range ? act / N : 0, pc = in_range ? act - (act / N) * N : 0;
  float rew0, rew1;
  bool flag;
  uint32_t forb = 0u;
  if constexpr (!SK) {
    const Move mv = gate_move<N, true>(L, R, m, skip, act == G::P, in_range, pr, pc);
    bool reset;
    uint32_t captured;
    apply_move<N>(L, R, m, a.rules, mv, rew0, rew1, flag, captured, reset);
  } else {
    const int sslot = L.boardok ? src : 0, dslot = L.boardok ? dst : 0;
    SkGame g = L.boardok ? sk_unpack(a.zcur[sslot]) : sk_fresh();
    const uint2* tab_r = a.zt + (size_t)sslot * Zt<N>::SLOTS;   // nothing writes to a source slot's table during the call
    uint2* tab_w = a.zt + (size_t)dslot * Zt<N>::SLOTS;
    for (uint64_t q = __ballot(L.valid && L.r == 0 && src != dst); q; q &= q - 1ull) {   // all lanes copy one table after the other
      const int ln = __ffsll((long long)q) - 1;
      const uint4* from = (const uint4*)(a.zt + (size_t)__shfl(sslot, ln) * Zt<N>::SLOTS);
      uint4* to = (uint4*)(a.zt + (size_t)__shfl(dslot, ln) * Zt<N>::SLOTS);
      for (uint32_t i = L.lane; i < Zt<N>::SLOTS / 2u; i += 64u) to[i] = from[i];
    }
    __threadfence();   // the copied tables are in place before entries are added to them or they are cleared
    SkWin none;
    none.home = ~0u; none.e = make_uint2(1u, 0u);
    auto board_final = [&](uint32_t) { if (a.obs) emit_obs<N, TIGHT, ST>(L, R.h, m.wtm, wave, a.n, a.obs, a.obs_pitch, lds_obs_all[wib], lut); };
    if constexpr (SK == 1) {
      const SkWin pre = sk_window_play<N>(L, tab_r, g, m, !skip);
      sk_step_core_play<N, true, true>(L, R, m, g, a.rules, skip, act == G::P, in_range, pr, pc, tab_r, tab_w, a.zt, dslot, lds_mask_all[wib], rew0, rew1, flag, pre,
                                       board_final, [&](Row<N>& Rr, Meta& mr, bool which) {   // the source slot still holds the state as loaded
                                         Lane<N> Ls = L;
                                         Ls.slot = src;
                                         Row<N> T;
                                         load_row<N>(a.planes, rows_total, Ls, T);
                                         if (which) { Rr = T; mr = unpack_meta(meta_raw); }
                                       });
    } else {
      forb = sk_forb_loaded<N>(L, tab_r, g, R, m, none, lds_mask_all[wib]);
      sk_step_core<N, true, true>(L, R, m, g, forb, a.rules, skip, act == G::P, in_range, pr, pc, tab_r, tab_w, a.zt, dslot, lds_mask_all[wib], rew0, rew1, flag,
                                  false, none, board_final);
      g.fw = sk_forb_word<N>(L, forb);
    }
    if (L.valid && L.r == 0) a.zcur[dslot] = sk_pack(g);
    if constexpr (SK != 2) forb = 0u;   // the mask shows the simple-ko set unless the rule proper is on
  }
  if ((threadIdx.x & 63) == L.j * G::STRIDE + 1 && L.j < G::W && L.b < a.n) {   // row-0 lane of the entry, inert or not
    if (bad) { if (a.term) a.term[L.b] = 255; }
    else {
      // a copied entry (action -1) reports what a skipped step reports for a fresh handle: no reward, and its terminated state
      if (a.rew) *(float2*)(a.rew + 2 * (size_t)L.b) = skip ? make_float2(0.f, 0.f) : make_float2(rew0, rew1);
      if (a.term) a.term[L.b] = (uint8_t)(skip ? m.term : (flag ? 1 : 0));
    }
  }
  const uint32_t legal = legal_row<N>(L, R, m.wtm, m.ko) & ~forb;
  if constexpr (!SK) { if (a.obs) emit_obs<N, TIGHT, ST>(L, R.h, m.wtm, wave, a.n, a.obs, a.obs_pitch, lds_obs_all[wib], lut); }
  if (a.mask) emit_mask<N, TIGHT, ST>(L, legal, wave, a.n, a.mask, a.mask_pitch, lds_mask_all[wib], lut);
  store_row<N>(a.planes, rows_total, L, R);
  if (L.valid && L.r == 0) a.meta[dst] = pack_meta(m);
}

// ------------------------------------------------------------------------------------------------
// the rollout kernel: one launch = `steps` plies of uniform random legal play of every environment.  The
// state stays in registers between plies; each ply's outputs go to slice (i mod slices) of the caller's
// trajectory buffers.
// ------------------------------------------------------------------------------------------------
struct RolloutArgs {
  uint4* planes;
  uint4* meta;
  int B;
  int wb;               // boards per wavefront of this launch
  Rules rules;
  int steps, slices;
  uint32_t seed, t0;
  const int32_t* start_t;
  int32_t* actions;     // [slices][B] or null
  float* rew;           // [slices][B][2] or null
  uint8_t* term;        // [slices][B] or null
  uint8_t* mask;        // [slices][B][mask_pitch] or null
  uint8_t* obs;         // [slices][B][obs_pitch] or null
  int64_t mask_pitch, obs_pitch;
  uint2* zt;            // positional superko (SK kernels): per-game tables, per-game current keys, mode 1 / 2
  uint4* zcur;
  int sk_mode;
};

// SK: 0 = simple ko only, 1 / 2 = positional superko at play time / in the legal mask
template <int N, bool TIGHT, int SK>
__global__ void __launch_bounds__(64 * kWavesPerBlock, SK ? 4 : 6) go_rollout_kernel(RolloutArgs a) {
  using G = Geo<N>;
  __shared__ __attribute__((aligned(16))) uint32_t lds_obs_all[kWavesPerBlock][G::W * G::OBS_DW];
  __shared__ __attribute__((aligned(16))) uint32_t lds_mask_all[kWavesPerBlock][64];
  __shared__ uint2 lut[256];
  fill_spread_table(lut);
  const int wib = wave_in_block();
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  if (wave * a.wb >= a.B) return;
  const Lane<N> L(wave, threadIdx.x & 63, a.B, a.wb);
  const size_t rows_total = (size_t)a.B * N;

  Row<N> R;
  load_row<N>(a.planes, rows_total, L, R);
  Meta m = unpack_meta(L.boardok ? a.meta[L.b] : make_uint4(0xFFFFFFFFu, 0u, 0u, 0u));
  const int64_t start = (L.boardok && a.start_t) ? (int64_t)a.start_t[L.b] : INT64_MIN;
  uint32_t legal = legal_row<N>(L, R, m.wtm, m.ko);
  SkGame g = sk_fresh();
  uint2* tab = nullptr;
  uint32_t forb = 0u;
  if constexpr (SK) {
    if (L.boardok) g = sk_unpack(a.zcur[L.b]);
    tab = a.zt + (size_t)(L.boardok ? L.b : 0) * Zt<N>::SLOTS;
    SkWin none;
    none.home = ~0u; none.e = make_uint2(1u, 0u);
    if constexpr (SK != 1) forb = sk_forb_loaded<N>(L, tab, g, R, m, none, lds_mask_all[wib]);
    if constexpr (SK == 2) legal &= ~forb;
  }
  // mode 1: the window the next ply looks at, loaded one ply ahead
  SkWin ahead;
  ahead.home = ~0u; ahead.e = make_uint2(1u, 0u);
  if constexpr (SK == 1) ahead = sk_window_play<N>(L, tab, g, m, L.boardok);
  int slice = 0;
  for (int i = 0; i < a.steps; ++i) {   // the same trip count for every wavefront
    const uint32_t t = a.t0 + (uint32_t)i;
    const bool wait = (int64_t)t < start;
    const Draw<N> d = draw_action<N>(L, legal, a.seed, t, wait);
    const bool skip = !L.boardok || wait;
    float rew0, rew1;
    bool flag;
    if constexpr (!SK) {
      step_core<N, false>(L, R, m, a.rules, skip, d.pass, d.point, d.pr, d.pc, rew0, rew1, flag);
      legal = legal_row<N>(L, R, m.wtm, m.ko);
    } else {
      SkWin none;
      none.home = ~0u; none.e = make_uint2(1u, 0u);
      uint8_t* const obs_t = a.obs ? a.obs + (size_t)slice * a.B * a.obs_pitch : nullptr;
      auto board_final = [&](uint32_t) {
        if (obs_t) emit_obs<N, TIGHT, kStoreThroughWhole>(L, R.h, m.wtm, wave, a.B, obs_t, a.obs_pitch, lds_obs_all[wib], lut, a.wb);
      };
      if constexpr (SK == 1) {
        sk_step_core_play<N, false, false>(L, R, m, g, a.rules, skip, d.pass, d.point, d.pr, d.pc, tab, tab, a.zt, L.b, lds_mask_all[wib], rew0, rew1, flag,
                                           ahead, board_final, [](Row<N>&, Meta&, bool) {});
        ahead = sk_window_play<N>(L, tab, g, m, L.boardok);
      } else {
        sk_step_core<N, false, true>(L, R, m, g, forb, a.rules, skip, d.pass, d.point, d.pr, d.pc, tab, tab, a.zt, L.b, lds_mask_all[wib], rew0, rew1, flag, false,
                                     none, board_final);
      }
      legal = legal_row<N>(L, R, m.wtm, m.ko) & ~(SK == 2 ? forb : 0u);
    }
    const size_t sb = (size_t)slice * a.B;
    if (L.valid && L.r == 0) {
      const size_t e = sb + L.b;
      if (a.actions) a.actions[e] = d.action();
      // a waiting environment reports the values a skipped step call leaves behind at the start: zeros
      if (a.rew) *(float2*)(a.rew + 2 * e) = skip ? make_float2(0.f, 0.f) : make_float2(rew0, rew1);
      if (a.term) a.term[e] = (uint8_t)((!skip && flag) ? 1 : 0);
    }
    emit_outputs<N, TIGHT, kStoreThroughWhole>(L, R, legal, m.wtm, wave, a.B, a.mask ? a.mask + sb * a.mask_pitch : nullptr, a.mask_pitch,
                    (!SK && a.obs) ? a.obs + sb * a.obs_pitch : nullptr, a.obs_pitch, lds_mask_all[wib], lds_obs_all[wib], lut, a.wb);
    wave_lds_fence();
    slice = slice + 1 == a.slices ? 0 : slice + 1;
  }
  store_row<N>(a.planes, rows_total, L, R);
  if (L.valid && L.r == 0) a.meta[L.b] = pack_meta(m);
  if constexpr (SK) {
    if constexpr (SK != 1) g.fw = sk_forb_word<N>(L, forb);
    if (L.valid && L.r == 0) a.zcur[L.b] = sk_pack(g);
  }
}

// ------------------------------------------------------------------------------------------------
// auxiliary kernels
// ------------------------------------------------------------------------------------------------
// SK: the legal mask leaves out the plays that would recreate an earlier position (positional superko, mode 2)
template <int N, bool TIGHT, bool SK>
__global__ void __launch_bounds__(64 * kWavesPerBlock) go_emit_kernel(const uint4* planes, const uint4* meta, int B, uint8_t* mask,
                                                                      int64_t mask_pitch, uint8_t* obs, int64_t obs_pitch, const uint2* zt,
                                                                      const uint4* zcur) {
  using G = Geo<N>;
  __shared__ __attribute__((aligned(16))) uint32_t lds_obs_all[kWavesPerBlock][G::W * G::OBS_DW];
  __shared__ __attribute__((aligned(16))) uint32_t lds_mask_all[kWavesPerBlock][64];
  __shared__ uint2 lut[256];
  fill_spread_table(lut);
  const int wib = wave_in_block();
  const int wave = piece_of_block() * kWavesPerBlock + wib;
  if (wave * G::W >= B) return;
  const Lane<N> L(wave, threadIdx.x & 63, B);
  Row<N> R;
  load_row<N>(planes, (size_t)B * N, L, R);
  Meta m = unpack_meta(L.boardok ? meta[L.b] : make_uint4(0xFFFFFFFFu, 0u, 0u, 0u));
  uint32_t legal = legal_row<N>(L, R, m.wtm, m.ko);
  if constexpr (SK) {
    if (mask) {
      const SkGame g = L.boardok ? sk_unpack(zcur[L.b]) : sk_fresh();
      SkWin none;
      none.home = ~0u; none.e = make_uint2(1u, 0u);
      legal &= ~sk_forb_loaded<N>(L, zt + (size_t)(L.boardok ? L.b : 0) * Zt<N>::SLOTS, g, R, m, none, lds_mask_all[wib]);
    }
  }
  emit_outputs<N, TIGHT>(L, R, legal, m.wtm, wave, B, mask, mask_pitch, obs, obs_pitch, lds_mask_all[wib], lds_obs_all[wib], lut);
}

// k-th legal action of the current position, same row-per-lane mapping as the step kernel
template <int N, bool SK>
__global__ void __launch_bounds__(64 * kWavesPerBlock) go_random_actions_kernel(const uint4* planes, const uint4* meta, int B, uint32_t seed,
                                                                                uint32_t t, const int32_t* start_t, int32_t* actions, const uint2* zt,
                                                                                const uint4* zcur) {
  using G = Geo<N>;
  __shared__ uint32_t sk_scratch[SK ? kWavesPerBlock : 1][64];
  const int wave = piece_of_block() * kWavesPerBlock + wave_in_block();
  if (wave * G::W >= B) return;
  const Lane<N> L(wave, threadIdx.x & 63, B);
  Row<N> R;
#pragma unroll
  for (int k = 0; k < G::HD; ++k) R.h[k] = 0u;
  R.bk = R.wt = R.ab = R.aw = 0u;
  if (L.valid) {   // stones and atari sets are the last four dwords of the row record
    const size_t idx = (size_t)L.b * N + L.r, rows_total = (size_t)B * N;
    uint32_t rec[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = G::HD + i;
      if (k < 4 * G::NQ) rec[i] = ((const uint32_t*)(planes + (size_t)(k / 4) * rows_total + idx))[k & 3];
      else rec[i] = ((const uint32_t*)(planes + (size_t)G::NQ * rows_total))[idx * G::REM + (k - 4 * G::NQ)];
    }
    R.bk = rec[0]; R.wt = rec[1]; R.ab = rec[2]; R.aw = rec[3];
  }
  Meta m = unpack_meta(L.boardok ? meta[L.b] : make_uint4(0xFFFFFFFFu, 0u, 0u, 0u));
  uint32_t legal = legal_row<N>(L, R, m.wtm, m.ko);
  if constexpr (SK) {
    const SkGame g = L.boardok ? sk_unpack(zcur[L.b]) : sk_fresh();
    SkWin none;
    none.home = ~0u; none.e = make_uint2(1u, 0u);
    legal &= ~sk_forb_loaded<N>(L, zt + (size_t)(L.boardok ? L.b : 0) * Zt<N>::SLOTS, g, R, m, none, sk_scratch[wave_in_block()]);
  }
  const bool wait = L.boardok && start_t && (int64_t)t < (int64_t)start_t[L.b];
  const Draw<N> d = draw_action<N>(L, legal, seed, t, wait);
  if (L.valid && L.r == 0) actions[L.b] = d.action();
}

// new episode for every environment: empty board, Black to move, seat from the hash
template <int N>
__global__ void go_reset_kernel(uint4* planes, uint4* meta, float* rew, uint8_t* term, int B, uint32_t seed, int first) {
  using G = Geo<N>;
  const size_t rows_total = (size_t)B * N;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows_total) {
#pragma unroll
    for (int k = 0; k < G::NQ; ++k) planes[(size_t)k * rows_total + i] = make_uint4(0u, 0u, 0u, 0u);
    uint32_t* tail = (uint32_t*)(planes + (size_t)G::NQ * rows_total);
#pragma unroll
    for (int k = 0; k < G::REM; ++k) tail[i * G::REM + k] = 0u;
  }
  if (i < (size_t)B) {
    Meta m;
    if (first) { m.episode = 0u; m.illegal = 0u; }
    else { Meta old = unpack_meta(meta[i]); m.episode = old.episode + 1u; m.illegal = old.illegal; }
    m.ko = -1; m.steps = 0; m.passes = 0; m.wtm = 0; m.term = 0;
    m.bp = (int)(env_hash(seed, 1u, (uint32_t)i, m.episode) & 1u);
    meta[i] = pack_meta(m);
    rew[2 * i] = 0.f; rew[2 * i + 1] = 0.f; term[i] = 0;
  }
}

template <int N>
__global__ void go_current_player_kernel(const uint4* meta, int B, uint8_t* dst) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  Meta m = unpack_meta(meta[b]);
  dst[b] = (uint8_t)(m.wtm ? 1 - m.bp : m.bp);
}

struct CanonArgs {
  int8_t* board; int8_t* history; int32_t* ko; int8_t* to_play; int32_t* steps; int8_t* passes;
  uint8_t* terminated; uint8_t* black_player; uint32_t* episode; uint32_t* illegal;
};

template <int N>
__global__ void __launch_bounds__(64) go_export_kernel(const uint4* planes, const uint4* meta, int B, CanonArgs c) {
  using G = Geo<N>;
  const Lane<N> L(blockIdx.x, threadIdx.x, B);
  Row<N> R;
  load_row<N>(planes, (size_t)B * N, L, R);
  if (!L.valid) return;
  const size_t cell0 = (size_t)L.b * G::P + (size_t)L.r * N;
#pragma unroll
  for (int col = 0; col < N; ++col) {
    if (c.board) c.board[cell0 + col] = (int8_t)((int)((R.bk >> col) & 1u) - (int)((R.wt >> col) & 1u));
    if (c.history) {
      uint32_t hw = (R.h[col >> 1] >> ((col & 1) * 16)) & 0xFFFFu;
      for (int i = 0; i < 8; ++i)
        c.history[((size_t)L.b * 8 + i) * G::P + (size_t)L.r * N + col] = (int8_t)((int)((hw >> (2 * i)) & 1u) - (int)((hw >> (2 * i + 1)) & 1u));
    }
  }
  if (L.r == 0) {
    Meta m = unpack_meta(meta[L.b]);
    if (c.ko) c.ko[L.b] = m.ko;
    if (c.to_play) c.to_play[L.b] = (int8_t)(m.wtm ? -1 : 1);
    if (c.steps) c.steps[L.b] = m.steps;
    if (c.passes) c.passes[L.b] = (int8_t)m.passes;
    if (c.terminated) c.terminated[L.b] = (uint8_t)m.term;
    if (c.black_player) c.black_player[L.b] = (uint8_t)m.bp;
    if (c.episode) c.episode[L.b] = m.episode;
    if (c.illegal) c.illegal[L.b] = m.illegal;
  }
}

// canonical arrays -> private state; the atari sets are rebuilt chain by chain
template <int N>
__global__ void __launch_bounds__(64) go_import_kernel(uint4* planes, uint4* meta, float* rew, uint8_t* term, int B, CanonArgs c) {
  using G = Geo<N>;
  const Lane<N> L(blockIdx.x, threadIdx.x, B);
  Row<N> R;
#pragma unroll
  for (int k = 0; k < G::HD; ++k) R.h[k] = 0u;
  R.bk = R.wt = R.ab = R.aw = 0u;
  Meta m;
  m.ko = -1; m.steps = 0; m.passes = 0; m.wtm = 0; m.term = 0; m.bp = 0; m.episode = 0u; m.illegal = 0u;
  if (L.boardok) {
    Meta old = unpack_meta(meta[L.b]);
    m.illegal = old.illegal;
    m.ko = c.ko[L.b]; m.wtm = c.to_play[L.b] < 0 ? 1 : 0; m.steps = c.steps[L.b] & 0xFFFF; m.passes = c.passes[L.b] & 3;
    m.term = c.terminated[L.b] ? 1 : 0; m.bp = c.black_player[L.b] & 1; m.episode = c.episode[L.b];
  }
  if (L.valid) {
    const size_t cell0 = (size_t)L.b * G::P + (size_t)L.r * N;
    for (int col = 0; col < N; ++col) {
      int v = c.board[cell0 + col];
      if (v > 0) R.bk |= 1u << col; else if (v < 0) R.wt |= 1u << col;
      uint32_t hw = 0u;
      for (int i = 0; i < 8; ++i) {
        int hv = c.history[((size_t)L.b * 8 + i) * G::P + (size_t)L.r * N + col];
        if (hv > 0) hw |= 1u << (2 * i); else if (hv < 0) hw |= 1u << (2 * i + 1);
      }
#pragma unroll
      for (int k = 0; k < G::HD; ++k) if (k == (col >> 1)) R.h[k] |= hw << ((col & 1) * 16);
    }
  }
  const uint32_t E = L.full & ~(R.bk | R.wt);
  uint32_t visited = 0u;
  for (;;) {
    // next unvisited stone of every board, its whole chain, its liberty class
    const uint32_t rest = (R.bk | R.wt) & ~visited;
    const uint64_t has = __ballot(rest != 0u);
    if (has == 0ull) break;
    const uint64_t mine = has & (((uint64_t)L.seghi << 32) | L.seglo);
    const bool first = mine != 0ull && (__ffsll((long long)mine) - 1) == L.lane;
    const uint32_t seed = first ? (rest & (0u - rest)) : 0u;
    const bool black = board_any((seed & R.bk) != 0u, L.seglo, L.seghi);
    const uint32_t F = flood_plain(seed, black ? R.bk : R.wt);
    bool one, two;
    board_count(dilate(F) & E, L.seglo, L.seghi, one, two);
    visited |= F;
    if (one) { if (black) R.ab |= F; else R.aw |= F; }
  }
  store_row<N>(planes, (size_t)B * N, L, R);
  if (L.valid && L.r == 0) {
    meta[L.b] = pack_meta(m);
    rew[2 * (size_t)L.b] = 0.f; rew[2 * (size_t)L.b + 1] = 0.f; term[L.b] = (uint8_t)m.term;
  }
}

__global__ void lane_shift_probe_kernel(const uint32_t* in, uint32_t* out) {
  uint32_t x = in[threadIdx.x];
  out[threadIdx.x] = from_lane_below(x);
  out[64 + threadIdx.x] = from_lane_above(x);
}

// Measurement helpers: a plain fill with 16-byte stores (the practical write ceiling of the machine on the same
// buffers the step kernel writes) and an empty kernel (the gap between dependent launches on one stream).
template <int ST>
__global__ void __launch_bounds__(256) fill_probe_kernel(uint4* __restrict__ dst, size_t n16, uint32_t value) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 16-byte store per thread
  if (i < n16) store16<ST>(&dst[i], make_uint2(value, value), make_uint2(value, value));
}
__global__ void empty_probe_kernel() {}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

template <int N>
size_t state_bytes_for(int B, size_t* off_meta, size_t* off_rew, size_t* off_term) {
  using G = Geo<N>;
  size_t o = 0;
  o += align_up((size_t)B * N * G::row_bytes, 256);
  if (off_meta) *off_meta = o;
  o += align_up((size_t)B * sizeof(uint4), 256);
  if (off_rew) *off_rew = o;
  o += align_up((size_t)B * 2 * sizeof(float), 256);
  if (off_term) *off_term = o;
  o += align_up((size_t)B, 256);
  return o;
}

}  // namespace

struct pgxgo_ctx {
  int B, N;
  int wb;        // boards per wavefront used by the step and rollout launches (1 .. W)
  uint32_t seed;
  int komi_x2, max_steps, auto_reset;
  int64_t obs_pitch, mask_pitch;
  hipStream_t stream;
  uint4* planes;
  uint4* meta;
  float* rew_int;
  uint8_t* term_int;
  uint8_t* mask_out;
  uint8_t* obs_out;
  float* rew_out;
  uint8_t* term_out;
  const uint8_t* mask_written;   // the buffers the last step (or bind) call wrote mask and observation to
  const uint8_t* obs_written;
  uint2* zt;     // positional superko: per-game key tables, or null when the rule is off
  uint4* zcur;   // key and stone counts of every game's current position
  int sk_mode;   // 0 off, 1 enforced when the move is played, 2 honoured by the legal mask
};

namespace {

template <int N>
int launch_reset(pgxgo_ctx* h, int first) {
  const size_t n = (size_t)h->B * N;
  const int threads = 256;
  const unsigned blocks = (unsigned)((n + threads - 1) / threads);
  hipLaunchKernelGGL(go_reset_kernel<N>, dim3(blocks), dim3(threads), 0, h->stream, h->planes, h->meta, h->rew_out, h->term_out, h->B, h->seed,
                     first);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

template <int N>
unsigned waves_for(int B) { return (unsigned)((B + Geo<N>::W - 1) / Geo<N>::W); }
template <int N>
unsigned blocks_for(int B) { return ((waves_for<N>(B) + kWavesPerBlock - 1) / kWavesPerBlock + 7u) & ~7u; }   // a multiple of 8: piece_of_block
unsigned blocks_for_wb(int B, int wb) { return (((unsigned)((B + wb - 1) / wb) + kWavesPerBlock - 1) / kWavesPerBlock + 7u) & ~7u; }

// Boards per wavefront for the step and rollout launches.  A wavefront can hold W boards; with few games it is
// better to spread them over more wavefronts (shorter floods, fewer output rounds per wavefront), so the count
// grows with the batch until about two wavefronts per SIMD exist.
// Kind of the output stores of a one-launch-per-ply kernel by the bytes the launch writes, measured at 19x19 with the
// observation: up to 32 MB (4096 games) everything written through the L2 is fastest (7.97 / 8.93 / 10.2 us per ply for
// 1024 / 2048 / 4096 games against 8.5 / 10.2 / 11.4 us with plain stores); from there to the size of the memory-side
// cache write-through for whole lines only (16384 games: 20.7 against 22.1 us); beyond it, where the hint costs
// 20-30 % below ~50 k games and gains 9-17 % above ~57 k, the non-temporal hint on top (65536 games: 88 us against
// 110 us plain).  The rollout kernel uses kStoreThroughWhole at every size (16384 games: 14.4 against 16.5 us per ply,
// 65536 games: 53.8 against 60.2 us; the non-temporal hint is slower there at every size).
// in_place: the launch overwrites the buffers the previous one wrote, whose lines are then still in the memory-side
// cache.  In the middle range a launch into other buffers (a caller that records a trajectory) has to reach DRAM and
// is faster with the hint as well (16384 games: 23.9 us per ply against 25.4 with ordinary stores and 25.9 with
// write-through alone).
constexpr size_t kWriteThroughUpTo = (size_t)32 << 20, kNonTemporalFrom = (size_t)350 << 20;
int store_kind_for(size_t out_bytes, bool in_place) {
  if (out_bytes <= kWriteThroughUpTo) return kStoreThrough;
  if (out_bytes <= kNonTemporalFrom) return in_place ? kStoreThroughWhole : kStoreStreamWhole;
  return kStoreStreamWhole;
}
size_t output_bytes_per_ply(const pgxgo_ctx* h, bool with_mask, bool with_obs) {
  return (size_t)h->B * ((with_mask ? (size_t)h->mask_pitch : 0) + (with_obs ? (size_t)h->obs_pitch : 0));
}

// One board per wavefront while every wavefront can have a SIMD to itself (1024 SIMDs), then as many boards per
// wavefront as keep it at one wavefront per SIMD, up to W (measured per ply, one launch per ply, best / worst choice:
// 9x9 x 2048 games 6.9 us with 2 boards against 7.5 with 1; x 4096 7.4 with 4 against 9.5 with 1; x 6144 7.7 with 6
// against 11.6 with 1; 19x19 x 3072 8.9 with 3 against 10.3 with 1).
template <int N>
int auto_boards_per_wavefront(int B) {
  const int want = (B + 1023) / 1024;
  return want < 1 ? 1 : (want > Geo<N>::W ? Geo<N>::W : want);
}

// both output pitches are the dense or the line-padded ones: the kernels treat a wavefront's boards as one run of bytes
// (with the line-padded pitch the pad bytes belong to that run and are written as zeros)
template <int N>
bool tight_pitches(const pgxgo_ctx* h) {
  using G = Geo<N>;
  return (h->mask_pitch == G::A || h->mask_pitch == G::A_PAD) && (h->obs_pitch == G::OBS || h->obs_pitch == G::OBS_PAD);
}

template <int N, bool TIGHT, bool SK>
void launch_emit_as(pgxgo_ctx* h, uint8_t* mask, uint8_t* obs) {
  hipLaunchKernelGGL((go_emit_kernel<N, TIGHT, SK>), dim3(blocks_for<N>(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, h->planes, h->meta, h->B, mask,
                     h->mask_pitch, obs, h->obs_pitch, h->zt, h->zcur);
}

template <int N>
int launch_emit(pgxgo_ctx* h, uint8_t* mask, uint8_t* obs) {
  const bool tight = tight_pitches<N>(h), sk = h->zt && h->sk_mode == 2;   // only then does the rule change the mask
  if (tight && sk) launch_emit_as<N, true, true>(h, mask, obs);
  else if (tight) launch_emit_as<N, true, false>(h, mask, obs);
  else if (sk) launch_emit_as<N, false, true>(h, mask, obs);
  else launch_emit_as<N, false, false>(h, mask, obs);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

template <int N>
int launch_step(pgxgo_ctx* h, const int32_t* actions, bool sample, uint32_t seed, uint32_t t, const int32_t* start_t, int32_t* next) {
  StepArgs a;
  a.planes = h->planes; a.meta = h->meta; a.actions = actions; a.rew = h->rew_out; a.term = h->term_out;
  a.mask = h->mask_out; a.obs = h->obs_out; a.mask_pitch = h->mask_pitch; a.obs_pitch = h->obs_pitch;
  a.B = h->B; a.wb = h->wb; a.rules.seed = h->seed; a.rules.komi_x2 = h->komi_x2; a.rules.max_steps = h->max_steps; a.rules.auto_reset = h->auto_reset;
  a.sample_seed = seed; a.sample_t = t; a.start_t = start_t; a.next_actions = next;
  // bytes one ply touches: state rows + outputs; 256 MB of memory-side cache on this part, keep a margin
  const size_t touched = (size_t)h->B * (Geo<N>::row_bytes * N + (h->mask_out ? (size_t)h->mask_pitch : 0) + (h->obs_out ? (size_t)h->obs_pitch : 0));
  a.sparse_store = touched < ((size_t)192 << 20) ? 1 : 0;
  a.store_kind = store_kind_for(output_bytes_per_ply(h, h->mask_out != nullptr, h->obs_out != nullptr),
                                h->mask_out == h->mask_written && h->obs_out == h->obs_written);
  h->mask_written = h->mask_out; h->obs_written = h->obs_out;
  const dim3 grid(blocks_for_wb(h->B, h->wb)), block(64 * kWavesPerBlock);
  const bool tight = tight_pitches<N>(h);
  if (h->zt) {
    if (!sample) a.next_actions = nullptr;
    auto sk = [&](auto tight_c, auto mode_c) {
      constexpr bool T = decltype(tight_c)::value;
      constexpr int M = decltype(mode_c)::value;
      if (a.store_kind == kStoreThrough) hipLaunchKernelGGL((go_step_superko_kernel<N, T, kStoreThrough, M>), grid, block, 0, h->stream, a, h->zt, h->zcur);
      else if (a.store_kind == kStoreThroughWhole) hipLaunchKernelGGL((go_step_superko_kernel<N, T, kStoreThroughWhole, M>), grid, block, 0, h->stream, a, h->zt, h->zcur);
      else hipLaunchKernelGGL((go_step_superko_kernel<N, T, kStoreStreamWhole, M>), grid, block, 0, h->stream, a, h->zt, h->zcur);
    };
    using M1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    if (tight && h->sk_mode == 1) sk(std::true_type{}, M1{});
    else if (tight) sk(std::true_type{}, M2{});
    else if (h->sk_mode == 1) sk(std::false_type{}, M1{});
    else sk(std::false_type{}, M2{});
    HIPCHK(hipGetLastError());
    return PGXGO_OK;
  }
  auto go = [&](auto sample_c, auto tight_c) {
    constexpr bool S = decltype(sample_c)::value, T = decltype(tight_c)::value;
    if (a.store_kind == kStoreThrough) hipLaunchKernelGGL((go_step_kernel<N, S, T, kStoreThrough>), grid, block, 0, h->stream, a);
    else if (a.store_kind == kStoreThroughWhole) hipLaunchKernelGGL((go_step_kernel<N, S, T, kStoreThroughWhole>), grid, block, 0, h->stream, a);
    else hipLaunchKernelGGL((go_step_kernel<N, S, T, kStoreStreamWhole>), grid, block, 0, h->stream, a);
  };
  if (sample && tight) go(std::true_type{}, std::true_type{});
  else if (sample) go(std::true_type{}, std::false_type{});
  else if (tight) go(std::false_type{}, std::true_type{});
  else go(std::false_type{}, std::false_type{});
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

template <int N>
int launch_random(pgxgo_ctx* h, uint32_t seed, uint32_t t, const int32_t* start_t, int32_t* actions) {
  if (h->zt && h->sk_mode == 2)
    hipLaunchKernelGGL((go_random_actions_kernel<N, true>), dim3(blocks_for<N>(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, h->planes, h->meta, h->B,
                       seed, t, start_t, actions, h->zt, h->zcur);
  else
    hipLaunchKernelGGL((go_random_actions_kernel<N, false>), dim3(blocks_for<N>(h->B)), dim3(64 * kWavesPerBlock), 0, h->stream, h->planes, h->meta, h->B,
                       seed, t, start_t, actions, h->zt, h->zcur);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

template <int N>
int launch_rollout(pgxgo_ctx* h, const RolloutArgs& a) {
  const dim3 grid(blocks_for_wb(h->B, h->wb)), block(64 * kWavesPerBlock);
  const bool tight = tight_pitches<N>(h), sk = h->zt != nullptr;
  if (tight && sk && h->sk_mode == 1) hipLaunchKernelGGL((go_rollout_kernel<N, true, 1>), grid, block, 0, h->stream, a);
  else if (tight && sk) hipLaunchKernelGGL((go_rollout_kernel<N, true, 2>), grid, block, 0, h->stream, a);
  else if (tight) hipLaunchKernelGGL((go_rollout_kernel<N, true, 0>), grid, block, 0, h->stream, a);
  else if (sk && h->sk_mode == 1) hipLaunchKernelGGL((go_rollout_kernel<N, false, 1>), grid, block, 0, h->stream, a);
  else if (sk) hipLaunchKernelGGL((go_rollout_kernel<N, false, 2>), grid, block, 0, h->stream, a);
  else hipLaunchKernelGGL((go_rollout_kernel<N, false, 0>), grid, block, 0, h->stream, a);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

template <int N>
int launch_slots(pgxgo_ctx* h, const SlotArgs& a) {
  const dim3 grid(blocks_for<N>(a.n)), block(64 * kWavesPerBlock);
  const bool tight = tight_pitches<N>(h), sk = h->zt != nullptr;
  const size_t out_bytes = (size_t)a.n * ((a.mask ? (size_t)a.mask_pitch : 0) + (a.obs ? (size_t)a.obs_pitch : 0));
  if (tight && sk && h->sk_mode == 1) hipLaunchKernelGGL((go_step_slots_kernel<N, true, 1>), grid, block, 0, h->stream, a);
  else if (tight && sk) hipLaunchKernelGGL((go_step_slots_kernel<N, true, 2>), grid, block, 0, h->stream, a);
  else if (tight && store_kind_for(out_bytes, true) == kStoreThrough) hipLaunchKernelGGL((go_step_slots_kernel<N, true, 0, kStoreThrough>), grid, block, 0, h->stream, a);
  else if (tight && store_kind_for(out_bytes, true) == kStoreThroughWhole) hipLaunchKernelGGL((go_step_slots_kernel<N, true, 0, kStoreThroughWhole>), grid, block, 0, h->stream, a);
  else if (tight) hipLaunchKernelGGL((go_step_slots_kernel<N, true, 0, kStoreStreamWhole>), grid, block, 0, h->stream, a);
  else if (sk && h->sk_mode == 1) hipLaunchKernelGGL((go_step_slots_kernel<N, false, 1>), grid, block, 0, h->stream, a);
  else if (sk) hipLaunchKernelGGL((go_step_slots_kernel<N, false, 2>), grid, block, 0, h->stream, a);
  else hipLaunchKernelGGL((go_step_slots_kernel<N, false, 0>), grid, block, 0, h->stream, a);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

template <int N>
int launch_export(pgxgo_ctx* h, const CanonArgs& c) {
  hipLaunchKernelGGL(go_export_kernel<N>, dim3(waves_for<N>(h->B)), dim3(64), 0, h->stream, h->planes, h->meta, h->B, c);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

template <int N>
int launch_import(pgxgo_ctx* h, const CanonArgs& c) {
  hipLaunchKernelGGL(go_import_kernel<N>, dim3(waves_for<N>(h->B)), dim3(64), 0, h->stream, h->planes, h->meta, h->rew_out, h->term_out, h->B,
                     c);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

template <int N>
size_t superko_bytes_for(int B, size_t* off_cur) {
  size_t o = align_up((size_t)B * Zt<N>::SLOTS * sizeof(uint2), 256);
  if (off_cur) *off_cur = o;
  return o + align_up((size_t)B * sizeof(uint4), 256);
}

// clears the tables, then (rebuild) fills them from the history window of the current state
template <int N>
int launch_superko_refresh(pgxgo_ctx* h, bool rebuild) {
  const size_t n16 = superko_bytes_for<N>(h->B, nullptr) / 16;
  const unsigned blocks = (unsigned)((n16 + 255) / 256 < 65536 ? (n16 + 255) / 256 : 65536);
  hipLaunchKernelGGL(go_zero_kernel, dim3(blocks), dim3(256), 0, h->stream, (uint4*)h->zt, n16);
  HIPCHK(hipGetLastError());
  if (rebuild) {
    hipLaunchKernelGGL(go_superko_rebuild_kernel<N>, dim3(waves_for<N>(h->B)), dim3(64), 0, h->stream, h->planes, h->meta, h->B, h->zt, h->zcur, h->sk_mode);
    HIPCHK(hipGetLastError());
  }
  return PGXGO_OK;
}

#define DISPATCH_N(h, call19, call9) ((h)->N == 19 ? (call19) : (call9))

// validates the arguments of an init call and fills the handle; launches nothing
int fill_ctx(pgxgo_ctx* h, int32_t batch, int32_t board_size, uint32_t seed, const pgxgo_opts* opts, void* state_dev, size_t state_bytes) {
  if (batch <= 0 || (board_size != 9 && board_size != 19) || !state_dev) return PGXGO_EINVAL;
  if (((uintptr_t)state_dev & 255u) != 0) return PGXGO_EINVAL;
  const int P = board_size * board_size;
  pgxgo_opts o;
  if (opts) o = *opts;
  else { o.komi_x2 = 15; o.max_steps = 0; o.auto_reset = 0; o.obs_pitch = 0; o.mask_pitch = 0; o.stream = nullptr; }
  if (o.max_steps == 0) o.max_steps = 2 * P;
  if (o.max_steps < 1 || o.max_steps > 65535) return PGXGO_EINVAL;
  if (o.obs_pitch == 0) o.obs_pitch = P * 17;
  if (o.mask_pitch == 0) o.mask_pitch = P + 1;
  if (o.obs_pitch < P * 17 || o.mask_pitch < P + 1) return PGXGO_EINVAL;
  size_t off_meta, off_rew, off_term;
  const size_t need = board_size == 19 ? state_bytes_for<19>(batch, &off_meta, &off_rew, &off_term)
                                       : state_bytes_for<9>(batch, &off_meta, &off_rew, &off_term);
  if (state_bytes < need) return PGXGO_EINVAL;
  *h = pgxgo_ctx{};
  h->B = batch; h->N = board_size; h->seed = seed;
  h->wb = board_size == 19 ? auto_boards_per_wavefront<19>(batch) : auto_boards_per_wavefront<9>(batch);
  h->komi_x2 = o.komi_x2; h->max_steps = o.max_steps; h->auto_reset = o.auto_reset ? 1 : 0;
  h->obs_pitch = o.obs_pitch; h->mask_pitch = o.mask_pitch;
  h->stream = (hipStream_t)o.stream;
  uint8_t* base = (uint8_t*)state_dev;
  h->planes = (uint4*)base;
  h->meta = (uint4*)(base + off_meta);
  h->rew_int = (float*)(base + off_rew);
  h->term_int = base + off_term;
  h->mask_out = nullptr; h->obs_out = nullptr; h->rew_out = h->rew_int; h->term_out = h->term_int;
  h->mask_written = nullptr; h->obs_written = nullptr;
  return PGXGO_OK;
}

// State of the handle made by pgxgo_init_static (callers that cannot allocate device memory).  In host code the
// array's name is only a stand-in: its device address comes from hipGetSymbolAddress, once per device.
constexpr int kMaxStaticDevices = 16;
void* g_scratch_ptr[kMaxStaticDevices] = {};
pgxgo_ctx g_static_ctx[kMaxStaticDevices] = {};

}  // namespace

static __device__ __align__(256) unsigned char scratch[PGXGO_STATIC_STATE_BYTES];

extern "C" {

size_t pgxgo_state_bytes(int32_t batch, int32_t board_size) {
  if (batch <= 0) return 0;
  if (board_size == 19) return state_bytes_for<19>(batch, nullptr, nullptr, nullptr);
  if (board_size == 9) return state_bytes_for<9>(batch, nullptr, nullptr, nullptr);
  return 0;
}

int32_t pgxgo_boards_per_wavefront(int32_t n) { return n == 19 ? Geo<19>::W : n == 9 ? Geo<9>::W : 0; }
int32_t pgxgo_num_actions(int32_t n) { return (n == 19 || n == 9) ? n * n + 1 : 0; }
int32_t pgxgo_obs_bytes(int32_t n) { return (n == 19 || n == 9) ? n * n * 17 : 0; }

int pgxgo_init(pgxgo_t* out, int32_t batch, int32_t board_size, uint32_t seed, const pgxgo_opts* opts, void* state_dev, size_t state_bytes) {
  if (!out) return PGXGO_EINVAL;
  *out = nullptr;
  if (!state_dev) return PGXGO_EINVAL;
  pgxgo_ctx* h = (pgxgo_ctx*)calloc(1, sizeof(pgxgo_ctx));
  if (!h) return PGXGO_ENOMEM;
  int rc = fill_ctx(h, batch, board_size, seed, opts, state_dev, state_bytes);
  if (rc == PGXGO_OK) rc = DISPATCH_N(h, launch_reset<19>(h, 1), launch_reset<9>(h, 1));
  if (rc == PGXGO_OK) {
    hipError_t e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) { g_last_hip = (int)e; rc = PGXGO_EHIP; }
  }
  if (rc != PGXGO_OK) { free(h); return rc; }
  *out = h;
  return PGXGO_OK;
}

int pgxgo_init_static(pgxgo_t* out, int32_t batch, int32_t board_size, uint32_t seed, const pgxgo_opts* opts) {
  if (!out) return PGXGO_EINVAL;
  *out = nullptr;
  int dev = -1;
  HIPCHK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxStaticDevices) return PGXGO_EINVAL;
  if (!g_scratch_ptr[dev]) {   // once per device, with that device current: each GPU holds its own copy of the array
    void* ptr = nullptr;
    HIPCHK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr || ((uintptr_t)ptr & 255u) != 0) return PGXGO_EINVAL;
    g_scratch_ptr[dev] = ptr;
  }
  if (batch <= 0 || (board_size != 9 && board_size != 19)) return PGXGO_EINVAL;
  const size_t need = board_size == 19 ? state_bytes_for<19>(batch, nullptr, nullptr, nullptr) : state_bytes_for<9>(batch, nullptr, nullptr, nullptr);
  if (need > (size_t)PGXGO_STATIC_STATE_BYTES) return PGXGO_ELIMIT;
  pgxgo_ctx* h = &g_static_ctx[dev];
  const int rc = fill_ctx(h, batch, board_size, seed, opts, g_scratch_ptr[dev], (size_t)PGXGO_STATIC_STATE_BYTES);
  if (rc != PGXGO_OK) return rc;
  // everything the handle reads is (re)written by this launch: rows, scalars, rewards, terminated flags of `batch` games
  const int rc2 = DISPATCH_N(h, launch_reset<19>(h, 1), launch_reset<9>(h, 1));
  if (rc2 != PGXGO_OK) return rc2;
  *out = h;
  return PGXGO_OK;
}

int pgxgo_destroy(pgxgo_t h) {
  if (!h) return PGXGO_EINVAL;
  if (h >= g_static_ctx && h < g_static_ctx + kMaxStaticDevices) return PGXGO_OK;   // a static handle owns no host memory
  free(h);
  return PGXGO_OK;
}

int pgxgo_reset(pgxgo_t h) {
  if (!h) return PGXGO_EINVAL;
  int rc = DISPATCH_N(h, launch_reset<19>(h, 0), launch_reset<9>(h, 0));
  if (rc != PGXGO_OK) return rc;
  if (h->zt) {   // empty tables; the rebuild pass writes the per-game records of the fresh games
    rc = DISPATCH_N(h, launch_superko_refresh<19>(h, true), launch_superko_refresh<9>(h, true));
    if (rc != PGXGO_OK) return rc;
  }
  if (h->mask_out || h->obs_out) return DISPATCH_N(h, launch_emit<19>(h, h->mask_out, h->obs_out), launch_emit<9>(h, h->mask_out, h->obs_out));
  return PGXGO_OK;
}

int pgxgo_bind_outputs(pgxgo_t h, uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev) {
  if (!h) return PGXGO_EINVAL;
  float* new_rew = rewards_dev ? rewards_dev : h->rew_int;
  uint8_t* new_term = terminated_dev ? terminated_dev : h->term_int;
  if (new_rew != h->rew_out) HIPCHK(hipMemcpyAsync(new_rew, h->rew_out, (size_t)h->B * 2 * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
  if (new_term != h->term_out) HIPCHK(hipMemcpyAsync(new_term, h->term_out, (size_t)h->B, hipMemcpyDeviceToDevice, h->stream));
  h->rew_out = new_rew; h->term_out = new_term;
  h->mask_out = mask_dev; h->obs_out = obs_dev;
  h->mask_written = mask_dev; h->obs_written = obs_dev;
  if (mask_dev || obs_dev) return DISPATCH_N(h, launch_emit<19>(h, mask_dev, obs_dev), launch_emit<9>(h, mask_dev, obs_dev));
  return PGXGO_OK;
}

int pgxgo_set_output_buffers(pgxgo_t h, uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev) {
  if (!h) return PGXGO_EINVAL;
  h->mask_out = mask_dev; h->obs_out = obs_dev;
  h->rew_out = rewards_dev ? rewards_dev : h->rew_int;
  h->term_out = terminated_dev ? terminated_dev : h->term_int;
  return PGXGO_OK;
}

int pgxgo_emit(pgxgo_t h, uint8_t* mask_dev, uint8_t* obs_dev) {
  if (!h || (!mask_dev && !obs_dev)) return PGXGO_EINVAL;
  return DISPATCH_N(h, launch_emit<19>(h, mask_dev, obs_dev), launch_emit<9>(h, mask_dev, obs_dev));
}

int pgxgo_step(pgxgo_t h, const int32_t* actions_dev) {
  if (!h || !actions_dev) return PGXGO_EINVAL;
  return DISPATCH_N(h, launch_step<19>(h, actions_dev, false, 0u, 0u, nullptr, nullptr), launch_step<9>(h, actions_dev, false, 0u, 0u, nullptr, nullptr));
}

int pgxgo_step_sample(pgxgo_t h, const int32_t* actions_dev, uint32_t seed, uint32_t t, const int32_t* start_t_dev, int32_t* next_actions_dev) {
  if (!h || !actions_dev || !next_actions_dev || next_actions_dev == actions_dev) return PGXGO_EINVAL;
  return DISPATCH_N(h, launch_step<19>(h, actions_dev, true, seed, t, start_t_dev, next_actions_dev),
                    launch_step<9>(h, actions_dev, true, seed, t, start_t_dev, next_actions_dev));
}

int pgxgo_rollout(pgxgo_t h, int32_t steps, int32_t slices, uint32_t seed, uint32_t t0, const int32_t* start_t_dev, int32_t* actions_dev,
                  float* rewards_dev, uint8_t* terminated_dev, uint8_t* mask_dev, uint8_t* obs_dev) {
  if (!h || steps < 0 || slices < 1) return PGXGO_EINVAL;
  if (steps == 0) return PGXGO_OK;
  RolloutArgs a;
  a.planes = h->planes; a.meta = h->meta; a.B = h->B; a.wb = h->wb;
  a.rules.seed = h->seed; a.rules.komi_x2 = h->komi_x2; a.rules.max_steps = h->max_steps; a.rules.auto_reset = h->auto_reset;
  a.steps = steps; a.slices = slices; a.seed = seed; a.t0 = t0; a.start_t = start_t_dev;
  a.actions = actions_dev; a.rew = rewards_dev; a.term = terminated_dev; a.mask = mask_dev; a.obs = obs_dev;
  a.mask_pitch = h->mask_pitch; a.obs_pitch = h->obs_pitch;
  a.zt = h->zt; a.zcur = h->zcur; a.sk_mode = h->sk_mode;
  return DISPATCH_N(h, launch_rollout<19>(h, a), launch_rollout<9>(h, a));
}

int pgxgo_step_slots(pgxgo_t h, int32_t n, const int32_t* src_slots_dev, const int32_t* actions_dev, const int32_t* dst_slots_dev,
                     uint8_t* mask_dev, uint8_t* obs_dev, float* rewards_dev, uint8_t* terminated_dev) {
  if (!h || n < 0 || n > h->B || !src_slots_dev || !dst_slots_dev) return PGXGO_EINVAL;
  if (n == 0) return PGXGO_OK;
  SlotArgs a;
  a.planes = h->planes; a.meta = h->meta; a.pool = h->B; a.n = n; a.src = src_slots_dev; a.dst = dst_slots_dev; a.actions = actions_dev;
  a.rew = rewards_dev; a.term = terminated_dev; a.mask = mask_dev; a.obs = obs_dev; a.mask_pitch = h->mask_pitch; a.obs_pitch = h->obs_pitch;
  a.rules.seed = h->seed; a.rules.komi_x2 = h->komi_x2; a.rules.max_steps = h->max_steps; a.rules.auto_reset = h->auto_reset;
  a.zt = h->zt; a.zcur = h->zcur; a.sk_mode = h->sk_mode;
  return DISPATCH_N(h, launch_slots<19>(h, a), launch_slots<9>(h, a));
}

int pgxgo_copy_slots(pgxgo_t h, int32_t n, const int32_t* src_slots_dev, const int32_t* dst_slots_dev) {
  return pgxgo_step_slots(h, n, src_slots_dev, nullptr, dst_slots_dev, nullptr, nullptr, nullptr, nullptr);
}

int pgxgo_random_actions(pgxgo_t h, uint32_t seed, uint32_t t, const int32_t* start_t_dev, int32_t* actions_dev) {
  if (!h || !actions_dev) return PGXGO_EINVAL;
  return DISPATCH_N(h, launch_random<19>(h, seed, t, start_t_dev, actions_dev), launch_random<9>(h, seed, t, start_t_dev, actions_dev));
}

int pgxgo_legal_mask(pgxgo_t h, uint8_t* dst_dev) {
  if (!h || !dst_dev) return PGXGO_EINVAL;
  return DISPATCH_N(h, launch_emit<19>(h, dst_dev, nullptr), launch_emit<9>(h, dst_dev, nullptr));
}

int pgxgo_observe(pgxgo_t h, uint8_t* dst_dev) {
  if (!h || !dst_dev) return PGXGO_EINVAL;
  return DISPATCH_N(h, launch_emit<19>(h, nullptr, dst_dev), launch_emit<9>(h, nullptr, dst_dev));
}

int pgxgo_rewards(pgxgo_t h, float* dst_dev) {
  if (!h || !dst_dev) return PGXGO_EINVAL;
  if (dst_dev != h->rew_out) HIPCHK(hipMemcpyAsync(dst_dev, h->rew_out, (size_t)h->B * 2 * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
  return PGXGO_OK;
}

int pgxgo_terminated(pgxgo_t h, uint8_t* dst_dev) {
  if (!h || !dst_dev) return PGXGO_EINVAL;
  if (dst_dev != h->term_out) HIPCHK(hipMemcpyAsync(dst_dev, h->term_out, (size_t)h->B, hipMemcpyDeviceToDevice, h->stream));
  return PGXGO_OK;
}

int pgxgo_current_player(pgxgo_t h, uint8_t* dst_dev) {
  if (!h || !dst_dev) return PGXGO_EINVAL;
  const int threads = 256;
  if (h->N == 19) hipLaunchKernelGGL(go_current_player_kernel<19>, dim3((h->B + threads - 1) / threads), dim3(threads), 0, h->stream, h->meta, h->B, dst_dev);
  else hipLaunchKernelGGL(go_current_player_kernel<9>, dim3((h->B + threads - 1) / threads), dim3(threads), 0, h->stream, h->meta, h->B, dst_dev);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

int pgxgo_export_state(pgxgo_t h, int8_t* board_dev, int8_t* history_dev, int32_t* ko_dev, int8_t* to_play_dev, int32_t* steps_dev,
                       int8_t* passes_dev, uint8_t* terminated_dev, uint8_t* black_player_dev, uint32_t* episode_dev, uint32_t* illegal_dev) {
  if (!h) return PGXGO_EINVAL;
  CanonArgs c = {board_dev, history_dev, ko_dev, to_play_dev, steps_dev, passes_dev, terminated_dev, black_player_dev, episode_dev, illegal_dev};
  return DISPATCH_N(h, launch_export<19>(h, c), launch_export<9>(h, c));
}

int pgxgo_import_state(pgxgo_t h, const int8_t* board_dev, const int8_t* history_dev, const int32_t* ko_dev, const int8_t* to_play_dev,
                       const int32_t* steps_dev, const int8_t* passes_dev, const uint8_t* terminated_dev, const uint8_t* black_player_dev,
                       const uint32_t* episode_dev) {
  if (!h || !board_dev || !history_dev || !ko_dev || !to_play_dev || !steps_dev || !passes_dev || !terminated_dev || !black_player_dev ||
      !episode_dev)
    return PGXGO_EINVAL;
  CanonArgs c = {(int8_t*)board_dev, (int8_t*)history_dev, (int32_t*)ko_dev, (int8_t*)to_play_dev, (int32_t*)steps_dev, (int8_t*)passes_dev,
                 (uint8_t*)terminated_dev, (uint8_t*)black_player_dev, (uint32_t*)episode_dev, nullptr};
  int rc = DISPATCH_N(h, launch_import<19>(h, c), launch_import<9>(h, c));
  if (rc != PGXGO_OK) return rc;
  if (h->zt) {
    rc = DISPATCH_N(h, launch_superko_refresh<19>(h, true), launch_superko_refresh<9>(h, true));
    if (rc != PGXGO_OK) return rc;
  }
  if (h->mask_out || h->obs_out) return DISPATCH_N(h, launch_emit<19>(h, h->mask_out, h->obs_out), launch_emit<9>(h, h->mask_out, h->obs_out));
  return PGXGO_OK;
}

int pgxgo_set_boards_per_wavefront(pgxgo_t h, int32_t boards) {
  if (!h) return PGXGO_EINVAL;
  const int wmax = h->N == 19 ? Geo<19>::W : Geo<9>::W;
  if (boards < 0 || boards > wmax) return PGXGO_EINVAL;
  h->wb = boards ? boards : (h->N == 19 ? auto_boards_per_wavefront<19>(h->B) : auto_boards_per_wavefront<9>(h->B));
  return h->wb;
}

size_t pgxgo_superko_bytes(int32_t batch, int32_t board_size) {
  if (batch <= 0) return 0;
  if (board_size == 19) return superko_bytes_for<19>(batch, nullptr);
  if (board_size == 9) return superko_bytes_for<9>(batch, nullptr);
  return 0;
}

int pgxgo_enable_superko(pgxgo_t h, int32_t mode, void* table_dev, size_t table_bytes) {
  if (!h || mode < 0 || mode > 2) return PGXGO_EINVAL;
  if (mode == 0 || !table_dev) {
    if (mode != 0) return PGXGO_EINVAL;
    h->zt = nullptr; h->zcur = nullptr; h->sk_mode = 0;
  } else {
    if (((uintptr_t)table_dev & 255u) != 0 || h->max_steps > 2 * h->N * h->N) return PGXGO_EINVAL;
    size_t off_cur;
    const size_t need = h->N == 19 ? superko_bytes_for<19>(h->B, &off_cur) : superko_bytes_for<9>(h->B, &off_cur);
    if (table_bytes < need) return PGXGO_EINVAL;
    h->zt = (uint2*)table_dev;
    h->zcur = (uint4*)((uint8_t*)table_dev + off_cur);
    h->sk_mode = mode;
    const int rc = DISPATCH_N(h, launch_superko_refresh<19>(h, true), launch_superko_refresh<9>(h, true));
    if (rc != PGXGO_OK) { h->zt = nullptr; h->zcur = nullptr; h->sk_mode = 0; return rc; }
  }
  // the bound mask follows the rule in force from now on
  if (h->mask_out) return DISPATCH_N(h, launch_emit<19>(h, h->mask_out, nullptr), launch_emit<9>(h, h->mask_out, nullptr));
  return PGXGO_OK;
}

int pgxgo_sync(pgxgo_t h) {
  if (!h) return PGXGO_EINVAL;
  HIPCHK(hipStreamSynchronize(h->stream));
  return PGXGO_OK;
}

const char* pgxgo_strerror(int code) {
  switch (code) {
    case PGXGO_OK: return "ok";
    case PGXGO_EINVAL: return "invalid argument";
    case PGXGO_EHIP: return "HIP runtime error";
    case PGXGO_ENOMEM: return "out of host memory";
    case PGXGO_ELIMIT: return "size beyond the limit of the library's static buffer";
    default: return "unknown error";
  }
}

int pgxgo_last_hip_error(void) { return g_last_hip; }

int pgxgo_fill_probe(void* dst_dev, size_t nbytes, uint32_t value, int32_t kind, void* stream) {
  if (!dst_dev || ((uintptr_t)dst_dev & 15u) != 0 || (nbytes & 15u) != 0 || kind < 0 || kind > 2) return PGXGO_EINVAL;
  if (nbytes == 0) return PGXGO_OK;
  const size_t n16 = nbytes / 16;
  if ((n16 + 255) / 256 > 0x7FFFFFFFull) return PGXGO_EINVAL;
  const dim3 grid((unsigned)((n16 + 255) / 256)), block(256);
  if (kind == 0) hipLaunchKernelGGL(fill_probe_kernel<kStorePlain>, grid, block, 0, (hipStream_t)stream, (uint4*)dst_dev, n16, value);
  else if (kind == 1) hipLaunchKernelGGL(fill_probe_kernel<kStoreStream>, grid, block, 0, (hipStream_t)stream, (uint4*)dst_dev, n16, value);
  else hipLaunchKernelGGL(fill_probe_kernel<kStoreThrough>, grid, block, 0, (hipStream_t)stream, (uint4*)dst_dev, n16, value);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

int pgxgo_empty_probe(void* stream, int32_t count) {
  if (count < 0) return PGXGO_EINVAL;
  for (int32_t i = 0; i < count; ++i) hipLaunchKernelGGL(empty_probe_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

int pgxgo_lane_shift_probe(const uint32_t* in_dev, uint32_t* out_dev, void* stream) {
  if (!in_dev || !out_dev) return PGXGO_EINVAL;
  hipLaunchKernelGGL(lane_shift_probe_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, in_dev, out_dev);
  HIPCHK(hipGetLastError());
  return PGXGO_OK;
}

}  // extern "C"
