// wave_common.hpp -- wavefront-level building blocks shared by the game kernels of this library (gfx950, wave64).
//
// Mapping they serve: one board row per lane, several boards per wavefront separated by all-zero sentinel
// lanes, so that a one-lane DPP shift brings every row its north / south neighbour; board-wide facts come from
// ballots masked with the board's lane segment; byte outputs (legal mask, observation planes; Fig. 2 and
// Table 1 of the Pgx paper, arXiv 2303.17503) are staged as a bit stream in LDS and expanded 16 bits ->
// 16 bytes per lane through a 256-entry LDS table.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pgxwave {

// counter-based hash of (seed, tag, env, t); tag 0 = action draw, tag 1 = seat draw (t = episode)
__device__ __forceinline__ uint32_t mixer(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du;
  x ^= x >> 15; x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}
__device__ __forceinline__ uint32_t env_hash(uint32_t seed, uint32_t tag, uint32_t env, uint32_t t) {
  return mixer(mixer(mixer(seed + 0x9E3779B9u * (tag + 1u)) ^ env) ^ t);
}

// index of the calling wavefront within its block, as a value the compiler knows to be the same in every lane
// (so that everything derived from it -- output addresses, trip counts -- is computed once per wavefront)
__device__ __forceinline__ int wave_in_block() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Which piece of the batch a block works on.  The hardware hands the blocks of a launch to the chip's eight dies (each
// with an L2 of its own) round-robin by block index; with piece = block index, neighbouring stretches of every array
// would be written through eight different L2s, and a 128-byte line shared by the output runs of two neighbouring
// blocks would reach memory as two partial writes.  Block i takes piece (i mod 8) * (blocks / 8) + i / 8 instead, so
// that each die reads and writes one contiguous eighth of the batch and such lines leave one L2 whole (65536 games of
// 19x19: 85.5 -> 82.5 us per ply; 16384 games: 20.4 -> 20.15).  The grid must be a multiple of 8 blocks (pieces
// beyond the batch are idle).
__device__ __forceinline__ int piece_of_block() { return (int)(blockIdx.x & 7u) * (int)(gridDim.x >> 3) + (int)(blockIdx.x >> 3); }

// ------------------------------------------------------------------------------------------------
// cross-lane primitives.  All of them must be called with every lane of the wavefront active.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t from_lane_below(uint32_t x) {  // lane i receives lane i-1, lane 0 receives 0
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x138 /* wave_shr:1 */, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t from_lane_above(uint32_t x) {  // lane i receives lane i+1, lane 63 receives 0
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x130 /* wave_shl:1 */, 0xF, 0xF, true);
}
// A fact about a whole board, known to every lane of the board: does `pred` hold in any of its rows?
// (seglo/seghi = the lanes holding the rows of the calling lane's board)
__device__ __forceinline__ bool board_any(bool pred, uint32_t seglo, uint32_t seghi) {
  const uint64_t m = __ballot(pred);
  return (((uint32_t)m & seglo) | ((uint32_t)(m >> 32) & seghi)) != 0u;
}

// Returns v; keeps the compiler from evaluating anything that depends on a loaded value before this point (it
// would otherwise move the first use, and with it the wait for the load, up to the load itself).
__device__ __forceinline__ int32_t held_back(int32_t v) {
  asm volatile("" : "+v"(v));
  return v;
}

// LDS traffic between the lanes of one wavefront needs no hardware barrier (a wavefront's LDS operations
// execute in program order); this only keeps the compiler from moving accesses across the hand-over.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ------------------------------------------------------------------------------------------------
// bit stream -> byte stream.  `bits` (LDS) holds bit (head+i) = byte i of the destination, head = the
// destination's offset from the previous 16-byte boundary.  Whole aligned 16-byte groups are written as
// vectors, the ragged ends byte by byte.  Lane l always writes a group whose address is l*16 modulo 128, so
// that every store instruction of the wavefront covers eight whole 128-byte lines: a 1 KB store that straddles
// line boundaries costs a quarter more time once the lines have to reach DRAM (measured with a plain fill).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t spread4(uint32_t nibble) { return (nibble * 0x00204081u) & 0x01010101u; }

// 256-entry table in LDS: entry x = the eight bytes (0/1) of the bits of x.  Filled once per block.
__device__ __forceinline__ void fill_spread_table(uint2* lut) {
  for (uint32_t x = threadIdx.x; x < 256u; x += blockDim.x) lut[x] = make_uint2(spread4(x & 15u), spread4(x >> 4));
  __syncthreads();
}

// The 16-byte output stores.  Basic kinds:
//   kStorePlain          ordinary store (write-back in the compute die's L2);
//   kStoreStream         with the non-temporal hint, for launches that write far more than the memory-side cache
//                        holds (below that size it is slower);
//   kStoreThrough        written through the L2 to the memory-side level (`sc1`).  Lines left dirty in the L2 have to
//                        be written back when the kernel ends: a plain fill of 106 MB pays 1.3 of its 16.8 us for
//                        that.  Partial lines written this way are expensive, though;
//   kStoreStreamThrough  both modifiers.
// and two that emit_bytes resolves per store instruction: the instructions of a stream that cover whole 128-byte
// lines only (all but its first and its last two) / the others, whose lines are shared with the streams next door:
//   kStoreThroughWhole   kStoreThrough / kStorePlain
//   kStoreStreamWhole    kStoreStreamThrough / kStoreStream
// Which kind a launch uses is decided on the host from the bytes it writes (all choices measured).
// The compiler has no builtin for a 16-byte store with the `sc1` modifier, hence the instruction itself.  It is
// followed by the two wait states this hardware needs between a store of more than 8 bytes and a write to its data
// registers (the compiler inserts them for its own stores; with one wait state rows of the state were stored wrong).
constexpr int kStorePlain = 0, kStoreStream = 1, kStoreThrough = 2, kStoreThroughWhole = 3, kStoreStreamThrough = 4, kStoreStreamWhole = 5;
template <int KIND>
__device__ __forceinline__ void store16(uint4* p, uint2 lo, uint2 hi) {
  typedef unsigned int vec4u __attribute__((ext_vector_type(4)));
  const vec4u v4 = {lo.x, lo.y, hi.x, hi.y};
  static_assert(KIND != kStoreThroughWhole && KIND != kStoreStreamWhole, "resolved by emit_bytes");
  if constexpr (KIND == kStorePlain) *p = make_uint4(lo.x, lo.y, hi.x, hi.y);
  else if constexpr (KIND == kStoreStream) __builtin_nontemporal_store(v4, (vec4u*)p);
  else if constexpr (KIND == kStoreStreamThrough) asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v4) : "memory");
  else asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v4) : "memory");
}

// MAXBYTES: upper bound of nbytes (fixes the number of rounds of 64 groups).  dst and nbytes must be the same in
// every lane.
template <int MAXBYTES, int ST = kStorePlain>
__device__ __forceinline__ void emit_bytes(const uint32_t* bits, const uint2* lut, uint8_t* dst, uint32_t nbytes, int lane) {
  constexpr int ROUNDS = (((MAXBYTES + 15) >> 4) + 7 + 63) / 64;   // groups + the at most 7 skipped at the front
  const uint32_t head = (uint32_t)((uintptr_t)dst & 15u);
  uint8_t* base = dst - head;
  const uint32_t q = ((uint32_t)(uintptr_t)base >> 4) & 7u;         // position of group 0 in its 128-byte line
  const uint32_t total = head + nbytes;
  const uint32_t m0 = head ? 1u : 0u, m1 = total >> 4;              // whole groups m0 .. m1-1
  const int32_t mine = lane - (int32_t)q;                           // this lane's group in round 0; round i adds 64*i
  const uint16_t* src = (const uint16_t*)bits + mine;
  uint4* out = (uint4*)base + mine;
  constexpr int GROUP = 6;   // rounds in flight at a time (bounds the registers held by pending LDS reads)
  // Round 0 skips the groups before m0; rounds 1 .. ROUNDS-3 are full for a full wavefront of boards and then run
  // without per-lane tests (the choice is the same for the whole wavefront).
  const bool full_mid = m1 + q >= 64u * (uint32_t)(ROUNDS > 2 ? ROUNDS - 2 : 0);
  auto active = [&](int i) { return mine + 64 * i >= (int32_t)m0 && mine + 64 * i < (int32_t)m1; };
  constexpr int ST_WHOLE = ST == kStoreThroughWhole ? kStoreThrough : (ST == kStoreStreamWhole ? kStoreStreamThrough : ST);
  constexpr int ST_EDGE = ST == kStoreThroughWhole ? kStorePlain : (ST == kStoreStreamWhole ? kStoreStream : ST);
  // the round before the last lies completely inside the stream when the last one is not empty (the same in every lane)
  const bool pen_whole = m1 + q >= 64u * (uint32_t)(ROUNDS - 1);
  if (full_mid) {
#pragma unroll
    for (int g = 0; g < ROUNDS; g += GROUP) {
      uint32_t v[GROUP];
#pragma unroll
      for (int i = g; i < g + GROUP && i < ROUNDS; ++i) {
        const bool test = (i == 0 || i >= ROUNDS - 2);
        v[i - g] = (!test || active(i)) ? (uint32_t)src[64 * i] : 0u;
      }
#pragma unroll
      for (int i = g; i < g + GROUP && i < ROUNDS; ++i) {
        const bool test = (i == 0 || i >= ROUNDS - 2);
        if (!test) store16<ST_WHOLE>(&out[64 * i], lut[v[i - g] & 255u], lut[v[i - g] >> 8]);
        else if (ST_WHOLE != ST_EDGE && i == ROUNDS - 2 && i > 0 && pen_whole) store16<ST_WHOLE>(&out[64 * i], lut[v[i - g] & 255u], lut[v[i - g] >> 8]);
        else if (active(i)) store16<ST_EDGE>(&out[64 * i], lut[v[i - g] & 255u], lut[v[i - g] >> 8]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
#pragma unroll
    for (int g = 0; g < ROUNDS; g += GROUP) {
      uint32_t v[GROUP];
#pragma unroll
      for (int i = g; i < g + GROUP && i < ROUNDS; ++i) v[i - g] = active(i) ? (uint32_t)src[64 * i] : 0u;
#pragma unroll
      for (int i = g; i < g + GROUP && i < ROUNDS; ++i)
        if (active(i)) store16<ST_EDGE>(&out[64 * i], lut[v[i - g] & 255u], lut[v[i - g] >> 8]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (lane < 32) {
    uint32_t i = lane & 15u, pos;
    bool ok;
    if (lane < 16) { pos = i; ok = head != 0u && i >= head; }
    else { pos = (m1 << 4) + i; ok = i < (total & 15u); }
    if (ok) base[pos] = (uint8_t)((bits[pos >> 5] >> (pos & 31u)) & 1u);
  }
}

}  // namespace pgxwave
