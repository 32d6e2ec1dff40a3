// Attention softmax -> dropout sublayer for gfx950 (Sec. 3.3, 3.4; App. E.3, E.4).
//
// Forward keeps only P (the softmax output) and a 1-bit keep mask; the dropout output is a
// transient.  Backward rebuilds the dropout output from (P, mask) by one multiply and derives
// the score gradient from P alone.  A group of LANES lanes owns one row in registers (CH
// 16-byte pieces per lane, piece c of lane t = c*LANES + t so every access of a group is
// contiguous).  The keep bits come from Philox4x32-10, one call per 8 elements, so the mask is
// a pure function of (seed, offset, element index) and does not depend on the launch shape;
// backward can therefore also draw the bits again instead of reading a stored mask.
#include <type_traits>

#include "tempo_device.h"
#include "tempo_host.h"

namespace tempo {
namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

struct RngArgs {
  uint32_t seed_lo, seed_hi, off_lo, off_hi;
  uint32_t t16;  // keep iff 16-bit draw < t16; 65536 keeps everything (generator skipped)
};

// a ^ b ^ c in one VALU op (v_bitop3_b32 with truth table 0x96).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64 multiplies,
// the key advanced by the two Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&w)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t n0 = xor3(static_cast<uint32_t>(p1 >> 32), c1, k0);
    const uint32_t n2 = xor3(static_cast<uint32_t>(p0 >> 32), c3, k1);
    c1 = static_cast<uint32_t>(p1);
    c3 = static_cast<uint32_t>(p0);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}

// Keep bits of the 8 elements of group g (bit i = element 8g + i).  A 16-bit draw r is kept iff
// r < t16, i.e. iff r - t16 is negative: v_alignbit shifts that sign bit into the byte, last
// element first.
__device__ __forceinline__ uint32_t keep_byte(uint64_t g, const RngArgs& a) {
  if (a.t16 >= 65536u) return 0xFFu;
  uint32_t w[4];
  philox4x32_10(static_cast<uint32_t>(g), static_cast<uint32_t>(g >> 32), a.off_lo, a.off_hi,
                a.seed_lo, a.seed_hi, w);
  uint32_t byte = 0;
#pragma unroll
  for (int i = 3; i >= 0; --i) {
    byte = __builtin_amdgcn_alignbit(byte, (w[i] >> 16) - a.t16, 31);      // byte << 1 | sign
    byte = __builtin_amdgcn_alignbit(byte, (w[i] & 0xFFFFu) - a.t16, 31);
  }
  return byte;
}

// All ones if bit K of bits is set, else zero.  Written as the instruction itself: spelled in
// C++ the compiler turns the following AND into test + compare + select, three operations per
// element where two suffice (these kernels run close to the vector-ALU limit).
template <int K>
__device__ __forceinline__ uint32_t bit_mask(uint32_t bits) {
  uint32_t m;
  asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(m) : "v"(bits), "n"(K));
  return m;
}

// Zero the dropped elements of a packed piece: keep bit i belongs to element i of the piece.
// bfloat16 words hold two elements: their two masks are merged byte-wise (v_perm_b32).
template <typename T>
__device__ __forceinline__ u32x4 apply_keep(u32x4 w, uint32_t bits) {
  if constexpr (Store<T>::kVec == 4) {
    w.x &= bit_mask<0>(bits);
    w.y &= bit_mask<1>(bits);
    w.z &= bit_mask<2>(bits);
    w.w &= bit_mask<3>(bits);
  } else {
    constexpr uint32_t kLoHalves = 0x05040100u;  // bytes 0,1 of the second source, then of the first
    w.x &= __builtin_amdgcn_perm(bit_mask<1>(bits), bit_mask<0>(bits), kLoHalves);
    w.y &= __builtin_amdgcn_perm(bit_mask<3>(bits), bit_mask<2>(bits), kLoHalves);
    w.z &= __builtin_amdgcn_perm(bit_mask<5>(bits), bit_mask<4>(bits), kLoHalves);
    w.w &= __builtin_amdgcn_perm(bit_mask<7>(bits), bit_mask<6>(bits), kLoHalves);
  }
  return w;
}


// Element offset of the start of a row: rows are counted in 32 bits on the register-resident
// paths (the host checks), so the product is one 32x32->64 multiply instead of a 64x64 one.
__device__ __forceinline__ int64_t row_offset(uint32_t row, int Sk) {
  return static_cast<int64_t>(static_cast<uint64_t>(row) * static_cast<uint32_t>(Sk));
}

// Number of leading key columns of query row i that take part in the softmax.
__device__ __forceinline__ int row_limit(int i, int key_limit, int causal, int Sq, int Sk) {
  int limit = key_limit;
  if (causal) limit = min(limit, max(i + (Sk - Sq) + 1, 0));
  return limit;
}

// Keep bits of the CH pieces a lane owns in one row.  Piece c of the lane is flat piece
// piece0 + c*LANES + t.  bfloat16 pieces (8 elements) are whole Philox groups.  float32 pieces
// (4 elements) are half groups: lanes 2k and 2k+1 hold the two halves of the same group for
// every c, so the pair splits the generator calls (the even lane draws the groups of even c,
// the odd lane those of odd c) and swaps the bytes with one DPP move.
template <typename T, int LANES, int CH>
__device__ __forceinline__ void lane_keep_bits(int64_t piece0, int t, const RngArgs& rng,
                                               uint32_t (&bits)[CH]) {
  if constexpr (Store<T>::kVec == 8) {
#pragma unroll
    for (int c = 0; c < CH; ++c)
      bits[c] = keep_byte(static_cast<uint64_t>(piece0 + c * LANES + t), rng);
  } else {
    const int odd = t & 1;
#pragma unroll
    for (int c = 0; c < CH; c += 2) {
      const int mine = (c + 1 < CH) ? c + odd : c;  // a trailing single piece: both lanes draw
      const uint32_t own = keep_byte(static_cast<uint64_t>(piece0 + mine * LANES + t) >> 1, rng);
      const uint32_t other = dpp_u32<kDppXor1>(own);
      const uint32_t even_c = (c + 1 < CH) ? (odd ? other : own) : own;
      bits[c] = (even_c >> (4 * odd)) & 0xFu;
      if (c + 1 < CH) bits[c + 1] = ((odd ? own : other) >> (4 * odd)) & 0xFu;
    }
  }
}

// Store the mask bits of one piece.  WORDS (Sk % 32 == 0): the lanes sharing a word merge their
// bits and one of them writes the word; otherwise (Sk % 8 == 0) bytes are written: by every
// lane (bf16) or by the even lane of each pair (f32).  All lanes of the sharing group must
// call this together; `valid` says whether the lane's piece exists.
template <typename T, bool WORDS>
__device__ __forceinline__ void store_keep_bits(uint32_t* keep_bits, int64_t piece, int t,
                                                uint32_t bits, bool valid, int64_t total_pieces) {
  constexpr int V = Store<T>::kVec;
  if constexpr (WORDS) {
    const uint32_t word = merge_mask_word<V>(bits, t);
    constexpr int kShare = 32 / V;
    if ((t & (kShare - 1)) == 0 && valid) keep_bits[piece / kShare] = word;
  } else {
    uint8_t* kb = reinterpret_cast<uint8_t*>(keep_bits);
    uint32_t byte = bits;
    int64_t bi = piece;  // byte index
    bool writer = valid;
    if constexpr (V == 4) {
      byte = bits << (4 * (t & 1));
      byte |= dpp_u32<kDppXor1>(byte);
      bi = piece >> 1;
      writer = valid && (t & 1) == 0;
    }
    if (writer) {
      kb[bi] = static_cast<uint8_t>(byte);
      const int64_t last = (V == 4 ? total_pieces >> 1 : total_pieces) - 1;
      if (bi == last) {
        for (int64_t b = bi + 1; (b & 3) != 0; ++b) kb[b] = 0;  // rest of the last word
      }
    }
  }
}

// Mask bits of one piece as read by backward.
template <typename T, bool WORDS>
__device__ __forceinline__ uint32_t load_keep_bits(const uint32_t* keep_bits, int64_t piece) {
  constexpr int V = Store<T>::kVec;
  if constexpr (WORDS) {
    constexpr int kShare = 32 / V;
    return (keep_bits[piece / kShare] >> (V * static_cast<int>(piece & (kShare - 1)))) &
           ((1u << V) - 1u);
  } else {
    const uint8_t* kb = reinterpret_cast<const uint8_t*>(keep_bits);
    if constexpr (V == 8) return kb[piece];
    return (kb[piece >> 1] >> (4 * static_cast<int>(piece & 1))) & 0xFu;
  }
}

// Work unit = one "row set": kGroups*R consecutive query rows of one [Sq, Sk] slice, where
// kGroups = kThreads/LANES lane groups each own R rows (rows base + r*kGroups + g) and CH
// 16-byte pieces per row (piece c of lane t = c*LANES + t).  All R rows of a group are fetched
// before any arithmetic: short rows would otherwise leave one 16-byte load per lane in
// flight, too little to cover the memory latency at 32 waves per compute unit.  With the
// default launch cap every row set has its own workgroup and the grid sweeps memory front to
// back; under a smaller cap workgroups walk the row sets grid-stride.
// LANES = 128 or 256 spreads a long row over 2 or 4 waves: the pieces per lane, and with them
// the registers per lane, stay small enough for many resident waves (a 3072-element bfloat16
// row on one wave needs over 200 registers per lane, which leaves 2 waves per SIMD).
template <typename T, int LANES, int CH, int R, bool WORDS, int THREADS>
__global__ __launch_bounds__(THREADS) void attn_fwd_kernel(
    const T* scores, const int32_t* __restrict__ key_len, int causal, T* probs,
    T* __restrict__ out, uint32_t* __restrict__ keep_bits, int slices, int A, int Sq, int Sk,
    float scale, RngArgs rng) {
  static_assert(THREADS % LANES == 0 && THREADS % kWave == 0, "whole lane groups, whole waves");
  constexpr int kGroups = THREADS / LANES;
  constexpr int V = Store<T>::kVec;
  const int g = threadIdx.x / LANES;
  const int t = threadIdx.x % LANES;
  const int pieces = Sk / V;
  const int sets_per_slice = (Sq + kGroups * R - 1) / (kGroups * R);
  const int64_t total_sets = static_cast<int64_t>(slices) * sets_per_slice;
  const int64_t total_pieces = static_cast<int64_t>(slices) * Sq * pieces;
  __shared__ float red[2][THREADS / kWave];
  static_assert(LANES <= kWave || R == 1, "rows over several waves: one row per group");

  for (int64_t rs = blockIdx.x; rs < total_sets; rs += gridDim.x) {
    const int slice = static_cast<int>(rs / sets_per_slice);
    const int i0 = static_cast<int>(rs % sets_per_slice) * (kGroups * R) + g;
    const int key_limit = key_len ? min(max(key_len[slice / A], 0), Sk) : Sk;
    // limit = number of leading columns of the row that take part in the softmax; -1: no row
    int limit[R];
    Raw<T> raw[R][CH];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int i = i0 + r * kGroups;
      limit[r] = (i < Sq) ? row_limit(i, key_limit, causal, Sq, Sk) : -1;
      const T* sr = scores + row_offset(static_cast<uint32_t>(slice) * Sq + i, Sk);
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int col0 = (c * LANES + t) * V;
        if constexpr (CH == 1) raw[r][c].a = Store<T>::neg_inf_piece();  // see below
        if (col0 < limit[r]) raw[r][c].load(sr + col0);
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      // no row: uniform over the lane group; a group of several waves walks on (no loads, no
      // stores) because the reductions below hold workgroup barriers
      const bool live = limit[r] >= 0;
      if (LANES <= kWave && !live) continue;
      const int64_t row0 = row_offset(static_cast<uint32_t>(slice) * Sq + i0 + r * kGroups, Sk);
      float v[CH][V];
      float mx = -INFINITY;
      // One piece per lane: the lanes of a masked piece cannot save time by idling (their wave
      // runs on for the others), so a piece that was not loaded holds -inf and goes through the
      // same straight-line code, which gives 0 for it.  Several pieces per lane: a masked piece
      // is skipped, which for a causal mask spares whole waves half of their work.
      constexpr bool kSkip = CH > 1;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int col0 = (c * LANES + t) * V;
        if (!kSkip || col0 < limit[r]) {
          raw[r][c].unpack(v[c]);
          if (col0 < limit[r] && col0 + V > limit[r]) {  // the piece the limit falls into
#pragma unroll
            for (int k = 0; k < V; ++k) v[c][k] = (col0 + k < limit[r]) ? v[c][k] : -INFINITY;
          }
#pragma unroll
          for (int k = 0; k < V; ++k) mx = fmaxf(mx, v[c][k]);
        }
      }
      mx = row_reduce<LANES, true>(mx, red[0]);
      const float shift = (mx == -INFINITY) ? 0.0f : mx * kLog2e;
      float sum = 0.0f;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int col0 = (c * LANES + t) * V;
        if (!kSkip || col0 < limit[r]) {
#pragma unroll
          for (int k = 0; k < V; ++k) {
            const float e = __builtin_amdgcn_exp2f(fmaf(v[c][k], kLog2e, -shift));
            v[c][k] = e;
            sum += e;
          }
        } else {  // masked, or padding beyond the row
#pragma unroll
          for (int k = 0; k < V; ++k) v[c][k] = 0.0f;
        }
      }
      sum = row_reduce<LANES, false>(sum, red[1]);
      const float rinv = (sum > 0.0f) ? __builtin_amdgcn_rcpf(sum) : 0.0f;
      const int64_t piece0 = row0 / V;  // Sk is a multiple of the piece length here
      uint32_t bits[CH];
      lane_keep_bits<T, LANES, CH>(piece0, t, rng, bits);
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int pc = c * LANES + t;
        const bool valid = live && pc < pieces;
        if (valid) {
          float p8[V], o8[V];
#pragma unroll
          for (int k = 0; k < V; ++k) p8[k] = v[c][k] * rinv;
          // round P once, into the words that are stored; Out is computed from the stored P
          const u32x4 pw = Store<T>::pack(p8);
          Store<T>::unpack(pw, p8);
          stg_stream(probs + row0 + pc * V, pw);
          if (out) {
#pragma unroll
            for (int k = 0; k < V; ++k) o8[k] = p8[k] * scale;
            stg_stream(out + row0 + pc * V, apply_keep<T>(Store<T>::pack(o8), bits[c]));
          }
        }
        store_keep_bits<T, WORDS>(keep_bits, piece0 + pc, t, valid ? bits[c] : 0u, valid,
                                  total_pieces);
      }
    }
  }
}

// Keep bits of one piece from a mask kept the way the paper's implementation keeps it, one
// byte per element (Sec. 3.3; any non-zero byte means kept): one 4-byte (float32 piece) or
// 8-byte (bfloat16 piece) load per lane.  Per 32-bit word: fold each byte's bits onto its bit 0,
// then gather the four bit-0s by one multiply (the partial products land on distinct bits).
__device__ __forceinline__ uint32_t nonzero_bytes_to_bits(uint32_t w) {
  w |= w >> 4;
  w |= w >> 2;
  w |= w >> 1;
  w &= 0x01010101u;
  return (w * 0x01020408u) >> 24;  // byte i -> bit i
}
template <typename T>
__device__ __forceinline__ uint32_t load_keep_bools(const uint8_t* keep_bytes, int64_t element) {
  if constexpr (Store<T>::kVec == 4) {
    return nonzero_bytes_to_bits(
        __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(keep_bytes + element)));
  } else {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 w =
        __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(keep_bytes + element));
    return nonzero_bytes_to_bits(w.x) | (nonzero_bytes_to_bits(w.y) << 4);
  }
}

// MASK says where backward takes the keep bits from: the stored bit mask read as whole words
// (Sk % 32 == 0) or as bytes, the generator (no mask is read; Sec. 3.3 weighs storing the
// mask against drawing it again), or a mask of one byte per element (keep_bits then points to
// bytes).
enum MaskSource { kMaskWords, kMaskBytes, kMaskRegen, kMaskBools };

template <typename T, int LANES, int CH, int R, MaskSource MASK, int THREADS>
__global__ __launch_bounds__(THREADS) void attn_bwd_kernel(
    const T* dout, const T* __restrict__ probs, const uint32_t* __restrict__ keep_bits,
    T* dscores, T* __restrict__ out_re, uint32_t rows, int Sk, float scale, RngArgs rng) {
  static_assert(THREADS % LANES == 0 && THREADS % kWave == 0, "whole lane groups, whole waves");
  constexpr int kGroups = THREADS / LANES;
  constexpr int V = Store<T>::kVec;
  const int g = threadIdx.x / LANES;
  const int t = threadIdx.x % LANES;
  const int pieces = Sk / V;
  __shared__ float red[2][THREADS / kWave];
  static_assert(LANES <= kWave || R == 1, "rows over several waves: one row per group");
  int flip = 0;  // one reduction per row set: consecutive sets alternate between the slot arrays
  for (int64_t base = static_cast<int64_t>(blockIdx.x) * (kGroups * R); base < rows;
       base += static_cast<int64_t>(gridDim.x) * (kGroups * R), flip ^= 1) {
    Raw<T> rdo[R][CH], rp[R][CH];
    uint32_t bits[R][CH];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t row = base + r * kGroups + g;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int pc = c * LANES + t;
        bits[r][c] = 0;
        if (row < rows && pc < pieces) {
          const int64_t row0 = row_offset(static_cast<uint32_t>(row), Sk);
          rdo[r][c].load(dout + row0 + pc * V);
          rp[r][c].load(probs + row0 + pc * V);
          if constexpr (MASK == kMaskBools)
            bits[r][c] = load_keep_bools<T>(reinterpret_cast<const uint8_t*>(keep_bits),
                                            row0 + pc * V);
          else if constexpr (MASK != kMaskRegen)
            bits[r][c] = load_keep_bits<T, MASK == kMaskWords>(keep_bits, row0 / V + pc);
        }
      }
    }
    if constexpr (MASK == kMaskRegen) {  // every lane takes part: lane pairs share draws
#pragma unroll
      for (int r = 0; r < R; ++r)
        lane_keep_bits<T, LANES, CH>(
            row_offset(static_cast<uint32_t>(base + r * kGroups + g), Sk) / V, t, rng, bits[r]);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t row = base + r * kGroups + g;
      // no row: uniform over the lane group; a group of several waves walks on (the reduction
      // holds a workgroup barrier) with zeros and stores nothing
      const bool live = row < rows;
      if (LANES <= kWave && !live) continue;
      const int64_t row0 = row_offset(static_cast<uint32_t>(row), Sk);
      float dp[CH][V], pr[CH][V];
      float dot = 0.0f;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int pc = c * LANES + t;
        if (live && pc < pieces) {
          Store<T>::unpack(apply_keep<T>(rdo[r][c].a, bits[r][c]), dp[c]);  // dropped: dP = 0
          rp[r][c].unpack(pr[c]);
        } else {
#pragma unroll
          for (int k = 0; k < V; ++k) dp[c][k] = pr[c][k] = 0.0f;
        }
#pragma unroll
        for (int k = 0; k < V; ++k) {
          dp[c][k] *= scale;
          dot = fmaf(dp[c][k], pr[c][k], dot);
        }
      }
      dot = row_reduce<LANES, false>(dot, red[flip]);
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int pc = c * LANES + t;
        if (live && pc < pieces) {
          float ds[V];
#pragma unroll
          for (int k = 0; k < V; ++k) ds[k] = pr[c][k] * (dp[c][k] - dot);
          store_piece<T>(dscores + row0 + pc * V, ds);
          if (out_re) {
            float o8[V];
#pragma unroll
            for (int k = 0; k < V; ++k) o8[k] = pr[c][k] * scale;
            stg_stream(out_re + row0 + pc * V,
                       apply_keep<T>(Store<T>::pack(o8), bits[r][c]));
          }
        }
      }
    }
  }
}

// ---- any Sk: one wave per row, scalar accesses, the row re-read from cache per pass --------

// Keep bits of a block of up to 448 consecutive elements (7 chunks of 64: at most 57 groups of 8
// whatever the block's alignment): each lane draws one group, and the lanes fetch the byte of
// their element's group from the lane that drew it, one generator call per 8 elements instead
// of one per element.  Every lane of the wave has to make both calls.
constexpr int kDrawBlock = 7 * kWave;
struct KeepBlock {
  uint32_t byte;
  int64_t group0;
  __device__ __forceinline__ void draw(int64_t e_block, int lane, const RngArgs& rng) {
    group0 = e_block >> 3;
    byte = keep_byte(static_cast<uint64_t>(group0) + lane, rng);
  }
  __device__ __forceinline__ bool kept(int64_t e) const {
    return (__shfl(byte, static_cast<int>((e >> 3) - group0), kWave) >> (e & 7)) & 1u;
  }
};

template <typename T>
__global__ __launch_bounds__(kThreads) void attn_fwd_generic_kernel(
    const T* scores, const int32_t* __restrict__ key_len, int causal, T* probs,
    T* __restrict__ out, int64_t rows, int64_t rows_per_batch, int Sq, int Sk, float scale,
    RngArgs rng) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  constexpr int kWaves = kThreads / kWave;
  for (int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + wave; row < rows;
       row += static_cast<int64_t>(gridDim.x) * kWaves) {
    const int key_limit = key_len ? min(max(key_len[row / rows_per_batch], 0), Sk) : Sk;
    const int limit = row_limit(static_cast<int>(row % Sq), key_limit, causal, Sq, Sk);
    const T* sr = scores + row * Sk;
    float mx = -INFINITY;
    for (int j = lane; j < limit; j += kWave) mx = fmaxf(mx, Store<T>::load1(sr + j));
    mx = group_max<kWave>(mx);
    const float shift = (mx == -INFINITY) ? 0.0f : mx * kLog2e;
    float sum = 0.0f;
    for (int j = lane; j < limit; j += kWave)
      sum += __builtin_amdgcn_exp2f(fmaf(Store<T>::load1(sr + j), kLog2e, -shift));
    sum = group_sum<kWave>(sum);
    const float rinv = (sum > 0.0f) ? 1.0f / sum : 0.0f;
    for (int b0 = 0; b0 < Sk; b0 += kDrawBlock) {  // uniform over the wave
      KeepBlock keep;
      if (out) keep.draw(row * Sk + b0, lane, rng);
      for (int c0 = b0; c0 < min(b0 + kDrawBlock, Sk); c0 += kWave) {
        const int j = c0 + lane;
        const int64_t e = row * Sk + j;
        const bool kb = out ? keep.kept(e) : false;
        if (j < Sk) {
          float p = 0.0f;
          if (j < limit)
            p = Store<T>::round(
                __builtin_amdgcn_exp2f(fmaf(Store<T>::load1(sr + j), kLog2e, -shift)) * rinv);
          Store<T>::store1(probs + e, p);
          if (out) Store<T>::store1(out + e, kb ? p * scale : 0.0f);
        }
      }
    }
  }
}

// Mask words for shapes whose rows do not end on chunk boundaries: one thread per word.
__global__ __launch_bounds__(kThreads) void keep_words_kernel(uint32_t* __restrict__ keep_bits,
                                                             int64_t n, RngArgs rng) {
  const int64_t words = (n + 31) >> 5;
  for (int64_t w = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; w < words;
       w += static_cast<int64_t>(gridDim.x) * kThreads) {
    uint32_t word = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) word |= keep_byte(static_cast<uint64_t>(w) * 4 + b, rng) << (8 * b);
    const int64_t left = n - w * 32;
    if (left < 32) word &= (1u << left) - 1u;
    keep_bits[w] = word;
  }
}

template <typename T, MaskSource MASK>
__global__ __launch_bounds__(kThreads) void attn_bwd_generic_kernel(
    const T* dout, const T* __restrict__ probs, const uint32_t* __restrict__ keep_bits,
    T* dscores, T* __restrict__ out_re, int64_t rows, int Sk, float scale, RngArgs rng) {
  auto stored = [&](int64_t e) -> bool {
    if constexpr (MASK == kMaskBools) return reinterpret_cast<const uint8_t*>(keep_bits)[e] != 0;
    else return (keep_bits[e >> 5] >> (e & 31)) & 1u;
  };
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  constexpr int kWaves = kThreads / kWave;
  for (int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + wave; row < rows;
       row += static_cast<int64_t>(gridDim.x) * kWaves) {
    float dot = 0.0f;
    for (int b0 = 0; b0 < Sk; b0 += kDrawBlock) {  // uniform over the wave
      KeepBlock keep;
      if constexpr (MASK == kMaskRegen) keep.draw(row * Sk + b0, lane, rng);
      for (int c0 = b0; c0 < min(b0 + kDrawBlock, Sk); c0 += kWave) {
        const int j = c0 + lane;
        const int64_t e = row * Sk + j;
        bool k = false;
        if constexpr (MASK == kMaskRegen) k = keep.kept(e);
        else if (j < Sk) k = stored(e);
        if (j < Sk) {
          const float dp = k ? Store<T>::load1(dout + e) * scale : 0.0f;
          dot = fmaf(dp, Store<T>::load1(probs + e), dot);
        }
      }
    }
    dot = group_sum<kWave>(dot);
    for (int b0 = 0; b0 < Sk; b0 += kDrawBlock) {
      KeepBlock keep;
      if constexpr (MASK == kMaskRegen) keep.draw(row * Sk + b0, lane, rng);
      for (int c0 = b0; c0 < min(b0 + kDrawBlock, Sk); c0 += kWave) {
        const int j = c0 + lane;
        const int64_t e = row * Sk + j;
        bool k = false;
        if constexpr (MASK == kMaskRegen) k = keep.kept(e);
        else if (j < Sk) k = stored(e);
        if (j < Sk) {
          const float p = Store<T>::load1(probs + e);
          const float dp = k ? Store<T>::load1(dout + e) * scale : 0.0f;
          Store<T>::store1(dscores + e, p * (dp - dot));
          if (out_re) Store<T>::store1(out_re + e, k ? p * scale : 0.0f);
        }
      }
    }
  }
}

// ---- any Sk up to 64 * KMAX: one wave per row, scalar accesses, the row held in registers ---
// Element j of a row belongs to lane j % 64 (chunk k = j / 64), so every access of a wave is one
// contiguous run whatever the row's alignment, and the row is read once.  Same arithmetic, in the
// same order per lane, as the any-length kernels above.

// Keep bits of the chunks of such a row.  One generator call yields the bits of 8 consecutive
// elements, so instead of one call per element each lane draws one group of a block of 7 chunks
// (448 elements: at most 57 groups, whatever the block's alignment) and the lanes fetch the byte
// of their element's group from the lane that drew it.
constexpr int kChunksPerDraw = 7;
template <int KMAX>
struct RowKeep {
  static constexpr int kBlocks = (KMAX + kChunksPerDraw - 1) / kChunksPerDraw;
  uint32_t bytes[kBlocks];
  int64_t e_row;
  __device__ __forceinline__ void draw(int64_t row_start, int Sk, int lane, const RngArgs& rng) {
    e_row = row_start;
#pragma unroll
    for (int b = 0; b < kBlocks; ++b) {
      bytes[b] = 0;
      if (b * kChunksPerDraw * kWave < Sk)  // uniform over the wave
        bytes[b] = keep_byte(
            static_cast<uint64_t>((e_row + b * kChunksPerDraw * kWave) >> 3) + lane, rng);
    }
  }
  // Every lane of the wave has to make the call (cross-lane fetch), also lanes beyond the row.
  __device__ __forceinline__ bool kept(int k, int lane) const {
    const int b = k / kChunksPerDraw;
    const int64_t e = e_row + k * kWave + lane;
    const int src = static_cast<int>((e >> 3) - ((e_row + b * kChunksPerDraw * kWave) >> 3));
    return (__shfl(bytes[b], src, kWave) >> (e & 7)) & 1u;
  }
};

// The stored keep bits of such a row: the row's words (at most 2 per lane: 64 * KMAX elements
// span up to 2 * KMAX + 1 words) are loaded once, one per lane, and fetched across lanes, instead
// of one load per element.
template <int KMAX>
struct RowMaskWords {
  static constexpr int kRegs = (2 * KMAX + 1 + kWave - 1) / kWave;
  uint32_t w[kRegs];
  int64_t e_row;
  __device__ __forceinline__ void load(const uint32_t* keep_bits, int64_t row_start,
                                       int64_t total_words, int lane) {
    e_row = row_start;
#pragma unroll
    for (int r = 0; r < kRegs; ++r) {
      const int64_t i = (e_row >> 5) + r * kWave + lane;
      w[r] = (i < total_words) ? keep_bits[i] : 0u;
    }
  }
  // Every lane of the wave has to make the call, also lanes beyond the row.
  __device__ __forceinline__ bool kept(int k, int lane) const {
    const int64_t e = e_row + k * kWave + lane;
    const int wi = static_cast<int>((e >> 5) - (e_row >> 5));
    uint32_t word = __shfl(w[0], wi & (kWave - 1), kWave);
    if constexpr (kRegs > 1) {
      const uint32_t hi = __shfl(w[1], wi & (kWave - 1), kWave);
      word = wi < kWave ? word : hi;
    }
    return (word >> (e & 31)) & 1u;
  }
};

template <typename T, int KMAX>
__global__ __launch_bounds__(kThreads) void attn_fwd_rows_kernel(
    const T* scores, const int32_t* __restrict__ key_len, int causal, T* probs,
    T* __restrict__ out, int64_t rows, int64_t rows_per_batch, int Sq, int Sk, float scale,
    RngArgs rng) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: row math stays scalar
  constexpr int kWaves = kThreads / kWave;
  for (int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + wave; row < rows;
       row += static_cast<int64_t>(gridDim.x) * kWaves) {
    const int key_limit = key_len ? min(max(key_len[row / rows_per_batch], 0), Sk) : Sk;
    const int limit = row_limit(static_cast<int>(row % Sq), key_limit, causal, Sq, Sk);
    const T* sr = scores + row * Sk;
    T* pr = probs + row * Sk;
    T* orow = out ? out + row * Sk : nullptr;
    float v[KMAX];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      const int j = k * kWave + lane;
      v[k] = -INFINITY;
      if (k * kWave < limit) {  // uniform over the wave
        if (j < limit) v[k] = Store<T>::load1(sr + j);
        mx = fmaxf(mx, v[k]);
      }
    }
    mx = group_max<kWave>(mx);
    const float shift = (mx == -INFINITY) ? 0.0f : mx * kLog2e;
    float sum = 0.0f;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      const int j = k * kWave + lane;
      float e = 0.0f;
      if (k * kWave < limit && j < limit) {
        e = __builtin_amdgcn_exp2f(fmaf(v[k], kLog2e, -shift));
        sum += e;
      }
      v[k] = e;
    }
    sum = group_sum<kWave>(sum);
    const float rinv = (sum > 0.0f) ? 1.0f / sum : 0.0f;
    RowKeep<KMAX> keep;
    if (out) keep.draw(row * Sk, Sk, lane, rng);
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      if (k * kWave < Sk) {  // uniform over the wave
        const int j = k * kWave + lane;
        const float p = (j < limit) ? Store<T>::round(v[k] * rinv) : 0.0f;
        const bool kb = out ? keep.kept(k, lane) : false;
        if (j < Sk) {
          Store<T>::store1(pr + j, p);
          if (out) Store<T>::store1(orow + j, kb ? p * scale : 0.0f);
        }
      }
    }
  }
}

template <typename T, MaskSource MASK, int KMAX>
__global__ __launch_bounds__(kThreads) void attn_bwd_rows_kernel(
    const T* dout, const T* __restrict__ probs, const uint32_t* __restrict__ keep_bits,
    T* dscores, T* __restrict__ out_re, int64_t rows, int Sk, float scale, RngArgs rng) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: row math stays scalar
  constexpr int kWaves = kThreads / kWave;
  for (int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + wave; row < rows;
       row += static_cast<int64_t>(gridDim.x) * kWaves) {
    const int64_t e_row = row * Sk;
    RowKeep<KMAX> keep;
    RowMaskWords<KMAX> stored;
    if constexpr (MASK == kMaskRegen) keep.draw(e_row, Sk, lane, rng);
    if constexpr (MASK == kMaskWords) stored.load(keep_bits, e_row, (rows * Sk + 31) >> 5, lane);
    const T* do_row = dout + e_row;
    const T* p_row = probs + e_row;
    T* ds_row = dscores + e_row;
    T* or_row = out_re ? out_re + e_row : nullptr;
    float dp[KMAX], pr[KMAX];
    uint32_t kept_bits = 0;  // bit k: element k * 64 + lane is kept
    float dot = 0.0f;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      dp[k] = pr[k] = 0.0f;
      if (k * kWave < Sk) {  // uniform over the wave
        const int j = k * kWave + lane;
        const int64_t e = e_row + j;
        bool kb = false;
        if constexpr (MASK == kMaskRegen) {
          kb = keep.kept(k, lane);
        } else if constexpr (MASK == kMaskWords) {
          kb = stored.kept(k, lane);
        } else if (j < Sk) {
          kb = reinterpret_cast<const uint8_t*>(keep_bits)[e] != 0;
        }
        if (j < Sk) {
          pr[k] = Store<T>::load1(p_row + j);
          dp[k] = kb ? Store<T>::load1(do_row + j) * scale : 0.0f;
          dot = fmaf(dp[k], pr[k], dot);
          kept_bits |= (kb ? 1u : 0u) << k;
        }
      }
    }
    dot = group_sum<kWave>(dot);
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      const int j = k * kWave + lane;
      if (k * kWave < Sk && j < Sk) {
        Store<T>::store1(ds_row + j, pr[k] * (dp[k] - dot));
        if (out_re) Store<T>::store1(or_row + j, ((kept_bits >> k) & 1u) ? pr[k] * scale : 0.0f);
      }
    }
  }
}

// Chunks of 64 elements a row of Sk elements needs in registers: 4, 16 or 32; 0: too long.
int row_chunks(int64_t Sk) { return Sk <= 256 ? 4 : (Sk <= 1024 ? 16 : (Sk <= 2048 ? 32 : 0)); }
template <typename F>
void with_row_chunks(int kmax, F&& f) {
  if (kmax == 4) f(std::integral_constant<int, 4>{});
  else if (kmax == 16) f(std::integral_constant<int, 16>{});
  else f(std::integral_constant<int, 32>{});
}

struct Shape {
  int lanes;
  int ch;
};

// One piece per lane while the row fits in a wave (every access of a wave is then one
// contiguous run of 16-byte pieces), more pieces per lane for longer rows.  min_lanes: 4 for
// bfloat16, 8 for float32 (the lanes that share a mask word).  ch == 0: row too long.
Shape pick_shape(int pieces, int min_lanes) {
  int lanes = min_lanes;
  while (lanes < 64 && lanes < pieces) lanes <<= 1;
  const int need = (pieces + lanes - 1) / lanes;
  static const int allowed[] = {1, 2, 3, 4, 6, 8, 12, 16};
  for (int a : allowed)
    if (a >= need) return {lanes, lanes == 64 || a == 1 ? a : 0};
  return {0, 0};
}

// A row whose pieces per lane on one wave would exceed max_ch is spread over 2 or 4 waves (at
// most 4 pieces per lane there).
Shape pick_wide_shape(int pieces, int min_lanes, int max_ch) {
  const Shape one = pick_shape(pieces, min_lanes);
  if (one.lanes == kWave && (one.ch == 0 || one.ch > max_ch)) {
    for (int lanes = 2 * kWave; lanes <= kThreads; lanes *= 2) {
      const int need = (pieces + lanes - 1) / lanes;
      if (need <= max_ch || lanes == kThreads) {
        if (need <= 4) return {lanes, need};
        break;
      }
    }
  }
  return one;
}

// Rows a lane group of the forward kernel fetches at once: 2 (if the knob allows) when a
// bfloat16 row is exactly one piece per lane of a whole wave, else 1.  Measured in steady state
// on rows of 128..1024 elements: 2 rows gain 5-7 % there (512 columns) and lose 3-9 % for
// shorter rows (several rows per wave already), for two pieces per lane and for float32;
// backward always takes 1.
int attn_rows(int ch, int lanes, int vec, int tuned) {
  return (vec == 8 && ch == 1 && lanes == kWave && tuned >= 2) ? 2 : 1;
}

// Lanes per workgroup of the register-resident kernels.  Small workgroups come and go
// independently, which the memory system rewards: against workgroups of four waves, two waves
// gain 2-8 % (forward at every size, backward on tensors from 2 GB up, never a loss); single
// waves do no better than two and lose 1-2 % in places.  So: two waves, and never fewer lanes
// than a row takes.
int group_threads(int lanes) {
  const int least = lanes > kWave ? lanes : kWave;  // 64, 128 or 256
  int want = tune_get(kTuneAttnThreads);
  want = want >= 256 ? 256 : (want >= 128 ? 128 : kWave);
  return want > least ? want : least;
}

int row_grid(int64_t rows, int lanes, int blocks_per_cu, int rows_per_group = 1, int threads = kThreads) {
  const int groups = (threads / lanes) * rows_per_group;
  const int64_t want = (rows + groups - 1) / groups;
  const int64_t cap = static_cast<int64_t>(compute_units()) * blocks_per_cu;
  const int64_t b = want < cap ? want : cap;
  return static_cast<int>(b < 1 ? 1 : b);
}

}  // namespace

// LAUNCH(lanes, pieces per lane); the rows per lane group come from attn_rows().
#define TEMPO_ATTN_DISPATCH(LAUNCH)                                                        \
  switch (sh.lanes * 100 + sh.ch) {                                                        \
    case 401: LAUNCH(4, 1); break;                                                         \
    case 801: LAUNCH(8, 1); break;                                                         \
    case 1601: LAUNCH(16, 1); break;                                                       \
    case 3201: LAUNCH(32, 1); break;                                                       \
    case 6401: LAUNCH(64, 1); break;                                                       \
    case 6402: LAUNCH(64, 2); break;                                                       \
    case 6403: LAUNCH(64, 3); break;                                                       \
    case 6404: LAUNCH(64, 4); break;                                                       \
    case 6406: LAUNCH(64, 6); break;                                                       \
    case 6408: LAUNCH(64, 8); break;                                                       \
    case 6412: LAUNCH(64, 12); break;                                                      \
    case 6416: LAUNCH(64, 16); break;                                                      \
    default: return TEMPO_ERR_UNSUPPORTED;                                                 \
  }

#define TEMPO_ATTN_WIDE_DISPATCH(LAUNCH)                                                   \
  switch (sh.lanes * 100 + sh.ch) {                                                        \
    case 12801: LAUNCH(128, 1); break;                                                     \
    case 12802: LAUNCH(128, 2); break;                                                     \
    case 12803: LAUNCH(128, 3); break;                                                     \
    case 12804: LAUNCH(128, 4); break;                                                     \
    case 25601: LAUNCH(256, 1); break;                                                     \
    case 25602: LAUNCH(256, 2); break;                                                     \
    case 25603: LAUNCH(256, 3); break;                                                     \
    case 25604: LAUNCH(256, 4); break;                                                     \
    default: return TEMPO_ERR_UNSUPPORTED;                                                 \
  }

// Calls f with the workgroup size as a compile-time constant (64, 128 or 256, at least L).
template <int L, typename F>
static void with_threads(int threads, F&& f) {
  using std::integral_constant;
  if constexpr (L <= 64) {
    if (threads == 64) return f(integral_constant<int, 64>{});
  }
  if constexpr (L <= 128) {
    if (threads == 128) return f(integral_constant<int, 128>{});
  }
  f(integral_constant<int, 256>{});
}

template <typename T, int L, int C>
static void attn_fwd_go(int rr, bool words, int threads, dim3 grid, hipStream_t st,
                        const void* scores, const int32_t* key_len, int causal, void* probs,
                        void* out, uint32_t* keep_bits, int slices, int64_t A, int64_t Sq,
                        int64_t Sk, float scale, const RngArgs& rng) {
  auto go = [&](auto rows, auto w) {
    with_threads<L>(threads, [&](auto th) {
      constexpr int TH = decltype(th)::value;
      hipLaunchKernelGGL(
          (attn_fwd_kernel<T, L, C, decltype(rows)::value, decltype(w)::value, TH>), grid, dim3(TH),
          0, st, static_cast<const T*>(scores), key_len, causal, static_cast<T*>(probs),
          static_cast<T*>(out), keep_bits, slices, static_cast<int>(A), static_cast<int>(Sq),
          static_cast<int>(Sk), scale, rng);
    });
  };
  using std::integral_constant;
  if constexpr (C <= 2 && L <= kWave) {
    if (rr == 2) {
      if (words) return go(integral_constant<int, 2>{}, std::true_type{});
      return go(integral_constant<int, 2>{}, std::false_type{});
    }
  }
  if (words) return go(integral_constant<int, 1>{}, std::true_type{});
  go(integral_constant<int, 1>{}, std::false_type{});
}

template <typename T, int L, int C>
static void attn_bwd_go(MaskSource mask, int threads, int grid, hipStream_t st, const void* dout,
                        const void* probs, const uint32_t* keep_bits, void* dscores, void* out_re,
                        int64_t rows, int64_t Sk, float scale, const RngArgs& rng) {
  auto go = [&](auto m) {
    with_threads<L>(threads, [&](auto th) {
      constexpr int TH = decltype(th)::value;
      hipLaunchKernelGGL((attn_bwd_kernel<T, L, C, 1, decltype(m)::value, TH>), dim3(grid), dim3(TH),
                         0, st, static_cast<const T*>(dout), static_cast<const T*>(probs), keep_bits,
                         static_cast<T*>(dscores), static_cast<T*>(out_re),
                         static_cast<uint32_t>(rows), static_cast<int>(Sk), scale, rng);
    });
  };
  using std::integral_constant;
  if (mask == kMaskWords) return go(integral_constant<MaskSource, kMaskWords>{});
  if (mask == kMaskBytes) return go(integral_constant<MaskSource, kMaskBytes>{});
  if (mask == kMaskBools) return go(integral_constant<MaskSource, kMaskBools>{});
  go(integral_constant<MaskSource, kMaskRegen>{});
}

static RngArgs make_rng(float p, uint64_t seed, uint64_t offset) {
  RngArgs rng;
  rng.seed_lo = static_cast<uint32_t>(seed);
  rng.seed_hi = static_cast<uint32_t>(seed >> 32);
  rng.off_lo = static_cast<uint32_t>(offset);
  rng.off_hi = static_cast<uint32_t>(offset >> 32);
  double t = (1.0 - static_cast<double>(p)) * 65536.0 + 0.5;
  t = t < 0.0 ? 0.0 : (t > 65536.0 ? 65536.0 : t);
  rng.t16 = (p == 0.0f) ? 65536u : static_cast<uint32_t>(t);  // floor for t >= 0
  return rng;
}

tempo_status launch_attn_fwd(const void* scores, const int32_t* key_len, int causal, void* probs,
                             void* out, uint32_t* keep_bits, int64_t B, int64_t A, int64_t Sq,
                             int64_t Sk, float p, uint64_t seed, uint64_t offset, tempo_dtype dt,
                             hipStream_t st) {
  const int64_t rows = B * A * Sq;
  const int64_t rows_per_batch = A * Sq;
  const float scale = 1.0f / (1.0f - p);
  const RngArgs rng = make_rng(p, seed, offset);
  const int bpc = tune_get(kTuneAttnFwdBlocksPerCu);
  const int vec = dt == TEMPO_F32 ? 4 : 8;
  Shape sh = pick_wide_shape(static_cast<int>(Sk / vec), 32 / vec,
                            tune_get(kTuneAttnFwdMaxPieces));
  if (Sk % 8 == 0 && sh.ch != 0 && rows <= UINT32_MAX) {  // rows counted in 32 bits
    const int slices = static_cast<int>(B * A);
    const int rr = sh.lanes > kWave ? 1 : attn_rows(sh.ch, sh.lanes, vec, tune_get(kTuneAttnFwdRows));
    const int threads = group_threads(sh.lanes);
    const int rows_per_set = (threads / sh.lanes) * rr;
    const int64_t total_sets =
        static_cast<int64_t>(slices) * ((Sq + rows_per_set - 1) / rows_per_set);
    const int64_t cap = static_cast<int64_t>(compute_units()) * bpc;
    const dim3 grid(static_cast<unsigned>(total_sets < cap ? total_sets : cap));
    const bool words = (Sk % 32 == 0);
#define TEMPO_LAUNCH(L, C)                                                                   \
  do {                                                                                       \
    if (dt == TEMPO_F32) attn_fwd_go<float, L, C>(rr, words, threads, grid, st, scores, key_len, causal, probs, out, keep_bits, slices, A, Sq, Sk, scale, rng);   \
    else attn_fwd_go<bf16_t, L, C>(rr, words, threads, grid, st, scores, key_len, causal, probs, out, keep_bits, slices, A, Sq, Sk, scale, rng);                  \
  } while (0)
    if (sh.lanes > kWave) {
      TEMPO_ATTN_WIDE_DISPATCH(TEMPO_LAUNCH)
    } else {
      TEMPO_ATTN_DISPATCH(TEMPO_LAUNCH)
    }
#undef TEMPO_LAUNCH
    return launch_status();
  }
  const int grid = row_grid(rows, kWave, bpc);
  if (const int kmax = row_chunks(Sk)) {
    with_row_chunks(kmax, [&](auto km) {
      constexpr int KM = decltype(km)::value;
      if (dt == TEMPO_F32)
        hipLaunchKernelGGL((attn_fwd_rows_kernel<float, KM>), dim3(grid), dim3(kThreads), 0, st,
                           static_cast<const float*>(scores), key_len, causal,
                           static_cast<float*>(probs), static_cast<float*>(out), rows,
                           rows_per_batch, static_cast<int>(Sq), static_cast<int>(Sk), scale, rng);
      else
        hipLaunchKernelGGL((attn_fwd_rows_kernel<bf16_t, KM>), dim3(grid), dim3(kThreads), 0, st,
                           static_cast<const bf16_t*>(scores), key_len, causal,
                           static_cast<bf16_t*>(probs), static_cast<bf16_t*>(out), rows,
                           rows_per_batch, static_cast<int>(Sq), static_cast<int>(Sk), scale, rng);
    });
  } else if (dt == TEMPO_F32)
    hipLaunchKernelGGL((attn_fwd_generic_kernel<float>), dim3(grid), dim3(kThreads), 0, st,
                       static_cast<const float*>(scores), key_len, causal,
                       static_cast<float*>(probs), static_cast<float*>(out), rows, rows_per_batch,
                       static_cast<int>(Sq), static_cast<int>(Sk), scale, rng);
  else
    hipLaunchKernelGGL((attn_fwd_generic_kernel<bf16_t>), dim3(grid), dim3(kThreads), 0, st,
                       static_cast<const bf16_t*>(scores), key_len, causal,
                       static_cast<bf16_t*>(probs), static_cast<bf16_t*>(out), rows,
                       rows_per_batch, static_cast<int>(Sq), static_cast<int>(Sk), scale, rng);
  if (hipGetLastError() != hipSuccess) return TEMPO_ERR_LAUNCH;
  const int64_t n = rows * Sk;
  const int64_t words = (n + 31) / 32;
  const int64_t wgrid = (words + kThreads - 1) / kThreads;
  const int64_t cap = static_cast<int64_t>(compute_units()) * 8;
  hipLaunchKernelGGL(keep_words_kernel, dim3(static_cast<int>(wgrid < cap ? wgrid : cap)),
                     dim3(kThreads), 0, st, keep_bits, n, rng);
  return launch_status();
}

// keep_bits == nullptr: no stored mask, the bits are drawn again from (seed, offset).
// bools: keep_bits points to one byte per element instead of packed bits.
static tempo_status attn_bwd_any(const void* dout, const void* probs, const uint32_t* keep_bits,
                                 bool bools, void* dscores, void* out_re, int64_t B, int64_t A,
                                 int64_t Sq, int64_t Sk, float p, const RngArgs& rng,
                                 tempo_dtype dt, hipStream_t st) {
  const int64_t rows = B * A * Sq;
  const float scale = 1.0f / (1.0f - p);
  const bool regen = keep_bits == nullptr;
  const int bpc = tune_get(kTuneAttnBwdBlocksPerCu);
  const int vec = dt == TEMPO_F32 ? 4 : 8;
  Shape sh = pick_wide_shape(static_cast<int>(Sk / vec), 32 / vec,
                            tune_get(kTuneAttnBwdMaxPieces));
  if (Sk % 8 == 0 && sh.ch != 0 && rows <= UINT32_MAX) {  // rows counted in 32 bits
    const int threads = group_threads(sh.lanes);
    const int grid = row_grid(rows, sh.lanes, bpc, 1, threads);
    const MaskSource mask =
        regen ? kMaskRegen : (bools ? kMaskBools : (Sk % 32 == 0 ? kMaskWords : kMaskBytes));
#define TEMPO_LAUNCH(L, C)                                                                   \
  do {                                                                                       \
    if (dt == TEMPO_F32) attn_bwd_go<float, L, C>(mask, threads, grid, st, dout, probs, keep_bits, dscores, out_re, rows, Sk, scale, rng);   \
    else attn_bwd_go<bf16_t, L, C>(mask, threads, grid, st, dout, probs, keep_bits, dscores, out_re, rows, Sk, scale, rng);                  \
  } while (0)
    if (sh.lanes > kWave) {
      TEMPO_ATTN_WIDE_DISPATCH(TEMPO_LAUNCH)
    } else {
      TEMPO_ATTN_DISPATCH(TEMPO_LAUNCH)
    }
#undef TEMPO_LAUNCH
    return launch_status();
  }
  const int grid = row_grid(rows, kWave, bpc);
  const int kmax = row_chunks(Sk);
  auto go = [&](auto tag, auto m) {
    using T = decltype(tag);
    if (kmax) {
      with_row_chunks(kmax, [&](auto km) {
        hipLaunchKernelGGL((attn_bwd_rows_kernel<T, decltype(m)::value, decltype(km)::value>),
                           dim3(grid), dim3(kThreads), 0, st, static_cast<const T*>(dout),
                           static_cast<const T*>(probs), keep_bits, static_cast<T*>(dscores),
                           static_cast<T*>(out_re), rows, static_cast<int>(Sk), scale, rng);
      });
      return;
    }
    hipLaunchKernelGGL((attn_bwd_generic_kernel<T, decltype(m)::value>), dim3(grid),
                       dim3(kThreads), 0, st, static_cast<const T*>(dout),
                       static_cast<const T*>(probs), keep_bits, static_cast<T*>(dscores),
                       static_cast<T*>(out_re), rows, static_cast<int>(Sk), scale, rng);
  };
  using std::integral_constant;
  auto with_mask = [&](auto tag) {
    if (regen) go(tag, integral_constant<MaskSource, kMaskRegen>{});
    else if (bools) go(tag, integral_constant<MaskSource, kMaskBools>{});
    else go(tag, integral_constant<MaskSource, kMaskWords>{});
  };
  if (dt == TEMPO_F32) with_mask(float{});
  else with_mask(bf16_t{});
  return launch_status();
}

tempo_status launch_attn_bwd(const void* dout, const void* probs, const uint32_t* keep_bits,
                             void* dscores, void* out_re, int64_t B, int64_t A, int64_t Sq,
                             int64_t Sk, float p, tempo_dtype dt, hipStream_t st) {
  return attn_bwd_any(dout, probs, keep_bits, false, dscores, out_re, B, A, Sq, Sk, p,
                      make_rng(0.0f, 0, 0), dt, st);
}

tempo_status launch_attn_bwd_bytemask(const void* dout, const void* probs,
                                      const uint8_t* keep_bytes, void* dscores, void* out_re,
                                      int64_t B, int64_t A, int64_t Sq, int64_t Sk, float p,
                                      tempo_dtype dt, hipStream_t st) {
  return attn_bwd_any(dout, probs, reinterpret_cast<const uint32_t*>(keep_bytes), true, dscores,
                      out_re, B, A, Sq, Sk, p, make_rng(0.0f, 0, 0), dt, st);
}

tempo_status launch_attn_bwd_regen(const void* dout, const void* probs, void* dscores,
                                   void* out_re, int64_t B, int64_t A, int64_t Sq, int64_t Sk,
                                   float p, uint64_t seed, uint64_t offset, tempo_dtype dt,
                                   hipStream_t st) {
  return attn_bwd_any(dout, probs, nullptr, false, dscores, out_re, B, A, Sq, Sk, p,
                      make_rng(p, seed, offset), dt, st);
}

}  // namespace tempo
