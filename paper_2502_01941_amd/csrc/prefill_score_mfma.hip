// Window-attention softmax partials on the gfx950 matrix cores (Section 5.1, Eq. 3: alpha_{t,h}).
//
// Shape: bf16, head_dim 128, up to 256 query rows (G*W) per KV head, instantiated for 1, 2, 4, 6 or 8
// blocks of 32 rows; rows past G*W are zero operands whose statistics are written as -inf.
//
// A workgroup is a pair of waves (one wave for a single row block) that takes the chunks starting inside
// one slice of a KV head's key axis and walks that contiguous span in blocks of 32 keys.  Each wave keeps
// its share of the window queries in registers as MFMA B operands and computes
// S^T[32 keys x 32 queries] = K_blk * Q^T per row block with v_mfma_f32_32x32x16_bf16.  Keys run along the
// accumulator registers and queries along the lanes, so the row-softmax statistics (max and sum over
// keys) are in-lane reductions; only the two lane halves are merged, once per chunk.  A block that
// contains a chunk boundary credits its weights to the chunks on either side with masked in-lane sums.
//
// K blocks are streamed global -> LDS with 16-byte direct-to-LDS loads (whole 256-byte rows, fully
// coalesced; each wave fetches half of every block) into a ring of three buffers, so two blocks are
// in flight while one is being consumed; both waves read the whole block back in MFMA A-operand
// layout.  One s_barrier per block tells the pair that a block has landed and that the buffer of the
// block before it may be refilled.  With ~166 registers per wave three waves fit on a SIMD.
//
// LDS layout of a block: key row r starts at r*256 + (r/4)*64 and its 16-byte column c sits in slot
// c ^ (r%4).  The 64-byte pad per four rows plus the two-bit XOR spread the 16 lanes of a 128-bit LDS
// read over all banks, while the address of MFMA step ks stays (lane base for ks parity) + 64*(ks/2),
// i.e. an immediate offset - no per-step address registers.
//
// The direct-to-LDS loads are written as inline assembly and their completion is tracked by hand with
// s_waitcnt vmcnt: when they are visible to the compiler it makes every LDS read wait for all loads
// in flight, including the prefetched blocks, which serialises load and compute.  Unknown
// vector-memory operations can only make the compiler's own waits stricter, never too weak, because
// loads complete in order.
#include "common.hpp"

namespace shotkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) const char lds_cchar;  // keeps LDS reads as ds_read, not flat
typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;

constexpr int kD = 128;
constexpr int kBlockKeys = 32;
constexpr int kRowBytes = kD * 2;                    // 256
constexpr int kGroupBytes = 4 * kRowBytes + 64;      // four rows + pad = one direct-to-LDS instruction
constexpr int kGroupsPerBlock = kBlockKeys / 4;      // 8
constexpr int kBufBytes = kGroupsPerBlock * kGroupBytes;  // 8704 bytes per block
#ifndef SHOTKV_SCORE_RING
#define SHOTKV_SCORE_RING 3
#endif
#ifndef SHOTKV_SCORE_WAVES_PER_SIMD
#define SHOTKV_SCORE_WAVES_PER_SIMD 3
#endif
constexpr int kRing = SHOTKV_SCORE_RING;  // LDS buffers per pair: kRing - 1 blocks in flight
static_assert(kRing >= 2 && kRing <= 5, "ring depth");

// Issue this wave's share of the direct-to-LDS loads of one 32-key block: groups [g0, g0 + NG).
// Group i fills rows 4i..4i+3: lane l writes LDS slot l of the group, which is row 4i + l/16, slot
// l%16, and therefore fetches column (l%16) ^ (l/16) of that row.  Rows past the end of the span
// (rem keys are left in it) re-read its last key (they are masked later), so every address stays inside it.
// The loads carry the non-temporal hint: K is read exactly once, and a stream that does not settle in L2
// and the memory-side cache leaves them to the statistics this kernel writes and the next kernels read
// (measured: 8 % faster here, and the per-chunk reduction that follows finds its input in cache).
template <int NG>
__device__ __forceinline__ void issue_block(const char* __restrict__ k_plane, int key0, int rem,
                                            uint32_t lds_addr, int g0, int lane) {
  const int last = rem - 1;  // rem >= 1
  const int hi = lane >> 4;
  const uint32_t col_bytes = static_cast<uint32_t>(((lane & 15) ^ hi) << 4);
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    const int rr = min(4 * (g0 + i) + hi, last);
    const uint32_t off = static_cast<uint32_t>(key0 + rr) * kRowBytes + col_bytes;
    // M0 = LDS address of the group (wave-uniform); lane l lands at M0 + 16*l
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :
                 : "s"(lds_addr + (g0 + i) * kGroupBytes), "v"(off), "s"(k_plane)
                 : "memory", "m0");
  }
}

// Fold the 16 logits a lane holds for one query (key rows 8*(v/4) + 4*half + v%4 of the block) into
// that query's running (reference, sum) in the log2 domain: sum = sum_k 2^(z_k - reference).
//
// Any reference gives the same softmax once the chunks are combined, so the reference found so far -
// the largest logit of some earlier block, carried over from chunk to chunk - is kept and the
// exponentials are summed against it directly.  That is safe unless a logit exceeds the reference by
// ~2^100 (or there is no reference yet); the case is caught on the sum, wave-uniformly, and the block
// is then redone as the usual online-softmax update, which raises the reference to the block maximum.
// A reference far above a chunk's logits costs nothing that the result could show: it is at most the
// row maximum, so a term that underflows against it underflows in the normalised weight as well.
// Both lane halves of a query always hold the same reference (the maximum is taken over both).
// l_grp is the sum over the workgroup's finished chunks against the same reference; it follows every
// change of the reference.
template <bool MASKED, bool EXACT>
__device__ __forceinline__ void softmax_fold(floatx16 acc, float c, int half, int rem, int key0,
                                             int last_visible, float& m_run, float& l_run, float& l_grp) {
  if (MASKED) {
    // row 8*(v/4) + v%4 + 4*half is masked when it is past the chunk or past the query's position:
    // one per-lane limit, compared against compile-time row constants
    const int limit = min(rem, last_visible - key0 + 1) - 4 * half;
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (8 * (v >> 2) + (v & 3) >= limit) acc[v] = -INFINITY;
  }
  if (!EXACT) {
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int v = 0; v < 16; v += 2) {
      s0 += __builtin_amdgcn_exp2f(fmaf(acc[v], c, -m_run));
      s1 += __builtin_amdgcn_exp2f(fmaf(acc[v + 1], c, -m_run));
    }
    const float s = s0 + s1;
    // wave-uniform decision, so the exact path below is taken by all lanes or none (a lane without a
    // reference yet gets inf or NaN here)
    if (__builtin_amdgcn_ballot_w64(!(s < 0x1p100f)) == 0) {
      l_run += s;
      return;
    }
  }
  float bm = fmaxf(acc[0], acc[1]);
#pragma unroll
  for (int v = 2; v < 16; v += 2) bm = fmaxf(fmaxf(bm, acc[v]), acc[v + 1]);
  bm = max_across_halves(bm);
  const float m_new = fmaxf(m_run, bm * c);
  const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
  float s0 = 0.f, s1 = 0.f;
#pragma unroll
  for (int v = 0; v < 16; v += 2) {
    s0 += __builtin_amdgcn_exp2f(fmaf(acc[v], c, -m_safe));
    s1 += __builtin_amdgcn_exp2f(fmaf(acc[v + 1], c, -m_safe));
  }
  l_run = l_run * alpha + (s0 + s1);
  l_grp *= alpha;
  m_run = m_new;
}

// One 32-key block against this wave's NQW query blocks (qb0 = index of its first one).
template <int NQW, bool MASKED, bool EXACT>
__device__ __forceinline__ void compute_block(lds_cchar* lds_buf, const bf16x8 (&bq)[NQW][8], int lane,
                                              int qb0, int key0, int rem, int causal_base, int W, float c,
                                              float (&m_run)[NQW], float (&l_run)[NQW], float (&l_grp)[NQW]) {
  const int row = lane & 31, half = lane >> 5;
  const int base_even = row * kRowBytes + (row >> 2) * 64 + ((half ^ (row & 3)) << 4);
  lds_cchar* even = lds_buf + base_even;
  lds_cchar* odd = lds_buf + (base_even ^ 32);
  floatx16 acc[NQW];
#pragma unroll
  for (int q = 0; q < NQW; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const bf16x8 a = *reinterpret_cast<lds_bf16x8*>(((ks & 1) ? odd : even) + 64 * (ks >> 1));
#pragma unroll
    for (int q = 0; q < NQW; ++q)
      acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[q][ks], acc[q], 0, 0, 0);
  }
#pragma unroll
  for (int q = 0; q < NQW; ++q) {
    const int last_visible = causal_base + ((qb0 + q) * 32 + row) % W;
    softmax_fold<MASKED, EXACT>(acc[q], c, half, rem, key0, last_visible, m_run[q], l_run[q], l_grp[q]);
  }
}

// The same block when a chunk ends inside it: the exact online-softmax update, then the sixteen weights
// 2^(z - reference) of every query stay in `e` so that the caller can credit them to the chunks on either
// side of each boundary.  Nothing is added to l_run here.
template <int NQW, bool MASKED>
__device__ __forceinline__ void weights_block(lds_cchar* lds_buf, const bf16x8 (&bq)[NQW][8], int lane, int qb0,
                                              int key0, int rem, int causal_base, int W, float c,
                                              float (&m_run)[NQW], float (&l_run)[NQW], float (&l_grp)[NQW],
                                              floatx16 (&e)[NQW]) {
  const int row = lane & 31, half = lane >> 5;
  const int base_even = row * kRowBytes + (row >> 2) * 64 + ((half ^ (row & 3)) << 4);
  lds_cchar* even = lds_buf + base_even;
  lds_cchar* odd = lds_buf + (base_even ^ 32);
#pragma unroll
  for (int q = 0; q < NQW; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) e[q][v] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const bf16x8 a = *reinterpret_cast<lds_bf16x8*>(((ks & 1) ? odd : even) + 64 * (ks >> 1));
#pragma unroll
    for (int q = 0; q < NQW; ++q) e[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[q][ks], e[q], 0, 0, 0);
  }
#pragma unroll
  for (int q = 0; q < NQW; ++q) {
    if (MASKED) {
      const int last_visible = causal_base + ((qb0 + q) * 32 + row) % W;
      const int limit = min(rem, last_visible - key0 + 1) - 4 * half;
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (8 * (v >> 2) + (v & 3) >= limit) e[q][v] = -INFINITY;
    }
    float bm = fmaxf(e[q][0], e[q][1]);
#pragma unroll
    for (int v = 2; v < 16; v += 2) bm = fmaxf(fmaxf(bm, e[q][v]), e[q][v + 1]);
    bm = max_across_halves(bm);
    const float m_new = fmaxf(m_run[q], bm * c);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run[q] - m_safe);
    l_run[q] *= alpha;
    l_grp[q] *= alpha;
    m_run[q] = m_new;
#pragma unroll
    for (int v = 0; v < 16; ++v) e[q][v] = __builtin_amdgcn_exp2f(fmaf(e[q][v], c, -m_safe));
  }
}

// Crediting the weights of a block to the chunks on either side of a boundary.  A lane holds key rows
// 8*(v/4) + v%4 of the block (+4 in the upper lane half) in element v, in ascending order, and a boundary
// is the same for the whole wave, so "element v lies in the interval" is one bit per lane half: the set
// of a half's elements is a 16-bit scalar mask.  The adds then run under an execution mask made from bit
// v of the two masks (s_bfe_i32 gives 0 or -1 for exec_lo / exec_hi): one vector add per weight and no
// vector compares or selects.  Even and odd elements go to separate accumulators (two dependency chains).

// elements of a lower-half lane whose row is below x, as a bit mask
__device__ __forceinline__ uint32_t elements_below(int x) {
  if (x <= 0) return 0u;
  const int n = min(4 * (x >> 3) + min(x & 7, 4), 16);
  return (1u << n) - 1u;
}

#define SHOTKV_MASKED_STEP2(V, ACC_A, ACC_B, XA, XB)                          \
  "s_bfe_i32 exec_lo, %[s0], 0x1000" #V "\n\t"                                \
  "s_bfe_i32 exec_hi, %[s1], 0x1000" #V "\n\t"                                \
  "v_add_f32 %[" #ACC_A "], %[" #ACC_A "], %[" #XA "]\n\t"                    \
  "v_add_f32 %[" #ACC_B "], %[" #ACC_B "], %[" #XB "]\n\t"
#define SHOTKV_MASKED_STEP1(V, ACC_A, XA)                                     \
  "s_bfe_i32 exec_lo, %[s0], 0x1000" #V "\n\t"                                \
  "s_bfe_i32 exec_hi, %[s1], 0x1000" #V "\n\t"                                \
  "v_add_f32 %[" #ACC_A "], %[" #ACC_A "], %[" #XA "]\n\t"

// elements 8*HALF .. 8*HALF+7 of two queries' weights; s0 / s1 already shifted so that bit i is element 8*HALF + i
__device__ __forceinline__ void masked_add8(float& ae, float& ao, float& be, float& bo, float a0, float a1,
                                            float a2, float a3, float a4, float a5, float a6, float a7,
                                            float b0, float b1, float b2, float b3, float b4, float b5,
                                            float b6, float b7, uint32_t s0, uint32_t s1) {
  uint64_t save;
  asm volatile("s_mov_b64 %[save], exec\n\t"
               SHOTKV_MASKED_STEP2(0, ae, be, a0, b0) SHOTKV_MASKED_STEP2(1, ao, bo, a1, b1)
               SHOTKV_MASKED_STEP2(2, ae, be, a2, b2) SHOTKV_MASKED_STEP2(3, ao, bo, a3, b3)
               SHOTKV_MASKED_STEP2(4, ae, be, a4, b4) SHOTKV_MASKED_STEP2(5, ao, bo, a5, b5)
               SHOTKV_MASKED_STEP2(6, ae, be, a6, b6) SHOTKV_MASKED_STEP2(7, ao, bo, a7, b7)
               "s_mov_b64 exec, %[save]"
               : [ae] "+v"(ae), [ao] "+v"(ao), [be] "+v"(be), [bo] "+v"(bo), [save] "=&s"(save)
               : [a0] "v"(a0), [a1] "v"(a1), [a2] "v"(a2), [a3] "v"(a3), [a4] "v"(a4), [a5] "v"(a5),
                 [a6] "v"(a6), [a7] "v"(a7), [b0] "v"(b0), [b1] "v"(b1), [b2] "v"(b2), [b3] "v"(b3),
                 [b4] "v"(b4), [b5] "v"(b5), [b6] "v"(b6), [b7] "v"(b7), [s0] "s"(s0), [s1] "s"(s1)
               : "scc");
}

__device__ __forceinline__ void masked_add8(float& ae, float& ao, float a0, float a1, float a2, float a3,
                                            float a4, float a5, float a6, float a7, uint32_t s0, uint32_t s1) {
  uint64_t save;
  asm volatile("s_mov_b64 %[save], exec\n\t"
               SHOTKV_MASKED_STEP1(0, ae, a0) SHOTKV_MASKED_STEP1(1, ao, a1) SHOTKV_MASKED_STEP1(2, ae, a2)
               SHOTKV_MASKED_STEP1(3, ao, a3) SHOTKV_MASKED_STEP1(4, ae, a4) SHOTKV_MASKED_STEP1(5, ao, a5)
               SHOTKV_MASKED_STEP1(6, ae, a6) SHOTKV_MASKED_STEP1(7, ao, a7)
               "s_mov_b64 exec, %[save]"
               : [ae] "+v"(ae), [ao] "+v"(ao), [save] "=&s"(save)
               : [a0] "v"(a0), [a1] "v"(a1), [a2] "v"(a2), [a3] "v"(a3), [a4] "v"(a4), [a5] "v"(a5),
                 [a6] "v"(a6), [a7] "v"(a7), [s0] "s"(s0), [s1] "s"(s1)
               : "scc");
}
#undef SHOTKV_MASKED_STEP2
#undef SHOTKV_MASKED_STEP1

// l_run[q] += sum of the elements of e[q] named by the masks (m0: lower lane half, m1: upper lane half)
template <int NQW>
__device__ __forceinline__ void credit_elements(const floatx16 (&e)[NQW], uint32_t m0, uint32_t m1,
                                                float (&l_run)[NQW]) {
  float se[NQW], so[NQW];
#pragma unroll
  for (int q = 0; q < NQW; ++q) se[q] = so[q] = 0.f;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t s0 = m0 >> (8 * h), s1 = m1 >> (8 * h);
    const int b = 8 * h;
#pragma unroll
    for (int q = 0; q + 1 < NQW; q += 2)
      masked_add8(se[q], so[q], se[q + 1], so[q + 1], e[q][b], e[q][b + 1], e[q][b + 2], e[q][b + 3], e[q][b + 4],
                  e[q][b + 5], e[q][b + 6], e[q][b + 7], e[q + 1][b], e[q + 1][b + 1], e[q + 1][b + 2],
                  e[q + 1][b + 3], e[q + 1][b + 4], e[q + 1][b + 5], e[q + 1][b + 6], e[q + 1][b + 7], s0, s1);
    if (NQW & 1) {
      constexpr int q = NQW - 1;
      masked_add8(se[q], so[q], e[q][b], e[q][b + 1], e[q][b + 2], e[q][b + 3], e[q][b + 4], e[q][b + 5],
                  e[q][b + 6], e[q][b + 7], s0, s1);
    }
  }
#pragma unroll
  for (int q = 0; q < NQW; ++q) l_run[q] += se[q] + so[q];
}

constexpr int kEndCache = 128;  // chunk ends of a workgroup kept in LDS

template <int NQB>
struct PairShape {
#ifndef SHOTKV_SCORE_MAX_WAVES
#define SHOTKV_SCORE_MAX_WAVES 2
#endif
  static constexpr int kWaves = NQB >= SHOTKV_SCORE_MAX_WAVES ? SHOTKV_SCORE_MAX_WAVES : (NQB >= 2 ? 2 : 1);  // waves per workgroup
  static constexpr int kNQW = NQB / kWaves;           // query blocks per wave
  static constexpr int kLoads = kGroupsPerBlock / kWaves;  // load instructions per wave per block
  static constexpr int kThreads = kWaves * kWave;
  // single-wave groups are LDS-limited; four query blocks per wave need the 256-register budget
  static constexpr int kMinWavesPerSimd = kWaves == 1 ? 1 : (kNQW > 2 ? 2 : SHOTKV_SCORE_WAVES_PER_SIMD);
};

template <int NQB>
__global__ __launch_bounds__(PairShape<NQB>::kThreads, PairShape<NQB>::kMinWavesPerSimd) void
score_partials_mfma_kernel(
    const bf16_t* __restrict__ q_obs, const bf16_t* __restrict__ k, int n_tokens, int H, int H_kv, int W,
    int n_rows, float c, const int32_t* __restrict__ group_first, const int32_t* __restrict__ chunk_start,
    const int32_t* __restrict__ chunk_len, int max_c,
    float* __restrict__ partial, float* __restrict__ group_stat) {
  typedef PairShape<NQB> S;
  constexpr int NQW = S::kNQW;
  constexpr int R = NQB * 32;
  __shared__ __attribute__((aligned(64))) char lds[kRing][kBufBytes];
  __shared__ int s_end[kEndCache];

  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int g = blockIdx.y, p = blockIdx.z;
  // this workgroup's chunks: those that start inside its slice of the key axis
  const int32_t* gf = group_first + static_cast<size_t>(p) * (gridDim.x + 1) + blockIdx.x;
  const int c_begin = gf[0], c_end = gf[1];
  if (c_begin >= c_end) {  // no chunk starts here (or the problem's offsets are bad): the whole
                           // workgroup leaves together, before any barrier
    for (int r = threadIdx.x; r < R; r += S::kThreads)
      group_stat[((static_cast<size_t>(p) * H_kv + g) * gridDim.x + blockIdx.x) * R + r] = -INFINITY;
    return;
  }

  const int32_t* cs = chunk_start + static_cast<size_t>(p) * max_c;
  const int32_t* cl = chunk_len + static_cast<size_t>(p) * max_c;
  const char* k_plane =
      reinterpret_cast<const char*>(k) + (static_cast<size_t>(p) * H_kv + g) * n_tokens * kRowBytes;
  const int G = H / H_kv;
  const bf16_t* q_rows = q_obs + (static_cast<size_t>(p) * H + static_cast<size_t>(g) * G) * W * kD;
  float* out = partial + (static_cast<size_t>(p) * max_c * H_kv + g) * R;  // chunk c of this head: + c * H_kv * R
  const int qb0 = wave * NQW;

  // B operands: query row (qb0+q)*32 + lane%32, head-dim slice 16*ks + 8*(lane/32) .. +8
  // Query rows past n_rows = G*W (a row count that is not one of 32/64/128/192/256) are zero operands; their
  // statistics are written as -inf, so they carry no weight further down.
  bf16x8 bq[NQW][8];
#pragma unroll
  for (int q = 0; q < NQW; ++q) {
    const int qi = (qb0 + q) * 32 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (qi < n_rows) raw = *reinterpret_cast<const u32x4*>(q_rows + qi * kD + ks * 16 + (lane >> 5) * 8);
      bq[q][ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }
  // the query loads must have landed before the streaming loop starts: inside the loop the only
  // vector-memory loads are the block loads, whose completion is tracked by hand
#pragma unroll
  for (int q = 0; q < NQW; ++q)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(bq[q][ks]));

  lds_cchar* lds_base = (lds_cchar*)&lds[0][0];
  const uint32_t lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds_base));
  const int causal_base = n_tokens - W;
  const int g0 = wave * S::kLoads;

  float m_run[NQW], l_run[NQW], l_grp[NQW];
#pragma unroll
  for (int q = 0; q < NQW; ++q) { m_run[q] = -INFINITY; l_run[q] = 0.f; l_grp[q] = 0.f; }

  // A finished chunk's statistic, log2(sum_k 2^z_k) per query, waits in registers until kStash chunks
  // have finished (or the stream ends) and is then stored right after a barrier, ahead of that
  // iteration's loads: vector stores share the loads' completion counter, so a store inside the
  // streaming loop puts its own latency into the wait for the next block, and the fewer of them the
  // better.  Both lane halves hold a query's value; chunk j of the batch is kept by the lanes of half
  // j / 4 in slot j % 4.  Row r of the partial array is query (lane%32)*NQB + qb.
  constexpr int kStash = 8;
  float stash[4][NQW];
#pragma unroll
  for (int sl = 0; sl < 4; ++sl)
#pragma unroll
    for (int q = 0; q < NQW; ++q) stash[sl][q] = 0.f;
  int n_stash = 0, stash_c0 = 0;
  const int my_half = lane >> 5;
  auto stash_put = [&](const float (&val)[NQW], int chunk) {
    if (n_stash == 0) stash_c0 = chunk;
    const bool mine = (n_stash >> 2) == my_half;
    const int slot = n_stash & 3;
#pragma unroll
    for (int sl = 0; sl < 4; ++sl)
#pragma unroll
      for (int q = 0; q < NQW; ++q) stash[sl][q] = (mine && sl == slot) ? val[q] : stash[sl][q];
    ++n_stash;
  };
  auto flush = [&]() {
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
      const int j = sl + 4 * my_half;
      if (j < n_stash) {
        float* dst = out + static_cast<size_t>(stash_c0 + j) * H_kv * R + (lane & 31) * NQB + qb0;
        if (NQW == 4) {
          *reinterpret_cast<float4*>(dst) =
              make_float4(stash[sl][0], stash[sl][1 % NQW], stash[sl][2 % NQW], stash[sl][3 % NQW]);
        } else if (NQW == 2) {
          *reinterpret_cast<float2*>(dst) = make_float2(stash[sl][0], stash[sl][NQW - 1]);
        } else {
#pragma unroll
          for (int q = 0; q < NQW; ++q) dst[q] = stash[sl][q];
        }
      }
    }
    n_stash = 0;
  };

  // The workgroup's chunks tile one contiguous span of the key axis, which is walked in blocks of 32
  // keys that take no notice of chunk boundaries: a block that contains a boundary credits its weights
  // to the chunks on either side with masked in-lane sums (sentence-sized units end inside most blocks,
  // shots of hundreds of tokens inside few), and no block carries padding except the span's last.
  // `cur` sits in ring slot cur_buf; up to kLook = kRing - 1 requested blocks follow it in the next slots.
  // A new block is requested each iteration, right after the barrier that frees the slot of the block
  // before cur.
  const int k_begin = cs[c_begin];
  const int k_end = cs[c_end - 1] + cl[c_end - 1];
  // ends of the first chunks go to LDS: one read per boundary instead of a dependent trip to the table
  for (int i = threadIdx.x; i < min(c_end - c_begin, kEndCache); i += S::kThreads)
    s_end[i] = cs[c_begin + i] + cl[c_begin + i];
  __syncthreads();
  auto chunk_end = [&](int ci) {
    const int i = ci - c_begin;
    const int e = i < kEndCache ? s_end[i] : cs[ci] + cl[ci];
    return __builtin_amdgcn_readfirstlane(e);
  };
  constexpr int kLook = kRing - 1;
  auto ring_slot = [](int sl) { return sl >= kRing ? sl - kRing : sl; };
  int cur_key0 = k_begin, next_key0 = k_begin + kBlockKeys;  // next block to request
  issue_block<S::kLoads>(k_plane, k_begin, k_end - k_begin, lds_addr, g0, lane);
  int n_q = 0;
#pragma unroll
  for (int i = 0; i < kLook - 1; ++i) {
    if (next_key0 < k_end) {
      issue_block<S::kLoads>(k_plane, next_key0, k_end - next_key0, lds_addr + (i + 1) * kBufBytes, g0, lane);
      n_q = i + 1;
      next_key0 += kBlockKeys;
    }
  }
  int cur_buf = 0;
  bool first_block = true;
  int cur_c = c_begin, cur_end = chunk_end(c_begin);

  // the current chunk is complete: add up the lane halves (same reference), keep its statistic
  auto finish_chunk = [&]() {
    float val[NQW];
#pragma unroll
    for (int q = 0; q < NQW; ++q) {
      const float l = sum_across_halves(l_run[q]);
      // log2(0) = -inf: a query that saw none of the chunk's keys; so is a padding query row
      val[q] = (l > 0.f && (qb0 + q) * 32 + (lane & 31) < n_rows) ? m_run[q] + __builtin_amdgcn_logf(l)
                                                                   : -INFINITY;
      l_grp[q] += l;
      l_run[q] = 0.f;  // the reference carries over to the next chunk
    }
    if (n_stash == kStash) flush();  // several chunks can end inside one block
    stash_put(val, cur_c);
    ++cur_c;
    cur_end = cur_c < c_end ? chunk_end(cur_c) : INT32_MAX;
  };

  while (true) {
    // this wave's share of `cur` has landed once only the loads of the queued blocks are outstanding
    // (stores of statistics issued meanwhile are younger than those loads and only make the wait stricter)
    if (n_q == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (n_q == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(S::kLoads) : "memory");
    else if (n_q == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * S::kLoads) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * S::kLoads) : "memory");
    // ... and after the barrier so has the partner's; the pair is also done reading the block before
    if (S::kWaves > 1) asm volatile("s_barrier" ::: "memory");
    if (n_stash == kStash) flush();
    if (next_key0 < k_end) {
      issue_block<S::kLoads>(k_plane, next_key0, k_end - next_key0,
                             lds_addr + ring_slot(cur_buf + n_q + 1) * kBufBytes, g0, lane);
      ++n_q;
      next_key0 += kBlockKeys;
    }
    // keys past the end of the span and keys a window query may not see yet are masked; both only
    // happen in the span's last block or in the last W keys, so the common block takes the plain path.
    // The workgroup's first block has no reference yet and takes the exact update straight away.
    const int cur_rem = min(kBlockKeys, k_end - cur_key0);
    const bool masked = cur_rem < kBlockKeys || cur_key0 + kBlockKeys - 1 > causal_base;
    lds_cchar* blk = lds_base + cur_buf * kBufBytes;
    if (cur_end >= cur_key0 + cur_rem) {  // no chunk ends inside the block
      if (first_block)
        compute_block<NQW, true, true>(blk, bq, lane, qb0, cur_key0, cur_rem, causal_base, W, c, m_run, l_run, l_grp);
      else if (masked)
        compute_block<NQW, true, false>(blk, bq, lane, qb0, cur_key0, cur_rem, causal_base, W, c, m_run, l_run, l_grp);
      else
        compute_block<NQW, false, false>(blk, bq, lane, qb0, cur_key0, cur_rem, causal_base, W, c, m_run, l_run, l_grp);
    } else {
      floatx16 e[NQW];
      if (masked)
        weights_block<NQW, true>(blk, bq, lane, qb0, cur_key0, cur_rem, causal_base, W, c, m_run, l_run, l_grp, e);
      else
        weights_block<NQW, false>(blk, bq, lane, qb0, cur_key0, cur_rem, causal_base, W, c, m_run, l_run, l_grp, e);
      uint32_t lo0 = 0u, lo1 = 0u;  // elements already credited (lower / upper lane half)
      do {
        const int hi = cur_end - cur_key0;  // wave-uniform, 1..31
        const uint32_t hi0 = elements_below(hi), hi1 = elements_below(hi - 4);
        credit_elements<NQW>(e, hi0 & ~lo0, hi1 & ~lo1, l_run);
        finish_chunk();
        lo0 = hi0;
        lo1 = hi1;
      } while (cur_end < cur_key0 + cur_rem);
      credit_elements<NQW>(e, 0xffffu & ~lo0, 0xffffu & ~lo1, l_run);
    }
    first_block = false;
    if (cur_end == cur_key0 + cur_rem) finish_chunk();  // the chunk ends with the block
    if (n_q == 0) break;
    cur_key0 += kBlockKeys;
    --n_q;
    cur_buf = ring_slot(cur_buf + 1);
  }
  if (n_stash > 0) flush();
  // the same statistic over all of the workgroup's chunks, from which the row denominators are built
  if (lane < 32) {
    float* dst = group_stat + ((static_cast<size_t>(p) * H_kv + g) * gridDim.x + blockIdx.x) * R +
                 (lane & 31) * NQB + qb0;
#pragma unroll
    for (int q = 0; q < NQW; ++q)
      dst[q] = (l_grp[q] > 0.f && (qb0 + q) * 32 + lane < n_rows) ? m_run[q] + __builtin_amdgcn_logf(l_grp[q])
                                                                 : -INFINITY;
  }
}

}  // namespace

int score_group_keys(int P, int H_kv, int n_tokens, int n_shots) {
#ifdef SHOTKV_SCORE_GROUP_KEYS
  return SHOTKV_SCORE_GROUP_KEYS;
#else
  // A workgroup takes the chunks that start inside a slice of the key axis.  Long slices amortise its
  // query registers and its start-up, but the chip wants a thousand workgroups or more: measured on
  // batches of 1 to 128 problems of 32K tokens, 2048-key slices win from about four thousand workgroups
  // on, 1024-key slices from about one thousand on, and below that the count matters more than the length.
  const long total_keys = static_cast<long>(n_tokens) * H_kv * P;
  long keys = 256;
  if (total_keys >= 2048L * 4096L) keys = 2048;
  else if (total_keys >= 1024L * 1024L) keys = 1024;
  else if (total_keys >= 512L * 1024L) keys = 512;
  // sentence-sized units: most blocks hold a boundary and cost twice a plain block, so the workgroups'
  // run times differ more and shorter ones balance better (3 % at 1240 units per 32K tokens)
  if (n_shots > 0 && n_tokens / n_shots < 64 && keys > 512) keys = 512;
  return static_cast<int>(keys);
#endif
}

bool score_uses_mfma(const PrefillDims& d) {
  return d.dtype == SHOTKV_BF16 && d.D == kD && d.R_rows <= 256 &&
         static_cast<long>(d.n_tokens) * kRowBytes < (1L << 32);
}

hipError_t launch_score_partials_mfma(const PrefillDims& d, const void* q_obs, const void* k,
                                      const PrefillWorkspace& w, hipStream_t s) {
  const dim3 grid(w.n_groups, d.H_kv, d.P);
  const float c = d.sm_scale * kLog2e;
  KernelTimer timer(d.timing, kKernelScore, s);
#define SHOTKV_LAUNCH_SCORE(NQB)                                                                      \
  hipLaunchKernelGGL(score_partials_mfma_kernel<NQB>, grid, dim3(PairShape<NQB>::kThreads), 0, s,     \
                     static_cast<const bf16_t*>(q_obs), static_cast<const bf16_t*>(k), d.n_tokens, d.H, \
                     d.H_kv, d.W, d.R_rows, c, w.group_first, w.chunk_start, w.chunk_len, w.max_c, w.partial,      \
                     w.group_stat)
  switch (d.R / 32) {
    case 1: SHOTKV_LAUNCH_SCORE(1); break;
    case 2: SHOTKV_LAUNCH_SCORE(2); break;
    case 4: SHOTKV_LAUNCH_SCORE(4); break;
    case 6: SHOTKV_LAUNCH_SCORE(6); break;
    case 8: SHOTKV_LAUNCH_SCORE(8); break;
    default: return hipErrorInvalidValue;
  }
#undef SHOTKV_LAUNCH_SCORE
  return hipGetLastError();
}

}  // namespace shotkv
