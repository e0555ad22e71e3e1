// Window-attention softmax partials on the gfx950 matrix cores (Section 5.1, Eq. 3: alpha_{t,h}).
//
// Shape: bf16, head_dim 128, R = G*W in {32, 64, 128} query rows per KV head.
//
// Work unit = (wave, chunk).  A wave keeps all R x 128 window queries of its KV head in registers as
// MFMA B operands and walks its chunks in blocks of 32 keys: S^T[32 keys x R queries] = K_blk * Q^T
// with v_mfma_f32_32x32x16_bf16.  Keys run along the accumulator registers and queries along the
// lanes, so the row-softmax statistics (max and sum over keys) are in-lane reductions; only the two
// lane halves are merged, once per chunk.  K blocks are streamed global -> LDS with 16-byte
// direct-to-LDS loads (whole 256-byte rows, fully coalesced), double buffered per wave, and read back
// in MFMA A-operand layout.  Waves never synchronise with each other.
//
// The direct-to-LDS loads are written as inline assembly and their completion is tracked by hand with
// s_waitcnt vmcnt: when they are visible to the compiler it makes every LDS read wait for all loads
// in flight, including the prefetch of the next block, which serialises load and compute.  Unknown
// vector-memory operations can only make the compiler's own waits stricter, never too weak, because
// the counter orders completions.
//
// LDS layout of a block: key row r starts at r*256 + (r/4)*64 and its 16-byte column c sits in slot
// c ^ (r%4).  The 64-byte pad per four rows plus the two-bit XOR spread the 16 lanes of a 128-bit LDS
// read over all banks, while the address of MFMA step ks stays (lane base for ks parity) + 64*(ks/2),
// i.e. an immediate offset - no per-step address registers.
#include "common.hpp"

namespace shotkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) const char lds_cchar;  // keeps LDS reads as ds_read, not flat
typedef __attribute__((address_space(1))) const void glb_void;

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kD = 128;
constexpr int kBlockKeys = 32;
constexpr int kRowBytes = kD * 2;                    // 256
constexpr int kGroupBytes = 4 * kRowBytes + 64;      // four rows + pad = one direct-to-LDS instruction
constexpr int kLoadsPerBlock = kBlockKeys / 4;       // 8
constexpr int kBufBytes = kLoadsPerBlock * kGroupBytes;  // 8704 bytes per wave per buffer

// Issue the 8 direct-to-LDS loads of one 32-key block.  Instruction i fills rows 4i..4i+3: lane l
// writes LDS slot l of the group, which is row 4i + l/16, slot l%16, and therefore fetches column
// (l%16) ^ (l/16) of that row.  Rows past the end of the chunk re-read its last key (they are masked
// later), so every address stays inside the chunk.
__device__ __forceinline__ void issue_block(const char* __restrict__ k_plane, int key0, int rem,
                                            uint32_t lds_addr, int lane) {
  const int last = rem - 1;  // rem >= 1
  const int hi = lane >> 4;
  const uint32_t col_bytes = static_cast<uint32_t>(((lane & 15) ^ hi) << 4);
#pragma unroll
  for (int i = 0; i < kLoadsPerBlock; ++i) {
    const int rr = min(4 * i + hi, last);
    const uint32_t off = static_cast<uint32_t>(key0 + rr) * kRowBytes + col_bytes;
    // M0 = LDS address of the group (wave-uniform); lane l lands at M0 + 16*l
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr + i * kGroupBytes), "v"(off), "s"(k_plane)
                 : "memory", "m0");
  }
}

// Fold the 16 logits a lane holds for one query (key rows 8*(v/4) + 4*half + v%4 of the block) into
// that query's running (max, sum) in the log2 domain.
template <bool MASKED>
__device__ __forceinline__ void softmax_fold(floatx16 acc, float c, int half, int rem, int key0,
                                             int last_visible, float& m_run, float& l_run) {
  if (MASKED) {
    // row 8*(v/4) + v%4 + 4*half is masked when it is past the chunk or past the query's position:
    // one per-lane limit, compared against compile-time row constants
    const int limit = min(rem, last_visible - key0 + 1) - 4 * half;
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (8 * (v >> 2) + (v & 3) >= limit) acc[v] = -INFINITY;
  }
  float bm = fmaxf(acc[0], acc[1]);
#pragma unroll
  for (int v = 2; v < 16; v += 2) bm = fmaxf(fmaxf(bm, acc[v]), acc[v + 1]);
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
  m_run = m_new;
}

// One 32-key block against all NQB query blocks, two query blocks at a time so that only two
// accumulator sets are live (the A operands are read from LDS once per pair).
template <int NQB, bool MASKED>
__device__ __forceinline__ void compute_block(lds_cchar* lds_buf, const bf16x8 (&bq)[NQB][8], int lane,
                                              int key0, int rem, int causal_base, int W, float c,
                                              float (&m_run)[NQB], float (&l_run)[NQB]) {
  constexpr int QG = NQB >= 2 ? 2 : 1;
  const int row = lane & 31, half = lane >> 5;
  const int base_even = row * kRowBytes + (row >> 2) * 64 + ((half ^ (row & 3)) << 4);
  lds_cchar* even = lds_buf + base_even;
  lds_cchar* odd = lds_buf + (base_even ^ 32);
#pragma unroll
  for (int grp = 0; grp < NQB / QG; ++grp) {
    floatx16 acc[QG];
#pragma unroll
    for (int q = 0; q < QG; ++q)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;
      const bf16x8 a = *reinterpret_cast<lds_bf16x8*>(((ks & 1) ? odd : even) + 64 * (ks >> 1));
#pragma unroll
      for (int q = 0; q < QG; ++q)
        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[grp * QG + q][ks], acc[q], 0, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < QG; ++q) {
      const int qb = grp * QG + q;
      const int last_visible = causal_base + (qb * 32 + row) % W;
      softmax_fold<MASKED>(acc[q], c, half, rem, key0, last_visible, m_run[qb], l_run[qb]);
    }
  }
}

template <int NQB>
__global__ __launch_bounds__(kThreads, 2) void score_partials_mfma_kernel(
    const bf16_t* __restrict__ q_obs, const bf16_t* __restrict__ k, int n_tokens, int H, int H_kv, int W,
    float c, const int32_t* __restrict__ n_chunks, const int32_t* __restrict__ chunk_start,
    const int32_t* __restrict__ chunk_len, int max_c, int chunks_per_wave,
    float2* __restrict__ partial) {
  constexpr int R = NQB * 32;
  __shared__ __attribute__((aligned(64))) char lds[kWavesPerBlock][2][kBufBytes];

  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int g = blockIdx.y, p = blockIdx.z;
  const int nc = n_chunks[p];
  const int c_begin = (blockIdx.x * kWavesPerBlock + wave) * chunks_per_wave;
  if (c_begin >= nc) return;  // whole wave leaves; there are no workgroup barriers in this kernel
  const int c_end = min(c_begin + chunks_per_wave, nc);

  const int32_t* cs = chunk_start + static_cast<size_t>(p) * max_c;
  const int32_t* cl = chunk_len + static_cast<size_t>(p) * max_c;
  const char* k_plane =
      reinterpret_cast<const char*>(k) + (static_cast<size_t>(p) * H_kv + g) * n_tokens * kRowBytes;
  const int G = H / H_kv;
  const bf16_t* q_rows = q_obs + (static_cast<size_t>(p) * H + static_cast<size_t>(g) * G) * W * kD;
  float2* out = partial + (static_cast<size_t>(p) * H_kv + g) * max_c * R;

  // B operands: query row qb*32 + lane%32, head-dim slice 16*ks + 8*(lane/32) .. +8
  bf16x8 bq[NQB][8];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      bq[qb][ks] = *reinterpret_cast<const bf16x8*>(q_rows + (qb * 32 + (lane & 31)) * kD + ks * 16 +
                                                    (lane >> 5) * 8);

  // the query loads must have landed before the streaming loop starts: inside the loop the only
  // vector-memory operations are the block loads, whose completion is tracked by hand
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(bq[qb][ks]));

  lds_cchar* lds_wave = (lds_cchar*)&lds[wave][0][0];
  const uint32_t lds_wave_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds_wave));
  const int causal_base = n_tokens - W;

  float m_run[NQB], l_run[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

  // A finished chunk's statistics are stored one block later, right after the wait for that block's
  // data: a store issued just before a wait would have to complete within it (the wait also covers
  // older stores), this way it has a whole block of compute to do so.  Row r of the partial array is
  // query lane*NQB + qb; one instruction stores everything (lanes 32..63 carry query blocks 2 and 3).
  float2 pend[NQB];
  int pend_c = -1;
  auto flush = [&]() {
    float2* dst = out + static_cast<size_t>(pend_c) * R + (lane & 31) * NQB;
    if (NQB == 4) {
      const bool upper = lane >= 32;
      const float2 x = upper ? pend[NQB - 2] : pend[0], y = upper ? pend[NQB - 1] : pend[NQB > 1 ? 1 : 0];
      *reinterpret_cast<float4*>(dst + (upper ? 2 : 0)) = make_float4(x.x, x.y, y.x, y.y);
    } else if (NQB == 2) {
      if (lane < 32) *reinterpret_cast<float4*>(dst) = make_float4(pend[0].x, pend[0].y, pend[NQB - 1].x, pend[NQB - 1].y);
    } else {
      if (lane < 32) dst[0] = pend[0];
    }
    pend_c = -1;
  };

  // stream of 32-key blocks over the wave's chunks; `cur` is in flight to / resident in buffer
  // cur_buf, its successor goes to the other one.  The table entry of the chunk after the current one is
  // fetched a whole chunk ahead, so stepping into a new chunk never waits on memory.
  int cur_c = c_begin;
  int cur_key0 = cs[cur_c];
  int cur_rem = cl[cur_c];
  int ahead_key0 = 0, ahead_len = 0;
  if (cur_c + 1 < c_end) { ahead_key0 = cs[cur_c + 1]; ahead_len = cl[cur_c + 1]; }
  issue_block(k_plane, cur_key0, cur_rem, lds_wave_addr, lane);
  int cur_buf = 0;

  while (true) {
    // successor block
    int nxt_c = cur_c, nxt_key0 = cur_key0 + kBlockKeys, nxt_rem = cur_rem - kBlockKeys;
    bool has_next = true;
    if (nxt_rem <= 0) {
      nxt_c = cur_c + 1;
      has_next = nxt_c < c_end;
      nxt_key0 = ahead_key0;
      nxt_rem = ahead_len;
      if (nxt_c + 1 < c_end) { ahead_key0 = cs[nxt_c + 1]; ahead_len = cl[nxt_c + 1]; }
    }
    // the loads of the next block go out first, then this wave waits only for the older ones
    if (has_next) {
      issue_block(k_plane, nxt_key0, nxt_rem, lds_wave_addr + (cur_buf ^ 1) * kBufBytes, lane);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerBlock) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    // keys past the end of the chunk and keys a window query may not see yet are masked; both only
    // happen in a chunk's last block or in the last W keys, so the common block takes the plain path
    if (pend_c >= 0) flush();
    const bool masked = cur_rem < kBlockKeys || cur_key0 + kBlockKeys - 1 > causal_base;
    if (masked)
      compute_block<NQB, true>(lds_wave + cur_buf * kBufBytes, bq, lane, cur_key0, cur_rem, causal_base, W, c, m_run, l_run);
    else
      compute_block<NQB, false>(lds_wave + cur_buf * kBufBytes, bq, lane, cur_key0, cur_rem, causal_base, W, c, m_run, l_run);

    if (cur_rem <= kBlockKeys) {  // last block of its chunk: merge the lane halves
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const float mo = __shfl_xor(m_run[qb], 32, kWave);
        const float lo = __shfl_xor(l_run[qb], 32, kWave);
        const float mn = fmaxf(m_run[qb], mo);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        // a + b is the same in both halves, so lanes l and l+32 now hold identical results
        pend[qb] = make_float2(mn, l_run[qb] * __builtin_amdgcn_exp2f(m_run[qb] - ms) +
                                       lo * __builtin_amdgcn_exp2f(mo - ms));
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
      }
      pend_c = cur_c;
    }
    if (!has_next) break;
    cur_c = nxt_c; cur_key0 = nxt_key0; cur_rem = nxt_rem;
    cur_buf ^= 1;
  }
  if (pend_c >= 0) flush();
}

int pick_chunks_per_wave(const PrefillDims& d, int max_c) {
#ifdef SHOTKV_CHUNKS_PER_WAVE
  return SHOTKV_CHUNKS_PER_WAVE;
#else
  // aim for a few thousand workgroups so that 256 CUs x 2 resident workgroups stay busy, while a wave
  // amortises its query registers over as many chunks as that allows
  const long total_chunks = static_cast<long>(max_c) * d.H_kv * d.P;
  long cpw = total_chunks / (kWavesPerBlock * 4096L);
  if (cpw < 1) cpw = 1;
  if (cpw > 8) cpw = 8;
  return static_cast<int>(cpw);
#endif
}

}  // namespace

bool score_uses_mfma(const PrefillDims& d) {
  return d.dtype == SHOTKV_BF16 && d.D == kD && (d.R == 32 || d.R == 64 || d.R == 128) &&
         static_cast<long>(d.n_tokens) * kRowBytes < (1L << 32);
}

hipError_t launch_score_partials_mfma(const PrefillDims& d, const void* q_obs, const void* k,
                                      const PrefillWorkspace& w, hipStream_t s) {
  const int cpw = pick_chunks_per_wave(d, w.max_c);
  const dim3 grid(ceil_div(w.max_c, kWavesPerBlock * cpw), d.H_kv, d.P), block(kThreads);
  const float c = d.sm_scale * kLog2e;
  KernelTimer timer(kKernelScore, s);
#define SHOTKV_LAUNCH_SCORE(NQB)                                                                      \
  hipLaunchKernelGGL(score_partials_mfma_kernel<NQB>, grid, block, 0, s,                              \
                     static_cast<const bf16_t*>(q_obs), static_cast<const bf16_t*>(k), d.n_tokens, d.H, \
                     d.H_kv, d.W, c, w.n_chunks, w.chunk_start, w.chunk_len, w.max_c, cpw, w.partial)
  switch (d.R / 32) {
    case 1: SHOTKV_LAUNCH_SCORE(1); break;
    case 2: SHOTKV_LAUNCH_SCORE(2); break;
    case 4: SHOTKV_LAUNCH_SCORE(4); break;
    default: return hipErrorInvalidValue;
  }
#undef SHOTKV_LAUNCH_SCORE
  return hipGetLastError();
}

}  // namespace shotkv
