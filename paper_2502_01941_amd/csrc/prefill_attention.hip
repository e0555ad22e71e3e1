// Causal attention forward of the whole prompt that also emits the window-softmax partials of Eq. 3
// (Section 5.1; the appendix on limitations leaves kernel-level optimisation of the scoring step open).
//
// The prefill phase of a decoder computes softmax(Q K^T) V for every prompt position anyway.  The last W
// query rows of that pass are the observation-window rows whose weights Eq. 3 pools per shot, so this
// kernel writes, next to the attention output, the same per-(window row, chunk) statistic the
// stand-alone score kernel writes - log2 of the chunk's sum of exponentials - plus each window row's
// log2 denominator.  The per-shot reduction, selection and compaction kernels then run unchanged, and
// K is not read a second time for scoring.
//
// Shape: bf16, head_dim 128.  A workgroup of four waves owns 128 consecutive queries of one query head,
// each wave 32 of them, and walks the keys 0..last query in blocks of 32.
//   S^T = K_blk Q^T   v_mfma_f32_32x32x16_bf16, keys along the accumulator registers, queries along the
//                     lanes (the window queries' layout of the score kernel), so the online softmax is
//                     in-lane and its statistics are per-lane scalars.
//   O^T += V_blk^T P^T  the same instruction with d along the accumulator registers and queries still
//                     along the lanes: the weights a lane holds after the softmax ARE its B operand, and
//                     rescaling the output is a per-lane multiply.  The A operand needs V with keys
//                     contiguous; a small pre-pass packs V once into 32-key blocks [d][key] in exactly the
//                     key order the accumulator registers have.
//   precision         this product runs in fp16 (v_mfma_f32_32x32x16_f16): a weight keeps 11 significant bits
//                     instead of bf16's 8, which holds the output within 4e-4 of its row maximum with one
//                     instruction per step (a bf16 weight is off by up to 2^-9; bf16 hi + lo would cost a
//                     second instruction).  fp16's narrow range is dealt with by two exact power-of-two
//                     scalings: the softmax reference sits 15 below the running maximum, so weights lie
//                     in (0, 2^15] and anything above 2^-39 of the largest survives; and the pre-pass
//                     scales every KV-head plane of V so that its largest finite |v| lands in [2^14, 2^15).
//                     Sums of weights stay in fp32 and carry the same reference.
// K and packed-V blocks are streamed global -> LDS with direct-to-LDS loads into a ring of three stages
// shared by the four waves (one barrier per block); the LDS layouts are bank-conflict free for the
// 128-bit operand reads (K as in the score kernel; V^T rows of 64 bytes with a two-bit XOR of the
// 16-byte column).  The grid puts the query tile in its slowest dimension, longest tiles first, so that
// every head's long tiles are dispatched before anybody's short ones.
#include "common.hpp"

namespace shotkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) float floatx2;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((address_space(3))) const char lds_cchar;
typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;
typedef __attribute__((address_space(3))) const f16x8 lds_f16x8;

constexpr int kD = 128;
constexpr int kBlockKeys = 32;
constexpr int kRowBytes = kD * 2;
constexpr int kGroupBytes = 4 * kRowBytes + 64;       // K: four rows + pad = one direct-to-LDS instruction
constexpr int kKBytes = 8 * kGroupBytes;              // 8704
constexpr int kVtBytes = kD * kBlockKeys * 2;         // 8192: [128 d][32 keys] fp16
constexpr int kWeightShift = 15;                      // softmax reference = running maximum - 15 (log2 domain)
constexpr int kStageBytes = kKBytes + kVtBytes;
constexpr int kRing = 3;
constexpr int kTileQ = 128;
constexpr int kWavesQ = 4;
constexpr int kThreadsQ = kWavesQ * kWave;
constexpr int kLoadsPerWave = 4;                      // 2 K groups + 2 V^T slabs per wave per block

// ---- V packing -----------------------------------------------------------------------------------
// Largest finite |v| of every KV-head plane, as bf16 bits (their order is the order of the magnitudes),
// collected with atomic maxima into v_absmax, which the planning kernel has set to zero.
__global__ __launch_bounds__(256) void v_absmax_kernel(const bf16_t* __restrict__ v, int n_tokens,
                                                       uint32_t* __restrict__ v_absmax) {
  const size_t plane = blockIdx.y;
  const size_t n16 = static_cast<size_t>(n_tokens) * kD / 8;  // 16-byte pieces of the plane
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;       // a contiguous share per workgroup
  const size_t lo = blockIdx.x * per, hi = min(n16, lo + per);
  const u32x4* src = reinterpret_cast<const u32x4*>(v + plane * n_tokens * kD);
  uint32_t best = 0u;
  auto fold = [&](const u32x4& raw) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t a = raw[e] & 0x7fffu, b = (raw[e] >> 16) & 0x7fffu;
      if (a < 0x7f80u) best = max(best, a);  // infinities and NaNs do not set the scale
      if (b < 0x7f80u) best = max(best, b);
    }
  };
  size_t i = lo + threadIdx.x;
  for (; i + 3 * 256 < hi; i += 4 * 256) {  // four loads in flight per thread
    const u32x4 r0 = src[i], r1 = src[i + 256], r2 = src[i + 512], r3 = src[i + 768];
    fold(r0); fold(r1); fold(r2); fold(r3);
  }
  for (; i < hi; i += 256) fold(src[i]);
  // one atomic per workgroup: a few dozen per plane, not thousands on one address
  __shared__ uint32_t wave_best[256 / kWave];
  best = wave_max(best);
  if (threadIdx.x % kWave == 0) wave_best[threadIdx.x / kWave] = best;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < 256 / kWave; ++w) best = max(best, wave_best[w]);
    if (best != 0u) atomicMax(v_absmax + plane, best);
  }
}

// The power of two that brings a plane's largest |v| (bf16 bits) into [2^14, 2^15): multiply V by
// plane_scale(bits, false) when packing, the output by plane_scale(bits, true).  Both are exact.
__device__ __forceinline__ float plane_scale(uint32_t absmax_bits, bool inverse) {
  int e = static_cast<int>(absmax_bits >> 7);  // biased exponent of the largest magnitude
  e = min(max(e, 15), 254);                    // all-zero, denormal or absurdly small planes: a fixed scale
  return __uint_as_float(static_cast<uint32_t>(inverse ? e - 14 : 268 - e) << 23);
}

// vt[p][g][block][d][c][j] = scale * V[p][g][32*block + 8*(2*(c/2) + j/4) + 4*(c%2) + j%4][d] as fp16: column
// c = 2*s + half holds, in order, the eight keys whose weights a lane of half `half` feeds to matrix step s.
// Keys past n_tokens are zero.
__global__ __launch_bounds__(256) void pack_vt_kernel(const bf16_t* __restrict__ v, int n_tokens, int n_blocks,
                                                      const uint32_t* __restrict__ v_absmax,
                                                      uint16_t* __restrict__ vt) {
  const int blk = blockIdx.x;
  const size_t plane = blockIdx.y;  // p * H_kv + g
  __shared__ uint16_t tile[kBlockKeys][kD + 2];
  const float scale = plane_scale(v_absmax[plane], false);
  const bf16_t* src = v + plane * n_tokens * kD;
  for (int i = threadIdx.x; i < kBlockKeys * kD / 8; i += 256) {
    const int key = i / (kD / 8), d8 = i % (kD / 8);
    const int t = blk * kBlockKeys + key;
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (t < n_tokens) raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + static_cast<size_t>(t) * kD + d8 * 8));
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const floatx2 f = {__uint_as_float(raw[e] << 16) * scale, __uint_as_float(raw[e] & 0xffff0000u) * scale};
      const f16x2 hh = __builtin_convertvector(f, f16x2);
      const uint32_t bits = __builtin_bit_cast(uint32_t, hh);
      tile[key][d8 * 8 + 2 * e] = static_cast<uint16_t>(bits & 0xffffu);
      tile[key][d8 * 8 + 2 * e + 1] = static_cast<uint16_t>(bits >> 16);
    }
  }
  __syncthreads();
  uint16_t* dst = vt + (plane * n_blocks + blk) * (kD * kBlockKeys);
  for (int i = threadIdx.x; i < kD * 4; i += 256) {  // one 16-byte column per thread
    const int d = i / 4, c = i % 4, s = c >> 1, half = c & 1;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j0 = 2 * e, j1 = 2 * e + 1;
      const int k0 = 8 * (2 * s + j0 / 4) + 4 * half + j0 % 4;
      const int k1 = 8 * (2 * s + j1 / 4) + 4 * half + j1 % 4;
      w[e] = static_cast<uint32_t>(tile[k0][d]) | (static_cast<uint32_t>(tile[k1][d]) << 16);
    }
    *reinterpret_cast<u32x4*>(dst + d * kBlockKeys + c * 8) = u32x4{w[0], w[1], w[2], w[3]};
  }
}

// ---- streaming helpers ---------------------------------------------------------------------------
// K groups [g0, g0 + 2) of a block: group i fills rows 4i..4i+3; lane l writes LDS slot l of the group
// (row 4i + l/16, slot l%16) and therefore fetches column (l%16) ^ (l/16) of that row.  Rows past the
// last token re-read it (they are masked by causality).
__device__ __forceinline__ void issue_k(const char* __restrict__ k_plane, int key0, int n_tokens,
                                        uint32_t lds_addr, int g0, int lane) {
  const int hi = lane >> 4;
  const uint32_t col_bytes = static_cast<uint32_t>(((lane & 15) ^ hi) << 4);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int rr = min(key0 + 4 * (g0 + i) + hi, n_tokens - 1);
    const uint32_t off = static_cast<uint32_t>(rr) * kRowBytes + col_bytes;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr + (g0 + i) * kGroupBytes), "v"(off), "s"(k_plane)
                 : "memory", "m0");
  }
}
// V^T slabs [i0, i0 + 2) of a packed block: slab i fills rows (d) 16i..16i+15 of 64 bytes; lane l writes
// row 16i + l/4, slot l%4 and fetches column (l%4) ^ ((row/4)%4) of that row: sixteen consecutive rows,
// read 16 bytes each by sixteen lanes, then cover the 64 LDS banks exactly once.
__device__ __forceinline__ void issue_vt(const char* __restrict__ vt_block, uint32_t lds_addr, int i0, int lane) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int d = 16 * (i0 + i) + (lane >> 2);
    const int c = (lane & 3) ^ ((d >> 2) & 3);
    const uint32_t off = static_cast<uint32_t>(d * 64 + c * 16);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr + (i0 + i) * 1024), "v"(off), "s"(vt_block)
                 : "memory", "m0");
  }
}

__device__ __forceinline__ f16x8 to_f16x8(const float* x) {
  f16x8 r;
#pragma unroll
  for (int j = 0; j < 8; j += 2) {
    const floatx2 f = {x[j], x[j + 1]};
    const f16x2 hh = __builtin_convertvector(f, f16x2);  // round to nearest even
    r[j] = hh[0];
    r[j + 1] = hh[1];
  }
  return r;
}

__global__ __launch_bounds__(kThreadsQ, 2) void attention_scores_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const uint16_t* __restrict__ vt,
    const uint32_t* __restrict__ v_absmax, int n_tokens, int n_blocks_total, int H, int H_kv, int W, float c, float* __restrict__ o_out,
    const int32_t* __restrict__ n_chunks, const int32_t* __restrict__ chunk_start,
    const int32_t* __restrict__ chunk_len, int max_c, int R, float* __restrict__ partial,
    float* __restrict__ row_stat) {
  __shared__ __attribute__((aligned(64))) char lds[kRing][kStageBytes];
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int tile = gridDim.z - 1 - blockIdx.z;  // long tiles first, for all heads and problems
  const int h = blockIdx.x, p = blockIdx.y;
  const int G = H / H_kv, g = h / G;
  const int q0 = tile * kTileQ;
  const int half = lane >> 5;
  const int q_row = q0 + 32 * wave + (lane & 31);       // this lane's query
  const int q_eff = min(q_row, n_tokens - 1);           // rows past the prompt repeat the last one, unstored
  const int wave_min_q = q0 + 32 * wave;
  const int wave_max_q = min(wave_min_q + 31, n_tokens - 1);
  const int last_q = min(q0 + kTileQ, n_tokens) - 1;
  const int n_blocks = last_q / kBlockKeys + 1;         // keys 0..last_q
  // the window rows of this wave, if any, take part in Eq. 3
  const int win0 = n_tokens - W;
  const bool wave_emits = wave_min_q + 31 >= win0 && wave_min_q < n_tokens;
  const int win_j = q_row - win0;
  const bool lane_emits = win_j >= 0 && q_row < n_tokens && half == 0;

  const char* k_plane = reinterpret_cast<const char*>(k) + (static_cast<size_t>(p) * H_kv + g) * n_tokens * kRowBytes;
  const char* vt_plane =
      reinterpret_cast<const char*>(vt) + (static_cast<size_t>(p) * H_kv + g) * n_blocks_total * kVtBytes;
  // B operands of S^T: query q_eff, head-dim slice 16*ks + 8*half .. +8
  const bf16_t* q_ptr = q + ((static_cast<size_t>(p) * H + h) * n_tokens + q_eff) * kD + half * 8;
  bf16x8 bq[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks)
    bq[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(q_ptr + ks * 16));
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(bq[ks]));  // landed before the hand-tracked loads start

  lds_cchar* lds_base = (lds_cchar*)&lds[0][0];
  const uint32_t lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds_base));
  auto issue = [&](int b, int slot) {
    issue_k(k_plane, b * kBlockKeys, n_tokens, lds_addr + slot * kStageBytes, 2 * wave, lane);
    issue_vt(vt_plane + static_cast<size_t>(b) * kVtBytes, lds_addr + slot * kStageBytes + kKBytes, 2 * wave, lane);
  };

  float m_run = -INFINITY, l_run = 0.f;
  floatx16 ot[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) ot[t][v] = 0.f;

  // Eq. 3 bookkeeping (emitting waves only): the chunk whose sum is being collected
  const int nc = wave_emits ? n_chunks[p] : 0;
  const int32_t* cs = chunk_start + static_cast<size_t>(p) * max_c;
  const int32_t* cl = chunk_len + static_cast<size_t>(p) * max_c;
  int cur_c = 0, cur_s = 0, cur_e = 0;
  if (nc > 0) { cur_s = cs[0]; cur_e = cur_s + cl[0]; }
  float l_chunk = 0.f;
  const int h_local = h - g * G;
  float* part_row = partial + static_cast<size_t>(p) * max_c * H_kv * R + static_cast<size_t>(g) * R +
                    h_local * W + win_j;  // + chunk * H_kv * R
  auto finish_chunk = [&]() {
    const float tot = sum_across_halves(l_chunk);
    if (lane_emits)
      part_row[static_cast<size_t>(cur_c) * H_kv * R] = tot > 0.f ? m_run + __builtin_amdgcn_logf(tot) : -INFINITY;
    l_chunk = 0.f;
    ++cur_c;
    if (cur_c < nc) { cur_s = cs[cur_c]; cur_e = cur_s + cl[cur_c]; }
  };

  issue(0, 0);
  if (n_blocks > 1) issue(1, 1);
  for (int b = 0; b < n_blocks; ++b) {
    // this wave's loads of block b have landed once only those of block b+1 can be outstanding
    if (b + 1 < n_blocks) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerWave) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // ... and after the barrier so have the other waves'; everybody is also done with block b-1
    asm volatile("s_barrier" ::: "memory");
    const int slot = b % kRing;
    if (b + 2 < n_blocks) issue(b + 2, (b + 2) % kRing);
    const int key0 = b * kBlockKeys;
    const bool has_work = key0 <= wave_max_q;
    float pw[16];
    if (has_work) {
      lds_cchar* blk = lds_base + slot * kStageBytes;
      // ---- S^T: keys along registers (row 8*(v/4) + 4*half + v%4), queries along lanes -------------
      const int row = lane & 31;
      const int base_even = row * kRowBytes + (row >> 2) * 64 + ((half ^ (row & 3)) << 4);
      lds_cchar* even = blk + base_even;
      lds_cchar* odd = blk + (base_even ^ 32);
      floatx16 acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 a = *reinterpret_cast<lds_bf16x8*>(((ks & 1) ? odd : even) + 64 * (ks >> 1));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[ks], acc, 0, 0, 0);
      }
      // ---- causal mask, online softmax ---------------------------------------------------------
      if (key0 + kBlockKeys - 1 > wave_min_q) {
        const int limit = q_eff - key0 + 1 - 4 * half;  // rows below this are visible
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (8 * (v >> 2) + (v & 3) >= limit) acc[v] = -INFINITY;
      }
      float bm = fmaxf(acc[0], acc[1]);
#pragma unroll
      for (int v = 2; v < 16; v += 2) bm = fmaxf(fmaxf(bm, acc[v]), acc[v + 1]);
      bm = max_across_halves(bm);
      // the reference sits kWeightShift below the largest logit: weights up to 2^15, well inside fp16, and
      // small ones far from its underflow.  Finite from the first block on: key 0 is always visible
      const float m_new = fmaxf(m_run, fmaf(bm, c, -static_cast<float>(kWeightShift)));
      if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 from -inf
        l_run *= alpha;
        l_chunk *= alpha;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int v = 0; v < 16; ++v) ot[t][v] *= alpha;
        m_run = m_new;
      }
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        pw[v] = __builtin_amdgcn_exp2f(fmaf(acc[v], c, -m_run));
        pw[v + 1] = __builtin_amdgcn_exp2f(fmaf(acc[v + 1], c, -m_run));
        s0 += pw[v];
        s1 += pw[v + 1];
      }
      l_run += s0 + s1;
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) pw[v] = 0.f;
    }
    // ---- Eq. 3: this block's weights credited to the chunks it overlaps --------------------------
    if (wave_emits) {
      while (cur_c < nc && cur_s < key0 + kBlockKeys) {
        const int lo = max(cur_s, key0) - key0 - 4 * half, hi = min(cur_e, key0 + kBlockKeys) - key0 - 4 * half;
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = 8 * (v >> 2) + (v & 3);
          sum += (r >= lo && r < hi) ? pw[v] : 0.f;
        }
        l_chunk += sum;
        if (cur_e <= key0 + kBlockKeys) finish_chunk();
        else break;
      }
    }
    // ---- O^T += V_blk^T P^T in fp16 -------------------------------------------------------------------
    if (has_work) {
      lds_cchar* vblk = lds_base + slot * kStageBytes + kKBytes;
      const f16x8 p16[2] = {to_f16x8(pw), to_f16x8(pw + 8)};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int d = 32 * t + (lane & 31);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          const int col = (2 * s + half) ^ ((d >> 2) & 3);
          const f16x8 a = *reinterpret_cast<lds_f16x8*>(vblk + d * 64 + col * 16);
          ot[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, p16[s], ot[t], 0, 0, 0);
        }
      }
    }
  }

  // ---- results -------------------------------------------------------------------------------------
  const float l_tot = sum_across_halves(l_run);
  if (wave_emits) {
    // chunks that reach past this tile's keys hold what their visible part gave; later ones nothing
    while (cur_c < nc) finish_chunk();
    if (lane_emits)
      row_stat[(static_cast<size_t>(p) * H_kv + g) * R + h_local * W + win_j] = m_run + __builtin_amdgcn_logf(l_tot);
  }
  if (q_row < n_tokens) {
    const float inv = 1.f / l_tot;
    // undoes V's scale; applied after the normalisation, because up / l_tot can fall below the normal range
    const float up = plane_scale(v_absmax[static_cast<size_t>(p) * H_kv + g], true);
    float* dst = o_out + ((static_cast<size_t>(p) * H + h) * n_tokens + q_row) * kD + 4 * half;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int a = 0; a < 4; ++a)
        *reinterpret_cast<float4*>(dst + 32 * t + 8 * a) =
            make_float4(ot[t][4 * a] * inv * up, ot[t][4 * a + 1] * inv * up, ot[t][4 * a + 2] * inv * up,
                        ot[t][4 * a + 3] * inv * up);
  }
}

}  // namespace

bool attention_supported(const PrefillDims& d) {
  return d.dtype == SHOTKV_BF16 && d.D == kD && d.W <= kTileQ &&
         static_cast<long>(d.n_tokens) * kRowBytes < (1L << 32);
}

int attention_key_blocks(int n_tokens) { return ceil_div(n_tokens, kBlockKeys); }

hipError_t launch_pack_vt(const PrefillDims& d, const void* v, const PrefillWorkspace& w, hipStream_t s) {
  const int nb = attention_key_blocks(d.n_tokens);
  KernelTimer timer(d.timing, kKernelPackVt, s);
  // enough workgroups to fill the chip a few times over, each with at least 128 rows of a plane
  const int planes = d.P * d.H_kv;
  const int shares = max(1, min(ceil_div(d.n_tokens, 128), ceil_div(1024, planes)));
  hipLaunchKernelGGL(v_absmax_kernel, dim3(shares, planes), dim3(256), 0, s, static_cast<const bf16_t*>(v),
                     d.n_tokens, w.v_absmax);
  hipLaunchKernelGGL(pack_vt_kernel, dim3(nb, d.P * d.H_kv), dim3(256), 0, s, static_cast<const bf16_t*>(v),
                     d.n_tokens, nb, w.v_absmax, static_cast<uint16_t*>(w.vt));
  return hipGetLastError();
}

hipError_t launch_attention_scores(const PrefillDims& d, const void* q, const void* k, const void* vt,
                                   float* attn_out, const PrefillWorkspace& w, hipStream_t s) {
  const int nb = attention_key_blocks(d.n_tokens);
  const dim3 grid(d.H, d.P, ceil_div(d.n_tokens, kTileQ));
  KernelTimer timer(d.timing, kKernelAttention, s);
  hipLaunchKernelGGL(attention_scores_kernel, grid, dim3(kThreadsQ), 0, s, static_cast<const bf16_t*>(q),
                     static_cast<const bf16_t*>(k), static_cast<const uint16_t*>(vt), w.v_absmax, d.n_tokens, nb, d.H,
                     d.H_kv,
                     d.W, d.sm_scale * kLog2e, attn_out, w.n_chunks, w.chunk_start, w.chunk_len, w.max_c, d.R,
                     w.partial, w.row_stat);
  return hipGetLastError();
}

}  // namespace shotkv
