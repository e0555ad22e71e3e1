// Split-KV decode attention for bf16, head_dim 128, with the logits on the matrix cores
// (Section 5.1, Eq. 7 and 9: attention of the current query over prefill rows and decode slots).
//
// A workgroup owns one token range of one (sequence, KV head) and makes two passes over it:
//   1. K pass: the logits of four tokens per v_mfma_f32_16x16x32_bf16, with the head dimension cut into
//      four pieces that sit in different operand rows/columns, so that the A operands are whole
//      256-byte K rows fetched straight from global memory with coalesced 16-byte loads (see the
//      kernel).  The scaled logits go to LDS.
//   between: validity mask (free slots), per-head maximum, weights 2^(z - max) and their sums, all on
//      the logits in LDS; decode-slot logits are also written out for the retention score (Eq. 7).
//   2. V pass: 16 lanes stream one V row each (16 bytes per lane) and accumulate weight * V with the
//      weights read from LDS.  No rescaling is needed because the maximum is already known.
// Compared with a one-pass online softmax this moves the dot products off the vector ALU, removes the
// cross-lane reductions per token and the per-token rescale of the output accumulators.
#include "common.hpp"

namespace shotkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float floatx4;

// 16 bytes of a K or V row with the non-temporal hint.  A step reads every live row once; once the caches
// of a batch outgrow L2 and the memory-side cache, rows that do not settle there stream faster (4-7 %
// at 16 and more sequences of 5K tokens, no change for one to four sequences).
__device__ __forceinline__ u32x4 stream_load(const u32x4* p) { return __builtin_nontemporal_load(p); }

// value of the lane N places away inside each row of 16 lanes (rotation, so every lane gets one)
template <int N>
__device__ __forceinline__ float row_rotate(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x120 | N, 0xf, 0xf, false));
}

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kD = 128;
constexpr int kMaxRange = kDecodeMaxRange;  // tokens per workgroup the LDS logit buffer can hold
#ifndef SHOTKV_DEC_V_UNROLL
#define SHOTKV_DEC_V_UNROLL 4
#endif
constexpr int kVUnroll = SHOTKV_DEC_V_UNROLL;  // V rows a lane group has in flight

// lowest free slot of a sequence, -1 if none; every thread of the block gets the answer
__device__ int lowest_free_slot(const int32_t* __restrict__ slot_pos, int n_slots, int* s_red) {
  int best = INT32_MAX;
  for (int i = threadIdx.x; i < n_slots; i += blockDim.x)
    if (slot_pos[i] < 0) { best = i; break; }
  for (int o = kWave / 2; o > 0; o >>= 1) best = min(best, __shfl_xor(best, o, kWave));
  if (threadIdx.x % kWave == 0) s_red[threadIdx.x / kWave] = best;
  __syncthreads();
  int r = INT32_MAX;
  for (int w = 0; w < kWaves; ++w) r = min(r, s_red[w]);
  __syncthreads();
  return r == INT32_MAX ? -1 : r;
}

template <int G>
__global__ __launch_bounds__(kThreads) void decode_partial_mfma_kernel(
    const bf16_t* __restrict__ k_prefill, const bf16_t* __restrict__ v_prefill,
    const int32_t* __restrict__ prefill_count, bf16_t* __restrict__ k_dec, bf16_t* __restrict__ v_dec,
    const int32_t* __restrict__ slot_pos, int cap, int n_slots, int H, int H_kv, int n_group,
    int n_splits, int split_tokens, float scale_log2e, const bf16_t* __restrict__ q_new,
    const bf16_t* __restrict__ k_new, const bf16_t* __restrict__ v_new, float2* __restrict__ part_ml,
    float* __restrict__ part_o, float* __restrict__ z_dec, int32_t* __restrict__ new_slot_out) {
  const int split = blockIdx.x, g = blockIdx.y, s = blockIdx.z;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;

  __shared__ __attribute__((aligned(16))) float zbuf[kMaxRange][G];  // logits, then weights
  __shared__ float s_M[G];
  __shared__ float s_L[G];
  __shared__ float s_o[kWaves][G][kD];
  __shared__ int s_red[kWaves];
  __shared__ int s_sp[kMaxRange];  // slot map of the decode slots inside this workgroup's range

  // G is the group size rounded up to a power of two; heads past the real n_group are zero queries
  // whose results are never written
  const size_t head0 = static_cast<size_t>(s) * H + static_cast<size_t>(g) * n_group;
  // Query operands first: these loads and the one of the row count below are in flight together.
  const int i16 = lane & 15, ksl = lane >> 4;  // A row / B column, and k-slice (8 elements) of the lane
  const int tau = i16 >> 2, piece = i16 & 3;   // as A row; as B/C column: piece i16 >> 2, head i16 & 3
  const int elem_off = 32 * piece + 8 * ksl;
  constexpr int kHeadSets = (G + 3) / 4;
  bf16x8 bq[kHeadSets];
#pragma unroll
  for (int m = 0; m < kHeadSets; ++m) {
    u32x4 raw = {0u, 0u, 0u, 0u};
    const int hq = (i16 & 3) + 4 * m;
    if (hq < n_group) raw = *reinterpret_cast<const u32x4*>(q_new + (head0 + hq) * kD + 32 * (i16 >> 2) + 8 * ksl);
    bq[m] = __builtin_bit_cast(bf16x8, raw);
  }
  const int32_t* sp = slot_pos + static_cast<size_t>(s) * n_slots;
  // Token axis of a sequence: t < cap is row t of the prefill cache (live while t < prefill_count), t >= cap
  // is decode slot t - cap.  Nothing about the ranges or the addresses depends on prefill_count, so the
  // first rows are requested while that count is still on its way; it only masks.
  const int pc = min(prefill_count[s], cap);
  const int t_begin = split * split_tokens;
  const int t_end = min(t_begin + split_tokens, cap + n_slots);
  const int T = max(t_end - t_begin, 0);
  // Only a range that reaches into the decode slots needs the slot map: its part of it goes to LDS
  // (so that the row fetches below do not wait on a second, dependent load), and the slot that takes
  // the new token is found in the same round trip.
  const int d_lo = max(t_begin - cap, 0);  // decode slots [d_lo, d_lo + n_range_slots) lie in the range
  const int n_range_slots = max(t_end - cap, 0) - d_lo;
  if (t_end > cap)
    for (int i = tid; i < n_range_slots; i += kThreads) s_sp[i] = sp[d_lo + i];
  const int new_slot = (t_end > cap) ? lowest_free_slot(sp, n_slots, s_red) : n_slots;  // has barriers
  if (t_end == cap + n_slots && g == 0 && tid == 0) new_slot_out[s] = new_slot;

  const size_t plane_p = (static_cast<size_t>(s) * H_kv + g) * cap;
  const size_t plane_d = (static_cast<size_t>(s) * H_kv + g) * n_slots;
  const size_t new_off = (static_cast<size_t>(s) * H_kv + g) * kD;

  // token t of the sequence: live prefill row, occupied slot, the slot taking the new token, or nothing
  auto token_valid = [&](int t) {
    if (t < cap) return t < pc;
    const int slot = t - cap;
    return slot < n_slots && (slot == new_slot || s_sp[slot - d_lo] >= 0);
  };

  if (new_slot >= 0 && T > 0) {
    // ---- pass 1: logits ------------------------------------------------------------------------
    // One v_mfma_f32_16x16x32_bf16 scores four tokens.  Row i = 4*tau + piece of its A operand holds
    // the 32-element piece `piece` of token `tau`, column j = 4*piece + h of its B operand the same
    // piece of query head h, so C[4*tau + piece][4*piece + h] is that piece's share of the logit and
    // the four shares sit in lanes 4 apart.  Laid out like this the 16 lanes that hold one token
    // read its whole 256-byte row with one 16-byte load each: every load instruction fetches four
    // complete rows, already in operand order.
    for (int blk = wave; blk * 32 < T; blk += kWaves) {
      // a block of dead prefill rows only (count below cap) is skipped: its logits are masked between the
      // passes whatever zbuf holds.  A wave's first block is fetched regardless, before the count is known.
      if (blk != wave && t_begin + blk * 32 >= pc && t_begin + blk * 32 + 31 < cap) continue;
      // so is a block of decode slots none of which holds a token (a pool that is still filling up)
      if (t_begin + blk * 32 >= cap) {
        const int tt = blk * 32 + (lane & 31);
        const bool holds = tt < T && token_valid(t_begin + tt);
        if (__builtin_amdgcn_ballot_w64(holds) == 0) continue;
      }
      u32x4 raw[8];
      const int tt0 = blk * 32 + tau;
      if (t_begin + blk * 32 + 31 < cap && blk * 32 + 31 < T) {  // the whole block lies in the prefill cache
        const bf16_t* kr = k_prefill + (plane_p + t_begin + tt0) * kD + elem_off;
#pragma unroll
        for (int gi = 0; gi < 8; ++gi) raw[gi] = stream_load(reinterpret_cast<const u32x4*>(kr + gi * 4 * kD));
      } else {
#pragma unroll
        for (int gi = 0; gi < 8; ++gi) {
          const int tt = tt0 + 4 * gi;
          const int t = t_begin + tt;
          // rows past the range and free slots read the new token's key instead (always valid
          // memory); their logits are masked between the passes
          const bf16_t* kr = k_new + new_off;
          bool is_new = false;
          if (tt < T) {
            if (t < cap) {
              kr = k_prefill + (plane_p + t) * kD;
            } else {
              const int slot = t - cap;
              is_new = slot == new_slot;
              if (!is_new && s_sp[slot - d_lo] >= 0) kr = k_dec + (plane_d + slot) * kD;
            }
          }
          raw[gi] = stream_load(reinterpret_cast<const u32x4*>(kr + elem_off));
          // append: only this workgroup reads the slot this step
          if (is_new) *reinterpret_cast<u32x4*>(k_dec + (plane_d + new_slot) * kD + elem_off) = raw[gi];
        }
      }
#pragma unroll
      for (int gi = 0; gi < 8; ++gi) {
#pragma unroll
        for (int m = 0; m < kHeadSets; ++m) {
          floatx4 acc = {0.f, 0.f, 0.f, 0.f};
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, raw[gi]), bq[m], acc, 0, 0, 0);
          // lane (column 4*piece + h, row group ksl) holds rows 4*ksl + v: token ksl of the group, piece v
          const int pb = i16 >> 2;
          float z = pb == 0 ? acc[0] : pb == 1 ? acc[1] : pb == 2 ? acc[2] : acc[3];
          z += row_rotate<4>(z);
          z += row_rotate<8>(z);  // now every lane of the column set {h, h+4, h+8, h+12} has the logit
          const int hq = i16 + 4 * m;
          const int ttc = blk * 32 + 4 * gi + ksl;
          if (i16 < 4 && hq < G && ttc < T) zbuf[ttc][hq] = z * scale_log2e;
        }
      }
    }
    __syncthreads();

    // ---- between the passes: mask, maximum, weights and their sum; one wave per query head, so
    //      only wave-level reductions and no workgroup barrier in between ----------------------------
    for (int h = wave; h < n_group; h += kWaves) {
      float mx = -INFINITY;
      for (int tt = lane; tt < T; tt += kWave) {
        float z = zbuf[tt][h];
        if (!token_valid(t_begin + tt)) { z = -INFINITY; zbuf[tt][h] = z; }
        mx = fmaxf(mx, z);
      }
      mx = wave_max(mx);
      float sum = 0.f;
      for (int tt = lane; tt < T; tt += kWave) {  // every lane re-reads what it wrote itself
        const float z = zbuf[tt][h];
        const int t = t_begin + tt;
        if (t >= cap && z != -INFINITY) z_dec[(head0 + h) * n_slots + (t - cap)] = z;
        const float p = (z == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(z - mx);
        zbuf[tt][h] = p;
        sum += p;
      }
      sum = wave_sum(sum);
      if (lane == 0) { s_M[h] = mx; s_L[h] = sum; }
    }
    __syncthreads();
  } else {
    if (tid < G) { s_M[tid] = -INFINITY; s_L[tid] = 0.f; }
    __syncthreads();
  }

  // ---- pass 2: weighted values -------------------------------------------------------------------
  constexpr int kGroups = kThreads / 16;  // 16 lanes per V row
  const int grp = tid >> 4, lir = tid & 15;
  float o[G][8];
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
#pragma unroll
    for (int e = 0; e < 8; ++e) o[hh][e] = 0.f;
  if (new_slot >= 0) {
    // kVUnroll rows per lane group are requested before any of them is used.  A token without weight
    // (masked, or underflowed to exactly zero) reads the new token's value row instead - always valid
    // memory - and contributes zero times that.
    for (int tt0 = grp; tt0 < T; tt0 += kGroups * kVUnroll) {
      float p[kVUnroll][G];
      u32x4 raw[kVUnroll];
      bool any[kVUnroll], is_new[kVUnroll];
      bool work = false;
#pragma unroll
      for (int u = 0; u < kVUnroll; ++u) {
        const int tt = tt0 + u * kGroups;
        const bool inside = tt < T;
        const int ttc = inside ? tt : 0;
        any[u] = false;
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
          p[u][hh] = (inside && hh < n_group) ? zbuf[ttc][hh] : 0.f;  // padding heads carry no weight
          any[u] = any[u] || p[u][hh] != 0.f;
        }
        // the slot taking the new token: its value row is appended whatever weight the token got
        // (a weight that underflows to zero must not leave a stale row behind for later steps)
        is_new[u] = inside && t_begin + ttc >= cap && (t_begin + ttc - cap) == new_slot;
        work = work || any[u] || is_new[u];
      }
      // dead prefill rows and empty decode slots: nothing to fetch, nothing to add
      if (__builtin_amdgcn_ballot_w64(work) == 0) continue;
#pragma unroll
      for (int u = 0; u < kVUnroll; ++u) {
        const int tt = tt0 + u * kGroups;
        const int t = t_begin + (tt < T ? tt : 0);
        const bf16_t* vr = v_new + new_off;
        if (any[u] && !is_new[u])
          vr = (t < cap) ? v_prefill + (plane_p + t) * kD : v_dec + (plane_d + (t - cap)) * kD;
        raw[u] = stream_load(reinterpret_cast<const u32x4*>(vr + lir * 8));
        if (is_new[u]) *reinterpret_cast<u32x4*>(v_dec + (plane_d + new_slot) * kD + lir * 8) = raw[u];
      }
#pragma unroll
      for (int u = 0; u < kVUnroll; ++u) {
        float vf[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          vf[2 * i] = __uint_as_float(raw[u][i] << 16);
          vf[2 * i + 1] = __uint_as_float(raw[u][i] & 0xffff0000u);
        }
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
#pragma unroll
          for (int e = 0; e < 8; ++e) o[hh][e] = fmaf(p[u][hh], vf[e], o[hh][e]);
      }
    }
  }
  // sum over the four row groups of a wave, then over the waves
#pragma unroll
  for (int hh = 0; hh < G; ++hh)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      o[hh][e] = sum_across_halves(sum_across_row_pairs(o[hh][e]));
    }
  if (lane < 16) {
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
      for (int e = 0; e < 8; ++e) s_o[wave][hh][lir * 8 + e] = o[hh][e];
  }
  __syncthreads();
  for (int idx = tid; idx < G * kD; idx += kThreads) {
    const int hh = idx / kD, dd = idx % kD;
    if (hh >= n_group) continue;
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) acc += s_o[w][hh][dd];
    const size_t r = (head0 + hh) * n_splits + split;
    part_o[r * kD + dd] = acc;
    if (dd == 0) part_ml[r] = make_float2(s_M[hh], s_L[hh]);
  }
}

}  // namespace

bool decode_uses_mfma(const DecodeDims& d) {
  return d.dtype == SHOTKV_BF16 && d.D == kD && d.split_tokens <= kMaxRange;
}

hipError_t launch_decode_partial_mfma(const DecodeDims& d, const shotkv_decode_state& st, const void* q_new,
                                      const void* k_new, const void* v_new, const DecodeWorkspace& w,
                                      hipStream_t s) {
  const dim3 grid(d.n_splits, d.H_kv, d.S), block(kThreads);
  const float c = d.sm_scale * kLog2e;
  KernelTimer timer(d.timing, kKernelDecodePartial, s);
#define SHOTKV_LAUNCH_DEC(GG)                                                                           \
  hipLaunchKernelGGL(decode_partial_mfma_kernel<GG>, grid, block, 0, s,                                 \
                     static_cast<const bf16_t*>(st.k_prefill), static_cast<const bf16_t*>(st.v_prefill), \
                     st.prefill_count, static_cast<bf16_t*>(st.k_dec), static_cast<bf16_t*>(st.v_dec),   \
                     st.slot_pos, d.cap, d.n_slots, d.H, d.H_kv, d.G, d.n_splits, d.split_tokens, c,     \
                     static_cast<const bf16_t*>(q_new), static_cast<const bf16_t*>(k_new),               \
                     static_cast<const bf16_t*>(v_new), w.part_ml, w.part_o, w.z_dec, w.new_slot)
  switch (padded_group(d.G)) {
    case 1: SHOTKV_LAUNCH_DEC(1); break;
    case 2: SHOTKV_LAUNCH_DEC(2); break;
    case 4: SHOTKV_LAUNCH_DEC(4); break;
    case 8: SHOTKV_LAUNCH_DEC(8); break;
    default: return hipErrorInvalidValue;
  }
#undef SHOTKV_LAUNCH_DEC
  return hipGetLastError();
}

}  // namespace shotkv
