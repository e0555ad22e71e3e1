// Decode step over the compressed cache (Section 5.1, Eq. 7-9; Algorithm 1 phase 2).
//
// decode_partial : split-KV attention of the new query heads over [prefill rows | decode slots],
//                  shape-generic version (fp32 inputs, head_dim 64; bf16 with head_dim 128 takes the
//                  matrix-core kernel in decode_mfma.hip).  Each workgroup owns one token range of one
//                  (sequence, KV head), streams K and V once with 16-byte lanes, and keeps an online
//                  softmax (max, sum, weighted V) per query head of the group.  It also appends
//                  k_new/v_new to the chosen free slot and records the scaled logits of decode tokens
//                  for the retention score.
// decode_finish  : per sequence, one workgroup computes Score(t) = sum_h alpha_{t,h} for the decode
//                  tokens (Eq. 7) and evicts the lowest-scored earlier token when the decode cache
//                  exceeds its budget (Eq. 8 in capacity form), while further workgroups merge the
//                  splits of four query heads each into the attention output.  (A kernel boundary
//                  after decode_partial is cheaper than a device-scope fence: the workgroups of a
//                  sequence sit on different XCDs with separate L2 caches.)
#include "common.hpp"

namespace shotkv {

namespace {

#ifndef SHOTKV_DEC_THREADS
#define SHOTKV_DEC_THREADS 256
#endif
#ifndef SHOTKV_DEC_UNROLL
#define SHOTKV_DEC_UNROLL 1
#endif
#ifndef SHOTKV_DEC_TARGET_GROUPS
#define SHOTKV_DEC_TARGET_GROUPS 1024
#endif
constexpr int kDecThreads = SHOTKV_DEC_THREADS;
constexpr int kDecWaves = kDecThreads / kWave;
constexpr int kUnroll = SHOTKV_DEC_UNROLL;  // tokens a lane group has in flight

// lowest free slot of a sequence, -1 if none; every thread of the block gets the answer
__device__ int find_free_slot(const int32_t* __restrict__ slot_pos, int n_slots, int* s_red) {
  int best = INT32_MAX;
  for (int i = threadIdx.x; i < n_slots; i += blockDim.x)
    if (slot_pos[i] < 0) { best = i; break; }
  for (int o = kWave / 2; o > 0; o >>= 1) best = min(best, __shfl_xor(best, o, kWave));
  if (threadIdx.x % kWave == 0) s_red[threadIdx.x / kWave] = best;
  __syncthreads();
  int r = INT32_MAX;
  for (int w = 0; w < static_cast<int>(blockDim.x) / kWave; ++w) r = min(r, s_red[w]);
  __syncthreads();
  return r == INT32_MAX ? -1 : r;
}

template <typename T> struct Vec16;
template <> struct Vec16<bf16_t> {
  static constexpr int kElems = 8;
  __device__ static void unpack(const uint4& raw, float* f) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <> struct Vec16<float> {
  static constexpr int kElems = 4;
  __device__ static void unpack(const uint4& raw, float* f) {
    f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y);
    f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
  }
};

template <typename T, int D, int G>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(
    const T* __restrict__ k_prefill, const T* __restrict__ v_prefill,
    const int32_t* __restrict__ prefill_count, T* __restrict__ k_dec, T* __restrict__ v_dec,
    const int32_t* __restrict__ slot_pos, int cap, int n_slots, int H, int H_kv, int n_group,
    int n_splits, int split_tokens, float scale_log2e, const T* __restrict__ q_new,
    const T* __restrict__ k_new,
    const T* __restrict__ v_new, float2* __restrict__ part_ml, float* __restrict__ part_o,
    float* __restrict__ z_dec, int32_t* __restrict__ new_slot_out) {
  constexpr int E = Vec16<T>::kElems;       // elements per 16-byte lane
  constexpr int LPR = D / E;                // lanes per K/V row
  constexpr int GPW = kWave / LPR;          // token groups per wave
  constexpr int NG = kDecWaves * GPW;       // token groups per workgroup
  const int split = blockIdx.x, g = blockIdx.y, s = blockIdx.z;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int lir = lane % LPR;               // lane within the row
  const int grp = wave * GPW + lane / LPR;

  __shared__ int s_red[kDecWaves];
  __shared__ float s_m[kDecWaves][G];
  __shared__ float s_l[kDecWaves][G];
  __shared__ float s_o[kDecWaves][G][D];

  const int32_t* sp = slot_pos + static_cast<size_t>(s) * n_slots;
  const int pc = min(prefill_count[s], cap);
  const int t_begin = split * split_tokens;
  const int t_end = min(t_begin + split_tokens, pc + n_slots);
  // only a range that reaches into the decode slots needs to know which slot takes the new token;
  // ranges of prefill rows start streaming at once (if the pool turns out to be full their partials
  // are simply not used)
  const int new_slot = (t_end > pc) ? find_free_slot(sp, n_slots, s_red) : n_slots;
  if (t_end > pc && g == 0 && tid == 0 && t_end == pc + n_slots) new_slot_out[s] = new_slot;

  float m[G], l[G], o[G][E], q[G][E];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = -INFINITY;
    l[h] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) o[h][e] = 0.f;
    // G is the group size rounded up to a power of two; heads past the real n_group are zero queries
    uint4 raw = make_uint4(0u, 0u, 0u, 0u);
    if (h < n_group)
      raw = *reinterpret_cast<const uint4*>(q_new + (static_cast<size_t>(s) * H + g * n_group + h) * D + lir * E);
    Vec16<T>::unpack(raw, q[h]);
  }

  const size_t plane_p = (static_cast<size_t>(s) * H_kv + g) * cap;
  const size_t plane_d = (static_cast<size_t>(s) * H_kv + g) * n_slots;
  const size_t new_off = (static_cast<size_t>(s) * H_kv + g) * D;

  if (new_slot >= 0) {
    for (int t0 = t_begin + grp; t0 < t_end; t0 += NG * kUnroll) {
      uint4 kraw[kUnroll], vraw[kUnroll];
      bool valid[kUnroll];
      int slot_of[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int t = t0 + u * NG;
        valid[u] = false;
        slot_of[u] = -1;
        const T* kr = nullptr;
        const T* vr = nullptr;
        if (t < t_end) {
          if (t < pc) {
            kr = k_prefill + (plane_p + t) * D;
            vr = v_prefill + (plane_p + t) * D;
          } else {
            const int slot = t - pc;
            if (slot == new_slot) {
              kr = k_new + new_off;
              vr = v_new + new_off;
              slot_of[u] = slot;
            } else if (sp[slot] >= 0) {
              kr = k_dec + (plane_d + slot) * D;
              vr = v_dec + (plane_d + slot) * D;
              slot_of[u] = slot;
            }
          }
        }
        if (kr) {
          valid[u] = true;
          kraw[u] = *reinterpret_cast<const uint4*>(kr + lir * E);
          vraw[u] = *reinterpret_cast<const uint4*>(vr + lir * E);
          if (slot_of[u] == new_slot) {  // append: this workgroup is the only reader of the slot
            *reinterpret_cast<uint4*>(k_dec + (plane_d + new_slot) * D + lir * E) = kraw[u];
            *reinterpret_cast<uint4*>(v_dec + (plane_d + new_slot) * D + lir * E) = vraw[u];
          }
        }
      }
      float z[kUnroll][G];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        float kf[E];
        if (valid[u]) Vec16<T>::unpack(kraw[u], kf);
#pragma unroll
        for (int h = 0; h < G; ++h) {
          float acc = 0.f;
          if (valid[u]) {
#pragma unroll
            for (int e = 0; e < E; ++e) acc = fmaf(q[h][e], kf[e], acc);
          }
#pragma unroll
          for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
          z[u][h] = valid[u] ? acc * scale_log2e : -INFINITY;
        }
        if (valid[u] && slot_of[u] >= 0 && lir == 0) {
#pragma unroll
          for (int h = 0; h < G; ++h)
            if (h < n_group) z_dec[(static_cast<size_t>(s) * H + g * n_group + h) * n_slots + slot_of[u]] = z[u][h];
        }
      }
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float mn = m[h];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) mn = fmaxf(mn, z[u][h]);
        if (mn == -INFINITY) continue;  // nothing valid yet for this group
        const float alpha = __builtin_amdgcn_exp2f(m[h] - mn);
        float pw[kUnroll];
        float psum = 0.f;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          pw[u] = __builtin_amdgcn_exp2f(z[u][h] - mn);
          psum += pw[u];
        }
        l[h] = l[h] * alpha + psum;
        m[h] = mn;
#pragma unroll
        for (int e = 0; e < E; ++e) o[h][e] *= alpha;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          if (valid[u]) {
            float vf[E];
            Vec16<T>::unpack(vraw[u], vf);
#pragma unroll
            for (int e = 0; e < E; ++e) o[h][e] = fmaf(pw[u], vf[e], o[h][e]);
          }
        }
      }
    }
  }

  // merge the token groups of a wave (same lir, different group) with shuffles ...
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float mo = __shfl_xor(m[h], off, kWave);
      const float lo = __shfl_xor(l[h], off, kWave);
      const float mn = fmaxf(m[h], mo);
      const float a = (m[h] == -INFINITY) ? 0.f : exp2f(m[h] - mn);
      const float b = (mo == -INFINITY) ? 0.f : exp2f(mo - mn);
      l[h] = l[h] * a + lo * b;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const float oo = __shfl_xor(o[h][e], off, kWave);
        o[h][e] = o[h][e] * a + oo * b;
      }
      m[h] = mn;
    }
  }
  // ... then the waves through LDS
  if (lane < LPR) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      if (lane == 0) { s_m[wave][h] = m[h]; s_l[wave][h] = l[h]; }
#pragma unroll
      for (int e = 0; e < E; ++e) s_o[wave][h][lir * E + e] = o[h][e];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * D; idx += kDecThreads) {
    const int h = idx / D, dd = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) M = fmaxf(M, s_m[w][h]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float a = (s_m[w][h] == -INFINITY) ? 0.f : exp2f(s_m[w][h] - M);
      L += s_l[w][h] * a;
      O += s_o[w][h][dd] * a;
    }
    if (h >= n_group) continue;
    const size_t row = (static_cast<size_t>(s) * H + g * n_group + h) * n_splits + split;
    part_o[row * D + dd] = O;
    if (dd == 0) part_ml[row] = make_float2(M, L);
  }
}

constexpr int kFinThreads = 1024;
constexpr int kFinWaves = kFinThreads / kWave;
constexpr int kFinMaxHeads = 64;

// lower score first, then the newer token: the order in which decode tokens are evicted
__device__ __forceinline__ bool evict_before(float sa, int pa, float sb, int pb) {
  return sa < sb || (sa == sb && pa > pb);
}

// Second half of a decode step.  Per sequence, workgroup 0 turns the decode-slot logits into
// Score(t) = sum over heads of the attention weight (Eq. 7) and retains under the budget (Eq. 8: the
// new token is exempt, the lowest score goes, the newest among equals); workgroups 1.. each merge the
// split partials of kFinHeadsPerGroup query heads into the attention output (Eq. 9).  Every workgroup
// first derives the softmax statistics of the heads it needs from the split partials; after that all
// of its loads are independent of one another, so the kernel costs two memory round trips.
constexpr int kFinHeadsPerGroup = 4;
__global__ __launch_bounds__(kFinThreads) void decode_finish_kernel(
    const float2* __restrict__ part_ml, const float* __restrict__ part_o,
    const float* __restrict__ z_dec, int32_t* __restrict__ slot_pos,
    const int32_t* __restrict__ new_slot_in, int n_slots, int H, int D, int n_splits, int budget,
    int step_index, float* __restrict__ out, float* __restrict__ token_scores,
    int32_t* __restrict__ evicted_pos, int32_t* __restrict__ status) {
  const int s = blockIdx.y, tid = threadIdx.x;
  const int lane = tid % kWave, wave = tid / kWave;
  __shared__ float s_M[kFinMaxHeads];
  __shared__ float s_invL[kFinMaxHeads];
  __shared__ float s_w[kFinHeadsPerGroup][kDecodeMaxSplits];  // merge workgroups only
  __shared__ float s_best_score[kFinWaves];
  __shared__ int s_best_pos[kFinWaves];
  __shared__ int s_best_slot[kFinWaves];
  __shared__ int s_count[kFinWaves];

  int32_t* sp = slot_pos + static_cast<size_t>(s) * n_slots;
  const int new_slot = new_slot_in[s];
  const size_t head0 = static_cast<size_t>(s) * H;
  const bool retain = blockIdx.x == 0;
  // heads whose statistics this workgroup needs: all of them for the scores, its own for the merge
  const int h_lo = retain ? 0 : (static_cast<int>(blockIdx.x) - 1) * kFinHeadsPerGroup;
  const int h_hi = retain ? H : min(h_lo + kFinHeadsPerGroup, H);
  // (requested before the slot index above is looked at, so that the two loads travel together)
  // global softmax statistics per head: one wave per head, lanes over the splits; each split's weight
  // 2^(m - M) is kept so that the merge below is a plain weighted sum
  // (a wave's heads are taken two at a time so that their first loads travel together)
  for (int h = h_lo + wave; h < h_hi; h += 2 * kFinWaves) {
    const int h2 = h + kFinWaves;
    const bool two = h2 < h_hi;
    const float2* ml = part_ml + (head0 + h) * n_splits;
    const float2* ml2 = part_ml + (head0 + (two ? h2 : h)) * n_splits;
    float M = -INFINITY, M2 = -INFINITY;
    for (int i = lane; i < n_splits; i += kWave) {
      const float a = ml[i].x, b = ml2[i].x;
      M = fmaxf(M, a);
      M2 = fmaxf(M2, b);
    }
    M = wave_max(M);
    M2 = wave_max(M2);
    float L = 0.f, L2 = 0.f;
    for (int i = lane; i < n_splits; i += kWave) {  // second look at the same few bytes: out of cache
      const float2 x = ml[i], y = ml2[i];
      const float wgt = x.y > 0.f ? __builtin_amdgcn_exp2f(x.x - M) : 0.f;
      const float wgt2 = y.y > 0.f ? __builtin_amdgcn_exp2f(y.x - M2) : 0.f;
      L += x.y * wgt;
      L2 += y.y * wgt2;
      if (!retain) {
        s_w[h - h_lo][i] = wgt;
        if (two) s_w[h2 - h_lo][i] = wgt2;
      }
    }
    L = wave_sum(L);
    L2 = wave_sum(L2);
    if (lane == 0) {
      s_M[h] = M; s_invL[h] = 1.f / L;
      if (two) { s_M[h2] = M2; s_invL[h2] = 1.f / L2; }
    }
  }
  if (new_slot < 0) {  // pool full: the step is void for this sequence
    if (retain) {
      if (token_scores)
        for (int i = tid; i < n_slots; i += kFinThreads) token_scores[static_cast<size_t>(s) * n_slots + i] = 0.f;
      if (tid == 0) {
        status[s] = SHOTKV_ST_NO_FREE_SLOT;
        if (evicted_pos) evicted_pos[s] = -1;
      }
    } else {
      for (int i = h_lo * D + tid; i < h_hi * D; i += kFinThreads) out[head0 * D + i] = 0.f;
    }
    return;
  }

  __syncthreads();

  if (!retain) {  // attention output of this workgroup's heads
    for (int idx = h_lo * D + tid; idx < h_hi * D; idx += kFinThreads) {
      const int h = idx / D, dd = idx - h * D;
      const float* po = part_o + (head0 + h) * n_splits * D + dd;
      float acc = 0.f;
      for (int i = 0; i < n_splits; ++i) acc = fmaf(po[static_cast<size_t>(i) * D], s_w[h - h_lo][i], acc);
      out[(head0 + h) * D + dd] = acc * s_invL[h];
    }
    return;
  }

  // retention scores and the eviction candidate
  float best_score = INFINITY;
  int best_pos = -1, best_slot = -1, count = 0;
  // A pool of budget + 1 slots is one more than a round of threads: the few slots past the last full
  // round are scored by one wave each, lanes over the heads, and their logits are requested here, ahead
  // of the main loop, so that they do not cost a dependent trip to memory of their own.
  constexpr int kMaxExtra = 4;  // per wave
  int n_extra = n_slots > kFinThreads ? n_slots % kFinThreads : 0;
  if (n_extra > kMaxExtra * kFinWaves) n_extra = 0;
  const int n_main = n_slots - n_extra;
  float ez[kMaxExtra];
  int epos[kMaxExtra];
#pragma unroll
  for (int k = 0; k < kMaxExtra; ++k) {
    const int slot = n_main + wave + k * kFinWaves;
    ez[k] = -INFINITY;
    epos[k] = -1;
    if (slot < n_slots) {
      epos[k] = (slot == new_slot) ? step_index : sp[slot];
      if (lane < H) ez[k] = z_dec[(head0 + lane) * n_slots + slot];
    }
  }
  for (int slot = tid; slot < n_main; slot += kFinThreads) {
    const int pos = (slot == new_slot) ? step_index : sp[slot];
    float score = 0.f;
    if (pos >= 0) {
      ++count;
      const float* z = z_dec + head0 * n_slots + slot;
      for (int h = 0; h < H; ++h)
        score += __builtin_amdgcn_exp2f(z[static_cast<size_t>(h) * n_slots] - s_M[h]) * s_invL[h];
      if (slot != new_slot && (best_slot < 0 || evict_before(score, pos, best_score, best_pos))) {
        best_score = score; best_pos = pos; best_slot = slot;
      }
    }
    if (token_scores) token_scores[static_cast<size_t>(s) * n_slots + slot] = score;
  }
#pragma unroll
  for (int k = 0; k < kMaxExtra; ++k) {
    const int slot = n_main + wave + k * kFinWaves;
    if (slot < n_slots) {  // wave-uniform
      const int pos = epos[k];
      float part = 0.f;
      if (pos >= 0 && lane < H) part = __builtin_amdgcn_exp2f(ez[k] - s_M[lane]) * s_invL[lane];
      // same order of the head sum as in the main loop would need a serial add; a tree sum over the
      // heads differs from it only in rounding, within the score tolerance
      const float score = wave_sum(part);
      if (lane == 0) {
        if (pos >= 0) {
          ++count;
          if (slot != new_slot && (best_slot < 0 || evict_before(score, pos, best_score, best_pos))) {
            best_score = score; best_pos = pos; best_slot = slot;
          }
        }
        if (token_scores) token_scores[static_cast<size_t>(s) * n_slots + slot] = score;
      }
    }
  }
  for (int o = kWave / 2; o > 0; o >>= 1) {
    const float os = __shfl_xor(best_score, o, kWave);
    const int op = __shfl_xor(best_pos, o, kWave);
    const int ol = __shfl_xor(best_slot, o, kWave);
    count += __shfl_xor(count, o, kWave);
    if (ol >= 0 && (best_slot < 0 || evict_before(os, op, best_score, best_pos))) {
      best_score = os; best_pos = op; best_slot = ol;
    }
  }
  if (lane == 0) {
    s_best_score[wave] = best_score; s_best_pos[wave] = best_pos;
    s_best_slot[wave] = best_slot; s_count[wave] = count;
  }
  __syncthreads();  // also: every thread has read its slot_pos entries before thread 0 rewrites two
  if (tid == 0) {
    int total = s_count[0];  // this thread already holds wave 0's candidate
    for (int w = 1; w < kFinWaves; ++w) {
      total += s_count[w];
      if (s_best_slot[w] >= 0 &&
          (best_slot < 0 || evict_before(s_best_score[w], s_best_pos[w], best_score, best_pos))) {
        best_score = s_best_score[w]; best_pos = s_best_pos[w]; best_slot = s_best_slot[w];
      }
    }
    sp[new_slot] = step_index;
    int ev = -1;
    if (total > budget && best_slot >= 0) {
      ev = best_pos;
      sp[best_slot] = -1;
    }
    if (evicted_pos) evicted_pos[s] = ev;
    status[s] = SHOTKV_ST_OK;
  }
}

}  // namespace

int decode_splits(int S, int H_kv, int total_tokens) {
  // enough workgroups to fill 256 CUs several times over, but no split shorter than 128 tokens and
  // no more splits than the finish kernel takes
  const int pairs = S * H_kv;
  int splits = ceil_div(SHOTKV_DEC_TARGET_GROUPS, pairs);
  const int max_by_tokens = total_tokens / 128 > 0 ? total_tokens / 128 : 1;
  if (splits > max_by_tokens) splits = max_by_tokens;
  const int min_by_range = ceil_div(total_tokens, kDecodeMaxRange);  // what the matrix-core path can hold
  if (splits < min_by_range) splits = min_by_range;
  if (splits > kDecodeMaxSplits) splits = kDecodeMaxSplits;
  if (splits < 1) splits = 1;
  return splits;
}

template <typename T, int D>
static hipError_t launch_partial_g(const DecodeDims& d, const shotkv_decode_state& st, const void* q_new,
                                   const void* k_new, const void* v_new, const DecodeWorkspace& w,
                                   hipStream_t s) {
  const dim3 grid(d.n_splits, d.H_kv, d.S), block(kDecThreads);
  const float c = d.sm_scale * kLog2e;
  KernelTimer timer(d.timing, kKernelDecodePartial, s);
#define SHOTKV_LAUNCH_DEC(GG)                                                                          \
  hipLaunchKernelGGL((decode_partial_kernel<T, D, GG>), grid, block, 0, s,                             \
                     static_cast<const T*>(st.k_prefill), static_cast<const T*>(st.v_prefill),         \
                     st.prefill_count, static_cast<T*>(st.k_dec), static_cast<T*>(st.v_dec),           \
                     st.slot_pos, d.cap, d.n_slots, d.H, d.H_kv, d.G, d.n_splits, d.split_tokens, c,    \
                     static_cast<const T*>(q_new), static_cast<const T*>(k_new),                       \
                     static_cast<const T*>(v_new), w.part_ml, w.part_o, w.z_dec, w.new_slot)
  switch (padded_group(d.G)) {  // the kernel is instantiated for power-of-two groups and skips the padding
    case 1: SHOTKV_LAUNCH_DEC(1); break;
    case 2: SHOTKV_LAUNCH_DEC(2); break;
    case 4: SHOTKV_LAUNCH_DEC(4); break;
    case 8: SHOTKV_LAUNCH_DEC(8); break;
    default: return hipErrorInvalidValue;
  }
#undef SHOTKV_LAUNCH_DEC
  return hipGetLastError();
}

hipError_t launch_decode_partial(const DecodeDims& d, const shotkv_decode_state& st, const void* q_new,
                                 const void* k_new, const void* v_new, const DecodeWorkspace& w,
                                 hipStream_t s) {
  if (decode_uses_mfma(d)) return launch_decode_partial_mfma(d, st, q_new, k_new, v_new, w, s);
  if (d.dtype == SHOTKV_BF16) {
    if (d.D == 128) return launch_partial_g<bf16_t, 128>(d, st, q_new, k_new, v_new, w, s);
    if (d.D == 64) return launch_partial_g<bf16_t, 64>(d, st, q_new, k_new, v_new, w, s);
  } else {
    if (d.D == 128) return launch_partial_g<float, 128>(d, st, q_new, k_new, v_new, w, s);
    if (d.D == 64) return launch_partial_g<float, 64>(d, st, q_new, k_new, v_new, w, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_decode_finish(const DecodeDims& d, const shotkv_decode_state& st, float* out,
                                float* token_scores, int32_t* evicted_pos, int32_t* status,
                                const DecodeWorkspace& w, hipStream_t s) {
  if (d.H > kFinMaxHeads || d.n_splits > kDecodeMaxSplits) return hipErrorInvalidValue;
  KernelTimer timer(d.timing, kKernelDecodeFinish, s);
  hipLaunchKernelGGL(decode_finish_kernel, dim3(1 + ceil_div(d.H, kFinHeadsPerGroup), d.S), dim3(kFinThreads), 0, s, w.part_ml, w.part_o, w.z_dec,
                     st.slot_pos, w.new_slot, d.n_slots, d.H, d.D, d.n_splits, d.budget, d.step, out,
                     token_scores, evicted_pos, status);
  return hipGetLastError();
}

}  // namespace shotkv
