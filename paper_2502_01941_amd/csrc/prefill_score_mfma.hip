// Window-attention softmax partials on the gfx950 matrix cores (Section 5.1, Eq. 3: alpha_{t,h}).
//
// Shape: bf16, head_dim 128, R = G*W in {32, 64, 128} query rows per KV head.
//
// Work unit = (wave, chunk).  A wave keeps all R x 128 window queries of its KV head in registers as
// MFMA B operands and walks its chunks in blocks of 32 keys: S^T[32 keys x R queries] = K_blk * Q^T
// with v_mfma_f32_32x32x16_bf16.  Keys run along the accumulator registers and queries along the
// lanes, so the row-softmax statistics (max and sum over keys) are in-lane reductions; only the two
// lane halves are merged, once per chunk.  K blocks are streamed global -> LDS with 16-byte
// direct-to-LDS loads (fully coalesced 256-byte rows), double buffered per wave, and read back in MFMA
// A-operand layout; a 16-byte-slot XOR swizzle keeps those reads free of bank conflicts.  Waves never
// synchronise with each other.
#include "common.hpp"

namespace shotkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kD = 128;
constexpr int kBlockKeys = 32;
constexpr int kRowBytes = kD * 2;                       // 256
constexpr int kBufBytes = kBlockKeys * kRowBytes;       // 8 KB per wave per buffer
constexpr int kLoadsPerBlock = kBufBytes / (kWave * 16);  // 8 direct-to-LDS instructions

// Issue the 8 direct-to-LDS loads of one 32-key block.  LDS slot p (16-byte units) = i*64 + lane
// holds key row r = p/16, 16-byte column (p%16) ^ (r%16) of that row.  Rows past the end of the chunk
// re-read its last key (they are masked later), so every address stays inside the chunk.
__device__ __forceinline__ void issue_block(const char* __restrict__ k_plane, int key0, int rem,
                                            char* lds_buf, int lane) {
  const int last = rem - 1;  // rem >= 1
#pragma unroll
  for (int i = 0; i < kLoadsPerBlock; ++i) {
    const int r = i * 4 + (lane >> 4);
    const int col = (lane & 15) ^ (r & 15);
    const int rr = min(r, last);
    const char* src = k_plane + static_cast<size_t>(key0 + rr) * kRowBytes + col * 16;
    __builtin_amdgcn_global_load_lds((glb_void*)src, (lds_void*)(lds_buf + i * 1024), 16, 0, 0);
  }
}

template <int NQB>
__device__ __forceinline__ void compute_block(const char* lds_buf, const bf16x8 (&bq)[NQB][8], int lane,
                                              int key0, int rem, int causal_base, int W, float c,
                                              float (&m_run)[NQB], float (&l_run)[NQB]) {
  floatx16 acc[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[qb][v] = 0.f;

  const int row = lane & 31, half = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const int col = (2 * ks + half) ^ (row & 15);
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(lds_buf + row * kRowBytes + col * 16);
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
      acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[qb][ks], acc[qb], 0, 0, 0);
  }

  // accumulator v of this lane is key row 8*(v/4) + 4*half + v%4 of the block, query column `row`
  const bool ragged = rem < kBlockKeys;
  const bool in_window = key0 + kBlockKeys - 1 > causal_base;  // causal_base = n_tokens - W
  if (ragged || in_window) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int j = (qb * 32 + row) % W;
      const int last_visible = causal_base + j;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int kr = 8 * (v >> 2) + 4 * half + (v & 3);
        if (kr >= rem || key0 + kr > last_visible) acc[qb][v] = -INFINITY;
      }
    }
  }
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    float bm = acc[qb][0];
#pragma unroll
    for (int v = 1; v < 16; ++v) bm = fmaxf(bm, acc[qb][v]);
    const float m_new = fmaxf(m_run[qb], bm * c);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_safe);
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) s += __builtin_amdgcn_exp2f(fmaf(acc[qb][v], c, -m_safe));
    l_run[qb] = l_run[qb] * alpha + s;
    m_run[qb] = m_new;
  }
}

template <int NQB>
__global__ __launch_bounds__(kThreads, 2) void score_partials_mfma_kernel(
    const bf16_t* __restrict__ q_obs, const bf16_t* __restrict__ k, int n_tokens, int H, int H_kv, int W,
    float c, const int32_t* __restrict__ n_chunks, const int32_t* __restrict__ chunk_start,
    const int32_t* __restrict__ chunk_len, int max_c, int chunks_per_wave,
    float2* __restrict__ partial) {
  constexpr int R = NQB * 32;
  // two separately declared buffers so that loads into one are independent of reads from the other
  __shared__ __attribute__((aligned(16))) char lds_a[kWavesPerBlock][kBufBytes];
  __shared__ __attribute__((aligned(16))) char lds_b[kWavesPerBlock][kBufBytes];

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

  char* buf_a = lds_a[wave];
  char* buf_b = lds_b[wave];
  const int causal_base = n_tokens - W;

  float m_run[NQB], l_run[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

  // stream of 32-key blocks over the wave's chunks; `cur` is in flight to / resident in buffer A on
  // even steps and buffer B on odd steps
  int cur_c = c_begin;
  int cur_key0 = __builtin_amdgcn_readfirstlane(cs[cur_c]);
  int cur_rem = __builtin_amdgcn_readfirstlane(cl[cur_c]);
  issue_block(k_plane, cur_key0, cur_rem, buf_a, lane);
  bool use_a = true;

  while (true) {
    // successor block
    int nxt_c = cur_c, nxt_key0 = cur_key0 + kBlockKeys, nxt_rem = cur_rem - kBlockKeys;
    bool has_next = true;
    if (nxt_rem <= 0) {
      nxt_c = cur_c + 1;
      has_next = nxt_c < c_end;
      if (has_next) {
        nxt_key0 = __builtin_amdgcn_readfirstlane(cs[nxt_c]);
        nxt_rem = __builtin_amdgcn_readfirstlane(cl[nxt_c]);
      }
    }
    if (has_next) {
      issue_block(k_plane, nxt_key0, nxt_rem, use_a ? buf_b : buf_a, lane);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerBlock) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    if (use_a)
      compute_block<NQB>(buf_a, bq, lane, cur_key0, cur_rem, causal_base, W, c, m_run, l_run);
    else
      compute_block<NQB>(buf_b, bq, lane, cur_key0, cur_rem, causal_base, W, c, m_run, l_run);

    if (cur_rem <= kBlockKeys) {  // last block of its chunk: merge the lane halves and emit
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const float mo = __shfl_xor(m_run[qb], 32, kWave);
        const float lo = __shfl_xor(l_run[qb], 32, kWave);
        const float mn = fmaxf(m_run[qb], mo);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        const float l = l_run[qb] * __builtin_amdgcn_exp2f(m_run[qb] - ms) +
                        lo * __builtin_amdgcn_exp2f(mo - ms);
        if (lane < 32) out[static_cast<size_t>(cur_c) * R + qb * 32 + lane] = make_float2(mn, l);
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
      }
    }
    if (!has_next) break;
    cur_c = nxt_c; cur_key0 = nxt_key0; cur_rem = nxt_rem;
    use_a = !use_a;
  }
}

int pick_chunks_per_wave(const PrefillDims& d, int max_c) {
  // aim for a few thousand workgroups so that 256 CUs x 2 resident workgroups stay busy, while a wave
  // amortises its query registers over as many chunks as that allows
  const long total_chunks = static_cast<long>(max_c) * d.H_kv * d.P;
  long cpw = total_chunks / (kWavesPerBlock * 4096L);
  if (cpw < 1) cpw = 1;
  if (cpw > 16) cpw = 16;
  return static_cast<int>(cpw);
}

}  // namespace

bool score_uses_mfma(const PrefillDims& d) {
  return d.dtype == SHOTKV_BF16 && d.D == kD && (d.R == 32 || d.R == 64 || d.R == 128);
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
