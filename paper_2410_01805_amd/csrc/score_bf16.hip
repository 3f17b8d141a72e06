// Retaining head (Section 3.3) on the bf16 matrix cores of gfx950:
//   S~[t][m] = sum_r SiLU( sum_c x[t][c] W1[c][r] ) W2[r][m],   x[t] = [q_t ; k_t ; v_t]
//
// The hidden pre-activations are formed transposed, H^T[r][t] = W1t[r][:] . x[t][:], with
// v_mfma_f32_32x32x16_bf16 (A = rows of the transposed weight, B = token rows; both are contiguous
// along the contraction, so LDS rows are read as 16-byte vectors).  The input row is never
// materialised: each 16-byte piece of a token's row is fetched from q, k or v directly.
// A workgroup owns 128 hidden units x 128 tokens; SiLU and the product with W2 run on the
// accumulators, and the workgroup writes its partial score part[nb][m][t] (nb = hidden block);
// partials are summed in a fixed order by a separate tiny kernel, so results are deterministic.
#include "device_util.h"
#include "kernels.h"

namespace locret {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int RT_M = 128;   // hidden units per workgroup
constexpr int RT_N = 128;   // tokens per workgroup
constexpr int RT_K = 64;    // contraction elements per stage
constexpr int RT_STR = RT_K + 8;

struct ScoreSmem {
  union {
    struct {
      bf16_t A[2][RT_M * RT_STR];
      bf16_t B[2][RT_N * RT_STR];
    } st;
    struct {
      float W2s[RT_M * 32];          // [hidden][m-chunk of up to 32]
      float red[2 * RT_N * 32];      // [wm][token][m-chunk]
    } ep;
  };
};

__global__ __launch_bounds__(256) void score_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                         const bf16_t* __restrict__ v, int Tn, int hd, int kvd,
                                                         const bf16_t* __restrict__ W1t,
                                                         const float* __restrict__ W2f, int K, int h_kv,
                                                         float* __restrict__ part, int part_T) {
  __shared__ ScoreSmem sm;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n32 = lane & 31, hi = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const int t0 = blockIdx.x * RT_N;
  const int nb = blockIdx.y;
  const int r0 = nb * RT_M;

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  // staging: 128 rows x 8 chunks of 16 bytes per operand per stage = 4 chunks per thread each
  uint4 areg[4], breg[4];
  auto load_stage = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int c = tid + 256 * i;
      int row = c >> 3, col = c & 7;
      areg[i] = *(const uint4*)(W1t + (int64_t)(r0 + row) * K + k0 + col * 8);
      int t = t0 + row;
      int cc = k0 + col * 8;                      // column of [q;k;v]; a chunk never straddles tensors
      const bf16_t* src;
      if (cc < hd) src = q + (int64_t)t * hd + cc;
      else if (cc < hd + kvd) src = k + (int64_t)t * kvd + (cc - hd);
      else src = v + (int64_t)t * kvd + (cc - hd - kvd);
      breg[i] = (t < Tn) ? *(const uint4*)src : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int c = tid + 256 * i;
      int row = c >> 3, col = c & 7;
      *(uint4*)(&sm.st.A[buf][row * RT_STR + col * 8]) = areg[i];
      *(uint4*)(&sm.st.B[buf][row * RT_STR + col * 8]) = breg[i];
    }
  };

  const int n_stages = K / RT_K;
  load_stage(0);
  store_stage(0);
  __syncthreads();
  for (int s = 0; s < n_stages; ++s) {
    const int buf = s & 1;
    if (s + 1 < n_stages) load_stage((s + 1) * RT_K);
    const bf16_t* ap = &sm.st.A[buf][(wm * 64 + n32) * RT_STR + hi * 8];
    const bf16_t* bp = &sm.st.B[buf][(wn * 64 + n32) * RT_STR + hi * 8];
#pragma unroll
    for (int ks = 0; ks < RT_K / 16; ++ks) {
      bf16x8 a0 = *(const bf16x8*)(ap + ks * 16);
      bf16x8 a1 = *(const bf16x8*)(ap + 32 * RT_STR + ks * 16);
      bf16x8 b0 = *(const bf16x8*)(bp + ks * 16);
      bf16x8 b1 = *(const bf16x8*)(bp + 32 * RT_STR + ks * 16);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
    }
    if (s + 1 < n_stages) store_stage(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: SiLU in place, then W2 in chunks of up to 32 KV heads ---------------------------
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float z = acc[a][b][r];
        acc[a][b][r] = z / (1.f + __expf(-z));
      }
  for (int m0 = 0; m0 < h_kv; m0 += 32) {
    const int mc = min(32, h_kv - m0);
    __syncthreads();                               // staging buffers / previous chunk no longer read
    for (int i = tid; i < RT_M * mc; i += 256) {
      int hh = i / mc, mm = i % mc;
      sm.ep.W2s[hh * 32 + mm] = W2f[(int64_t)(r0 + hh) * h_kv + m0 + mm];
    }
    __syncthreads();
    for (int mm = 0; mm < mc; ++mm) {
      float s0 = 0.f, s1 = 0.f;                    // token blocks b = 0, 1
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int hh = wm * 64 + a * 32 + (r >> 2) * 8 + hi * 4 + (r & 3);
          float w = sm.ep.W2s[hh * 32 + mm];
          s0 = fmaf(acc[a][0][r], w, s0);
          s1 = fmaf(acc[a][1][r], w, s1);
        }
      s0 += __shfl_xor(s0, 32, 64);
      s1 += __shfl_xor(s1, 32, 64);
      if (hi == 0) {
        sm.ep.red[(wm * RT_N + wn * 64 + n32) * 32 + mm] = s0;
        sm.ep.red[(wm * RT_N + wn * 64 + 32 + n32) * 32 + mm] = s1;
      }
    }
    __syncthreads();
    for (int i = tid; i < RT_N * mc; i += 256) {
      int tl = i % RT_N, mm = i / RT_N;
      int t = t0 + tl;
      if (t < Tn)
        part[((int64_t)nb * h_kv + m0 + mm) * part_T + t] = sm.ep.red[tl * 32 + mm] + sm.ep.red[(RT_N + tl) * 32 + mm];
    }
  }
}

int score_parts_bf16(const Dims& D) {
  if (!D.bf16) return 0;
  if (D.d_R % RT_M != 0 || D.K % RT_K != 0 || D.d % 8 != 0) return 0;
  return D.d_R / RT_M;
}

void launch_score_bf16(const Dims& D, const void* q, const void* k, const void* v, int T, const void* W1t,
                       const float* W2f, float* part, hipStream_t st) {
  dim3 grid((T + RT_N - 1) / RT_N, D.d_R / RT_M);
  hipLaunchKernelGGL(score_mfma_kernel, grid, dim3(256), 0, st, (const bf16_t*)q, (const bf16_t*)k,
                     (const bf16_t*)v, T, D.h * D.d, D.h_kv * D.d, (const bf16_t*)W1t, W2f, D.K, D.h_kv, part, T);
}

}  // namespace locret
