// Retaining head (Section 3.3) on the bf16 matrix cores of gfx950:
//   S~[t][m] = sum_r SiLU( sum_c x[t][c] W1[c][r] ) W2[r][m],   x[t] = [q_t ; k_t ; v_t]
//
// The hidden pre-activations are formed transposed, H^T[r][t] = W1t[r][:] . x[t][:], with
// v_mfma_f32_32x32x16_bf16 (A = rows of the transposed weight, B = token rows; both contiguous
// along the contraction).  A workgroup owns 128 hidden units x 128 tokens (2 x 2 wavefronts of
// 64 x 64), or x 64 tokens (wavefronts of 64 x 32) for chunks too short to give every CU a 128-token tile.
// The input row is never materialised: each stage of 64 contraction elements lies inside
// one of q, k, v and is fetched from that tensor directly.
//
// Operand staging goes global -> LDS without passing through registers (buffer_load ... lds,
// 16 bytes per lane) into a ring of four stages, so three stages are always in flight.  A direct load
// holds its wavefront's issue slot for 60-80 cycles while the CU's vector-memory path (64 B/clk) is
// busy, and a stage needs 32 of them: issued by the computing wavefronts they cost as much time as the
// stage's 16 MFMAs.  So the workgroup has eight wavefronts: 0..3 only compute, 4..7 (their SIMD mates)
// only issue loads, one barrier per stage between them.
// Such a load writes lane L's 16 bytes at LDS base + 16 L, so an instruction fills 8 rows of 128
// bytes back to back; bank conflicts are avoided by permuting WHICH 16-byte chunk a lane fetches:
// position c' of row r holds chunk c' ^ ((r >> 1) & 7), and a fragment read of logical chunk c goes to
// position c ^ ((r >> 1) & 7): rows are 128 bytes, so even and odd rows already sit in different halves
// of the 64 banks, and the 8 even (or odd) rows among 16 consecutive ones must take 8 different positions.
// Rows past the chunk (t >= T) fall outside the buffer descriptor and arrive as zeros.
// The computing wavefronts keep two sets of fragment registers: the MFMAs of a stage run on one while
// the fragments of the next stage are read into the other, one LDS read behind each MFMA.
//
// SiLU and the product with W2 run on the accumulators (the W2 rows of the hidden block were fetched by
// the load wavefronts before the pipeline started); the workgroup writes its partial score
// part[nb][m][t] (nb = hidden block) and a tiny kernel sums the partials in a fixed order, so the
// scores are deterministic.
#include "device_util.h"
#include "kernels.h"

namespace locret {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int RT_M = 128;      // hidden units per workgroup
constexpr int RT_N = 128;      // tokens per workgroup
constexpr int RT_K = 64;       // contraction elements per stage (128 bytes per row)
constexpr int RT_STAGES = 4;
constexpr int RT_TILE_B = RT_M * RT_K * 2;            // bytes of one operand tile (16 KB)
constexpr int RT_STAGE_B = 2 * RT_TILE_B;             // A then B

struct ScoreSmem {
  union {
    unsigned char ring[RT_STAGES * RT_STAGE_B];       // 128 KB
    struct {
      float W2s[RT_M * 32];          // [hidden][m-chunk of up to 32]
      float red[2 * RT_N * 33];      // [wm][token][m-chunk], rows padded to 33 floats (bank spread)
    } ep;
  };
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// sum over the two half-waves without a trip through LDS: after the swap one register holds the low half's
// value in both halves and the other the high half's (the order of the two addends is the same in both halves)
__device__ __forceinline__ float sum_across_halves(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// KSPLIT (short chunks, too few 128 x 128 tiles for the CUs): blockIdx.z takes a slice of the contraction and
// the workgroup leaves its partial pre-activations zpart[z][t][r]; score_finish_kernel sums the slices and
// applies SiLU and W2.  KSPLIT = false: the whole contraction, epilogue below.
// NT = tokens per workgroup: 128 (2 x 2 wavefronts of 64 hidden units x 64 tokens), or 64 (64 x 32 each) for chunks
// that would leave half of the CUs without a 128-token tile; the hidden block stays 128 wide.
template <bool KSPLIT, int NT>
__global__ __launch_bounds__(512) void score_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                         const bf16_t* __restrict__ v, int Tn, int hd, int kvd,
                                                         const bf16_t* __restrict__ W1t,
                                                         const float* __restrict__ W2f, int K, int h_kv,
                                                         float* __restrict__ part, int part_T,
                                                         float* __restrict__ zpart, int d_R) {
  __shared__ __attribute__((aligned(1024))) ScoreSmem sm;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, hi = lane >> 5;
  const bool producer = wave >= 4;               // wave-uniform
  const int pw = wave & 3;                       // producer: fills rows pw*32 .. pw*32+31 of both tiles
  const int wm = (wave >> 1) & 1, wn = wave & 1; // consumer: 64 x 64 sub-tile
  static_assert(NT == 128 || NT == 64, "token tile");
  constexpr int NBT = NT / 64;                   // 32-token blocks per wavefront
  constexpr int B_LOADS = NT / 32;               // direct loads of a producer for the token tile of a stage
  const int t0 = blockIdx.x * NT;
  const int nb = blockIdx.y;
  const int r0 = nb * RT_M;

  f32x16 acc[2][NBT];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < NBT; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  // ---- loads: producer p fills rows p*32 .. p*32+31 of the weight tile and its quarter of the token tile, 8 rows
  // per instruction ----
  const int l_row = lane >> 3;                           // row inside the instruction's 8 rows
  // byte offset of the chunk this lane fetches: row = 8 * instruction + l_row, so (row >> 1) & 7 is
  // (l_row >> 1) for even instructions and (l_row >> 1) ^ 4 for odd ones (ii & 1 below)
  const int l_csw0 = ((lane & 7) ^ (l_row >> 1)) * 16;
  const int l_csw1 = ((lane & 7) ^ (l_row >> 1) ^ 4) * 16;
  const int a_vo = (pw * 32 + l_row) * (K * 2);        // + ii * 8 rows + chunk offset
  const int b_row = pw * (NT / 4) + l_row;               // + ii * 8
  const int n_stages_all = K / RT_K;
  // this workgroup's stages: [s_lo, s_lo + n_stages)
  const int per_z = KSPLIT ? (n_stages_all + (int)gridDim.z - 1) / (int)gridDim.z : n_stages_all;
  const int s_lo = KSPLIT ? (int)blockIdx.z * per_z : 0;
  const int n_stages = KSPLIT ? max(0, min(n_stages_all, s_lo + per_z) - s_lo) : n_stages_all;
  const int q_stages = hd / RT_K, k_stages = kvd / RT_K;
  const int rows_left = min(max(Tn - t0, 0), NT);      // valid token rows of this workgroup

  auto issue = [&](int s_rel, int buf) {
    // (a stage past the last one would get empty descriptors: zeros, no memory access; the loops below
    // do not ask for one: 24 such loads per producer at the end kept every wavefront waiting ~4000 cycles)
    const bool live = s_rel < n_stages;
    const int s = s_lo + s_rel;
    {
      __amdgpu_buffer_rsrc_t ar = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(W1t + (int64_t)r0 * K + (int64_t)s * RT_K), 0, live ? (RT_M * K * 2 - s * RT_K * 2) : 0, 0x00020000);
#pragma unroll
      for (int ii = 0; ii < 4; ++ii)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            ar, (lds_ptr_t)(sm.ring + buf * RT_STAGE_B + (pw * 4 + ii) * 1024), 16, a_vo + ii * 8 * (K * 2) + ((ii & 1) ? l_csw1 : l_csw0), 0, 0, 0);
    }
    {
      const bf16_t* src;
      int rowb, col;
      if (s < q_stages) { src = q; rowb = hd * 2; col = s * RT_K; }
      else if (s < q_stages + k_stages) { src = k; rowb = kvd * 2; col = (s - q_stages) * RT_K; }
      else { src = v; rowb = kvd * 2; col = (s - q_stages - k_stages) * RT_K; }
      // the descriptor starts at (t0, col) and ends with the last valid row, so rows >= T read as zero
      const int64_t span = (int64_t)rows_left * rowb - col * 2;
      __amdgpu_buffer_rsrc_t br = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(src + (int64_t)t0 * (rowb / 2) + col), 0, (live && span > 0) ? (int)span : 0, 0x00020000);
#pragma unroll
      for (int ii = 0; ii < B_LOADS; ++ii)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            br, (lds_ptr_t)(sm.ring + buf * RT_STAGE_B + RT_TILE_B + (pw * B_LOADS + ii) * 1024), 16,
            (b_row + ii * 8) * rowb + ((ii & 1) ? l_csw1 : l_csw0), 0, 0, 0);
    }
  };

  // ---- fragment reads: row (wave part + n32), logical chunk 2 ks + hi at position chunk ^ ((row >> 1) & 7)
  int a_rd[4], b_rd[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int pos = ((2 * ks + hi) ^ ((n32 >> 1) & 7)) * 16;
    a_rd[ks] = (wm * 64 + n32) * 128 + pos;
    b_rd[ks] = RT_TILE_B + (wn * (NT / 2) + n32) * 128 + pos;
  }

  // Fragments: two register sets.  While the 16 (or 8) MFMAs of a stage run on one set, the fragments of the whole
  // next stage (in LDS already, see the invariant below) are requested into the other, one or two reads behind each
  // MFMA, so every read has a full stage to arrive.  (Measured equal to reading six MFMAs ahead: a computing
  // wavefront takes about 720 cycles per stage for 512 cycles of MFMAs either way, almost none of them at the
  // barrier.)
  constexpr int NFR = 4 * (2 + NBT);             // fragments of a stage: per contraction step 2 of W1, NBT of tokens
  bf16x8 fr[2][NFR];
  auto fetch = [&](bf16x8 (&f)[NFR], int buf) {
    const unsigned char* base = sm.ring + buf * RT_STAGE_B;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      f[ks * (2 + NBT) + 0] = *(const bf16x8*)(base + a_rd[ks]);
      f[ks * (2 + NBT) + 1] = *(const bf16x8*)(base + a_rd[ks] + 32 * 128);
      f[ks * (2 + NBT) + 2] = *(const bf16x8*)(base + b_rd[ks]);
      if (NBT == 2) f[ks * (2 + NBT) + 3] = *(const bf16x8*)(base + b_rd[ks] + 32 * 128);
    }
  };
  auto compute = [&](bf16x8 (&f)[NFR], bf16x8 (&fn)[NFR], int next_buf) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NBT; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[ks * (2 + NBT) + a], f[ks * (2 + NBT) + 2 + b], acc[a][b], 0, 0, 0);
    fetch(fn, next_buf);
    // issue order: the fragment reads spread evenly behind the MFMAs (16 for 16, or 12 for 8)
    if (NBT == 2) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
  };

  // The load wavefronts fetch the W2 rows of this hidden block (first 32 KV heads, zero beyond h_kv) before the
  // pipeline starts and hold them until the epilogue: 16 registers they have to spare, and the epilogue does not
  // begin with a trip to memory.  Element i = hidden unit i / 32, KV head i % 32.
  float w2pre[16];
  if (!KSPLIT && producer) {
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      const int i = (tid - 256) + 256 * jj, hh = i >> 5, mm = i & 31;
      const float x = W2f[(int64_t)(r0 + hh) * h_kv + min(mm, h_kv - 1)];     // address clamped, value masked: no branch
      w2pre[jj] = mm < h_kv ? x : 0.f;
    }
  }

  // One barrier per stage.  Invariant at barrier s: stages up to s+1 are in LDS (a producer arrives once at
  // most one stage = 8 of its loads is still in flight) and every consumer has left stage s-1.  Behind it a
  // producer starts stage s+3 in the buffer of stage s-1; a consumer computes stage s and then requests the
  // first fragments of stage s+1.  A bare s_barrier: __syncthreads() would first drain every load in flight.
  if (n_stages == 0) {
    // an empty slice (the host does not launch one): both roles skip the pipeline, the partial is zero
  } else if (producer) {
    issue(0, 0);
    if (1 < n_stages) issue(1, 1);
    if (2 < n_stages) issue(2, 2);
    for (int s0 = 0; s0 < n_stages; s0 += RT_STAGES) {
#pragma unroll
      for (int u = 0; u < RT_STAGES; ++u)
        if (s0 + u < n_stages) {
          // at most stage s+2 may still be in flight; past the end nothing more is issued, and then the
          // count has to drop to zero for stage s+1 to be known complete
          if (s0 + u + 2 < n_stages) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(4 + B_LOADS) : "memory");
          else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          asm volatile("s_barrier" ::: "memory");
          if (s0 + u + RT_STAGES - 1 < n_stages) issue(s0 + u + RT_STAGES - 1, (u + RT_STAGES - 1) % RT_STAGES);
        }
    }
  } else {
    asm volatile("s_barrier" ::: "memory");
    fetch(fr[0], 0);
    for (int s0 = 0; s0 < n_stages; s0 += RT_STAGES) {
#pragma unroll
      for (int u = 0; u < RT_STAGES; ++u)
        if (s0 + u < n_stages) {
          compute(fr[u & 1], fr[(u + 1) & 1], (u + 1) % RT_STAGES);     // (behind the last stage the fetch reads a buffer nobody needs)
          if (s0 + u + 1 < n_stages) asm volatile("s_barrier" ::: "memory");
        }
    }
  }

  if (KSPLIT) {
    if (!producer) {
      float* zp = zpart + (int64_t)blockIdx.z * Tn * d_R;
#pragma unroll
      for (int b = 0; b < NBT; ++b) {
        const int t = t0 + wn * (NT / 2) + b * 32 + n32;
        if (t >= Tn) continue;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq)
            *(float4*)(zp + (int64_t)t * d_R + r0 + wm * 64 + a * 32 + rq * 8 + hi * 4) =
                make_float4(acc[a][b][rq * 4 + 0], acc[a][b][rq * 4 + 1], acc[a][b][rq * 4 + 2], acc[a][b][rq * 4 + 3]);
      }
    }
    return;
  }
  // ---- epilogue: SiLU in place, then W2 in chunks of up to 32 KV heads ---------------------------
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < NBT; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        // SiLU(z) = z / (1 + 2^(-z log2 e)) with the hardware exp2 and reciprocal (1 ulp each: far inside
        // what the bf16 operands of this kernel leave of the result)
        const float z = acc[a][b][r];
        acc[a][b][r] = z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(z * -1.4426950408889634f));
      }
  for (int m0 = 0; m0 < h_kv; m0 += 32) {
    const int mc = min(32, h_kv - m0);
    __syncthreads();                               // ring / previous chunk no longer read
    if (m0 == 0 && producer) {
#pragma unroll
      for (int jj = 0; jj < 16; ++jj) sm.ep.W2s[(tid - 256) + 256 * jj] = w2pre[jj];
    } else if (m0 > 0) {
      for (int i = tid; i < RT_M * 32; i += 512) {
        const int hh = i >> 5, mm = i & 31;
        sm.ep.W2s[i] = mm < mc ? W2f[(int64_t)(r0 + hh) * h_kv + m0 + mm] : 0.f;
      }
    }
    __syncthreads();
    // four KV heads at a time: one 16-byte read of the W2 row per accumulator element
    for (int mq = 0; mq < mc && !producer; mq += 4) {
      float sb[NBT][4];                            // [token block][KV head of the four]
#pragma unroll
      for (int b = 0; b < NBT; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) sb[b][i] = 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int hh = wm * 64 + a * 32 + (r >> 2) * 8 + hi * 4 + (r & 3);
          const float4 w = *(const float4*)&sm.ep.W2s[hh * 32 + mq];
#pragma unroll
          for (int b = 0; b < NBT; ++b) {
            sb[b][0] = fmaf(acc[a][b][r], w.x, sb[b][0]);
            sb[b][1] = fmaf(acc[a][b][r], w.y, sb[b][1]);
            sb[b][2] = fmaf(acc[a][b][r], w.z, sb[b][2]);
            sb[b][3] = fmaf(acc[a][b][r], w.w, sb[b][3]);
          }
        }
#pragma unroll
      for (int b = 0; b < NBT; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float v = sum_across_halves(sb[b][i]);
          if (hi == 0) sm.ep.red[(wm * NT + wn * (NT / 2) + b * 32 + n32) * 33 + mq + i] = v;   // columns >= mc: zeros, not read
        }
    }
    __syncthreads();
    for (int i = tid; i < NT * mc; i += 512) {
      int tl = i % NT, mm = i / NT;
      int t = t0 + tl;
      if (t < Tn)
        part[((int64_t)nb * h_kv + m0 + mm) * part_T + t] = sm.ep.red[tl * 33 + mm] + sm.ep.red[(NT + tl) * 33 + mm];
    }
  }
}

// scores[m][t] = sum_r SiLU(sum_z zpart[z][t][r]) W2[r][m] for the contraction-split launches: one workgroup per
// token, thread i owns hidden units i, i + 256, ... (neighbouring lanes read neighbouring partials and
// neighbouring rows of W2: few cache lines per load instruction), sums over the workgroup in LDS.  Fixed orders
// throughout: deterministic.
constexpr int FIN_THREADS = 256;
__global__ __launch_bounds__(FIN_THREADS) void score_finish_kernel(const float* __restrict__ zpart, int n_z, int Tn,
                                                                   int d_R, const float* __restrict__ W2f, int h_kv,
                                                                   float* __restrict__ part, int part_T) {
  __shared__ float red[FIN_THREADS / 64][8];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int m0 = 0; m0 < h_kv; m0 += 8) {
    const int mc = min(8, h_kv - m0);
    float p[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) p[i] = 0.f;
    const bool vec8 = mc == 8 && (h_kv & 3) == 0;          // a row's 8 weights as two aligned 16-byte loads
    for (int r = tid; r < d_R; r += FIN_THREADS) {
      float z = zpart[(int64_t)t * d_R + r];
      for (int s = 1; s < n_z; ++s) z += zpart[((int64_t)s * Tn + t) * d_R + r];
      const float a = z * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(z * -1.4426950408889634f));
      const float* w = W2f + (int64_t)r * h_kv + m0;
      if (vec8) {
        const float4 w0 = *(const float4*)w, w1 = *(const float4*)(w + 4);
        p[0] = fmaf(a, w0.x, p[0]); p[1] = fmaf(a, w0.y, p[1]); p[2] = fmaf(a, w0.z, p[2]); p[3] = fmaf(a, w0.w, p[3]);
        p[4] = fmaf(a, w1.x, p[4]); p[5] = fmaf(a, w1.y, p[5]); p[6] = fmaf(a, w1.z, p[6]); p[7] = fmaf(a, w1.w, p[7]);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (i < mc) p[i] = fmaf(a, w[i], p[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
      for (int x = 32; x >= 1; x >>= 1) p[i] += __shfl_xor(p[i], x, 64);
    }
    __syncthreads();                                   // the previous chunk's sums have been read
    if (lane == 0)
#pragma unroll
      for (int i = 0; i < 8; ++i) red[wave][i] = p[i];
    __syncthreads();
    if (tid < mc) {
      float sum = red[0][tid];
      for (int w2 = 1; w2 < FIN_THREADS / 64; ++w2) sum += red[w2][tid];
      part[(int64_t)(m0 + tid) * part_T + t] = sum;
    }
  }
}

// Floats of workspace for the partial pre-activations of contraction-split launches.
constexpr int RT_ZROWS = 4096;     // token rows times slices at most
size_t score_bf16_split_floats(const Dims& D, int chunk_max) {
  if (score_parts_bf16(D) == 0 || D.d_R % 4 != 0) return 0;
  const int rows = chunk_max < RT_ZROWS / 4 ? 4 * chunk_max : RT_ZROWS;
  return (size_t)rows * D.d_R;
}

int score_parts_bf16(const Dims& D) {
  if (!D.bf16) return 0;
  // stages must not straddle q / k / v, and byte offsets inside one operand panel must fit 31 bits
  if (D.d_R % RT_M != 0 || (D.h * D.d) % RT_K != 0 || (D.h_kv * D.d) % RT_K != 0) return 0;
  if ((int64_t)RT_M * D.K * 2 >= (1ll << 31) || (int64_t)RT_N * D.h * D.d * 2 >= (1ll << 31)) return 0;
  return D.d_R / RT_M;
}

// Returns the number of partial score tensors written to `part` (the caller sums them): d_R / 128, or 1 when the
// launch split the contraction (short chunks: at most half as many tiles as CUs; each slice keeps at least 8
// stages; Tuning::score_split: 0 = never, k = k slices).  Measured on 32q/8kv x 128, d_R = 1024, in microseconds
// (hot caches): chunks of 2048 tokens 42.4 with 128-token tiles, 37.3 with 64-token tiles, 49.6 with those and two
// slices; chunks of 1024 tokens 32.9 (128-token tiles, 4 slices), 33.3 (64-token tiles), 29.4 (64-token tiles,
// 2 slices); chunks of 3072 or 4096 tokens are a third slower with 64-token tiles (more LDS traffic per MFMA).
int launch_score_bf16(const Dims& D, const void* q, const void* k, const void* v, int T, const void* W1t,
                      const float* W2f, float* part, hipStream_t st, float* zpart, size_t zpart_floats) {
  // Token tile: 64 when 128-token tiles would leave at least half of the 256 CUs without one (T <= 2048 at
  // d_R = 1024).  Tuning::score_nt: 0 = this rule, 64 / 128 = always.
  const int tiles128 = ((T + 127) / 128) * (D.d_R / RT_M);
  const int nt = D.tune.score_nt == 64 || D.tune.score_nt == 128 ? D.tune.score_nt : (tiles128 <= 128 ? 64 : 128);
  dim3 grid((T + nt - 1) / nt, D.d_R / RT_M);
  int n_z = 1;
  if (zpart != nullptr) {
    const int forced = D.tune.score_split;
    const int tiles = (int)(grid.x * grid.y), stages = D.K / RT_K;
    n_z = forced >= 0 ? forced : (256 / tiles >= 2 ? 256 / tiles : 1);
    n_z = n_z > 8 ? 8 : n_z;
    auto last_empty = [&](int n) { return (n - 1) * ((stages + n - 1) / n) >= stages; };   // slices are ceil(stages / n) long
    while (n_z > 1 && ((size_t)n_z * T * D.d_R > zpart_floats || (forced < 0 && stages / n_z < 8) || last_empty(n_z))) --n_z;
    if (n_z < 1) n_z = 1;
  }
  grid.z = n_z;
#define LOCRET_SCORE_LAUNCH(KS, NTT)                                                                                  \
  launch_kernel(score_mfma_kernel<KS, NTT>, grid, dim3(512), 0, st, (const bf16_t*)q, (const bf16_t*)k,                \
                (const bf16_t*)v, T, D.h * D.d, D.h_kv * D.d, (const bf16_t*)W1t, W2f, D.K, D.h_kv, part, T,          \
                KS ? zpart : (float*)nullptr, D.d_R)
  if (n_z == 1) {
    if (nt == 64) LOCRET_SCORE_LAUNCH(false, 64); else LOCRET_SCORE_LAUNCH(false, 128);
    return D.d_R / RT_M;
  }
  if (nt == 64) LOCRET_SCORE_LAUNCH(true, 64); else LOCRET_SCORE_LAUNCH(true, 128);
#undef LOCRET_SCORE_LAUNCH
  launch_kernel(score_finish_kernel, dim3(T), dim3(FIN_THREADS), 0, st, (const float*)zpart, n_z, T, D.d_R, W2f,
                     D.h_kv, part, T);
  return 1;
}

}  // namespace locret
