// Chunk attention (Eq. 1) on the bf16 matrix cores of gfx950, head_dim 128, with K and V tiles
// staged global -> LDS directly (buffer_load ... lds, 16 bytes per lane): no staging registers,
// no LDS stores, no register transposes, and a ring of tiles deep enough to cover memory latency.
//
// Products as in attention_bf16.hip: S^T = K Q^T and O^T += V^T P^T with v_mfma_f32_32x32x16_bf16,
// one wavefront = 32 queries of one head, all wavefronts of a workgroup on one KV head.
//
// Softmax with as little vector-ALU work as the arithmetic allows (the matrix pipe and the vector
// ALU overlap only partly, so every VALU instruction per tile costs time): the queries are scaled
// by scale * log2(e) when they are loaded, and the S chain starts from an accumulator that holds
// -(running max), so the MFMA result is already the exponent; per tile the VALU then only does the
// 32 exp2, 16 bf16 packs and 32 adds (v_dot2c over the packed pairs would halve the adds, but it
// shares the matrix pipe and queues behind the other wavefront's MFMAs).  The running max moves only
// on the first tile and when a lane's probability sum reaches 2^8: no row max is formed otherwise.
//
// This kernel lets its wavefronts run freely between barriers; attention_pp.hip is the same kernel
// with the two wavefronts of a SIMD held in anti-phase, and is the one launched by default.
//
// LDS layout of one ring stage (32 KB): K tile then V tile, both [64 keys][128 dims] row-major,
// 256 bytes per row, no padding.  A direct load writes lane L's 16 bytes at base + 16 L, i.e. one
// instruction fills 4 rows; conflicts are avoided by choosing WHICH 16-byte chunk a lane fetches:
//   K: position c' of row r holds chunk c' ^ (r & 15).  A fragment (key row = lane % 32, chunk
//      2 ks + hi) is one 16-byte read at position chunk ^ (row & 15): 16 consecutive rows hit 16
//      different positions.
//   V: position c' of row r holds chunk c' ^ ((r & 3) << 2).  The A operand of the PV product needs,
//      per lane, 8 keys of ONE dim: two ds_read_b64_tr_b16 (transposing 8-byte reads) fetch keys
//      kc*16 + hi*4 + 0..3 and kc*16 + 8 + hi*4 + 0..3, which is the key order the S accumulator
//      registers already have.  In a group of 16 lanes, lane s reads 8 bytes at row (base + s/4),
//      dims (16-dim block) + 4 (s % 4); the hardware hands lane i dim (block + i) of the four rows.
//      The swizzle moves the four rows of such a read into four different 64-byte bank groups.
// Every address is a per-lane constant XOR / plus a compile-time term, precomputed once.
//
// Ring: with 4 stages a pair of tiles is computed per barrier while the next pair is in flight;
// with 2 stages one tile per barrier.  A wavefront waits for its own loads (s_waitcnt vmcnt(0)),
// passes a bare s_barrier (a fenced barrier would be the same here, but the loads must be issued
// right after it and stay in flight across the compute that follows), starts the loads into the
// stages just vacated, and computes.  Tiles past the staged slots are fetched through an empty
// buffer descriptor: they arrive as zeros without touching memory.
#include <hip/hip_ext.h>

#include "attn_common.h"
#include "kernels.h"

namespace locret {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr int DM_D = 128;
constexpr int DM_TILE_B = KT * DM_D * 2;       // 16 KB per operand tile
constexpr int DM_STAGE_B = 2 * DM_TILE_B;      // K then V

template <int NW, int NSTAGE>
__global__ __launch_bounds__(NW * 64, 2) void attn_dma_kernel(const bf16_t* __restrict__ q, const float2* __restrict__ tab, const bf16_t* __restrict__ Kx,
                                                              const bf16_t* __restrict__ V, bf16_t* __restrict__ out,
                                                              int Tn, int h, int g, int cap, int n_c_common, float c_log2,
                                                              int hpw, int n_hgroups, int n_ttiles, HeadLens n_c_h) {
  constexpr int D = DM_D;
  constexpr int NKS = D / 16;
  constexpr int NDB = D / 32;
  constexpr int LPW = 32 / NW;                 // direct loads per wavefront per tile (16 K + 16 V instructions)
  __shared__ __attribute__((aligned(1024))) unsigned char ring[NSTAGE * DM_STAGE_B];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31;
  const int hi = lane >> 5;

  const int bid = blockIdx.x;
  int hgroup, tt;
  if ((n_hgroups & 7) == 0) {                  // one KV head per XCD (workgroup ids go round the XCDs)
    const int g8 = n_hgroups >> 3;
    hgroup = (bid & 7) * g8 + (bid >> 3) % g8;
    tt = bid / n_hgroups;
  } else {
    hgroup = bid % n_hgroups;
    tt = bid / n_hgroups;
  }
  tt = n_ttiles - 1 - tt;                      // longest key ranges first
  const int wph = NW / hpw;
  const int TW = wph * 32;
  const int t0 = tt * TW;
  const int j = hgroup * hpw + wave / wph;
  const int m = (hgroup * hpw) / g;
  const int n_c = __builtin_amdgcn_readfirstlane(head_len(n_c_h, m, n_c_common));   // this KV head's cache length
  const int tw0 = t0 + (wave % wph) * 32;
  const int t_last_wg = min(Tn, t0 + TW) - 1;
  const int n_keys = n_c + t_last_wg + 1;
  const int n_tiles = (n_keys + KT - 1) / KT;
  const int wave_last_slot = n_c + min(Tn - 1, tw0 + 31);
  const int my_t = min(tw0 + n32, Tn - 1);
  const int limit = n_c + my_t;

  auto scalar_ptr = [](const bf16_t* p) -> const bf16_t* {
    uint64_t a = (uint64_t)p;
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    uint32_t hi32 = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return (const bf16_t*)(((uint64_t)hi32 << 32) | lo);
  };
  const bf16_t* Kb = scalar_ptr(Kx + (int64_t)m * cap * D);
  const bf16_t* Vb = scalar_ptr(V + (int64_t)m * cap * D);

  bf16x8 qf[NKS];
  {
    const bf16_t* qp = q + ((int64_t)my_t * h + j) * D + hi * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const bf16x8*)(qp + ks * 16);
    const float qscale = c_log2;                 // logits come out of the MFMA in log2 units
    if (tab != nullptr) {
      // un-rotated queries: rotate to position n_c + t here (pairs (i, i + D/2) sit in fragments ks
      // and ks + NKS/2 of the same lane), round to bf16 as the append kernel would have
      const float2* tp = tab + (int64_t)(n_c + my_t) * (D / 2) + hi * 8;
#pragma unroll
      for (int ks = 0; ks < NKS / 2; ++ks) {
        float lo[8], up[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float2 cs = tp[ks * 16 + e];
          const float a = (float)qf[ks][e], b = (float)qf[ks + NKS / 2][e];
          lo[e] = (a * cs.x - b * cs.y) * qscale;
          up[e] = (b * cs.x + a * cs.y) * qscale;
        }
        uint4 pl = make_uint4(pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]), pack_bf16(lo[4], lo[5]), pack_bf16(lo[6], lo[7]));
        uint4 pu = make_uint4(pack_bf16(up[0], up[1]), pack_bf16(up[2], up[3]), pack_bf16(up[4], up[5]), pack_bf16(up[6], up[7]));
        qf[ks] = __builtin_bit_cast(bf16x8, pl);
        qf[ks + NKS / 2] = __builtin_bit_cast(bf16x8, pu);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (float)qf[ks][e] * qscale;
        uint4 px = make_uint4(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7]));
        qf[ks] = __builtin_bit_cast(bf16x8, px);
      }
    }
  }
  f32x16 oacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_run = 0.f, l_run = 0.f;
  // m_run is in log2 units and negm holds -m_run in all 16 registers: the first MFMA of every S
  // chain takes it as its addend, so the accumulator ends as (logit - running max) and exp2 applies
  // to it directly.  `fresh` (wave-uniform) is true until the first tile has set the max.
  f32x16 negm;
#pragma unroll
  for (int r = 0; r < 16; ++r) negm[r] = 0.f;
  bool fresh = true;

  // ---- direct loads: instruction i of a tile covers rows 4i .. 4i+3; wavefront w issues
  // ---- instructions w, w + NW, ... so (i & 3) is the same for all of them -------------------------
  const int l_row = lane >> 4, l_pos = lane & 15;
  const int k_vo = l_row * 256 + ((l_pos ^ l_row ^ ((wave & 3) << 2)) * 16);   // + i * 1024
  const int v_vo = l_row * 256 + ((l_pos ^ (l_row << 2)) * 16);                // + i * 1024
  auto issue = [&](int tile, int stage) {
    const int tile_u = __builtin_amdgcn_readfirstlane(tile);
    const int left = __builtin_amdgcn_readfirstlane(max(n_keys - tile_u * KT, 0) * (D * 2));   // 0 past the end
    __amdgpu_buffer_rsrc_t kr =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Kb + (int64_t)tile_u * (KT * D)), 0, left, 0x00020000);
    __amdgpu_buffer_rsrc_t vr =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Vb + (int64_t)tile_u * (KT * D)), 0, left, 0x00020000);
    unsigned char* sb = ring + stage * DM_STAGE_B;
#pragma unroll
    for (int u = 0; u < LPW / 2; ++u) {
      const int i = wave + u * NW;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, (lds_ptr_t)(sb + i * 1024), 16, k_vo + i * 1024, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < LPW / 2; ++u) {
      const int i = wave + u * NW;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(vr, (lds_ptr_t)(sb + DM_TILE_B + i * 1024), 16, v_vo + i * 1024, 0, 0, 0);
    }
  };

  // ---- fragment addresses (bytes inside a stage) ---------------------------------------------------
  // K: row kb*32 + n32, chunk (2 ks + hi) ^ (n32 & 15)  ==  kb_base ^ (ks << 5)
  const int kx = n32 & 15;
  const int k_base = n32 * 256 + ((kx >> 1) << 5) + ((hi ^ (kx & 1)) << 4);
  int k_rd[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) k_rd[ks] = k_base ^ (ks << 5);
  // V: 16-lane group G = lane / 16 (dims block (G & 1) * 16, keys + (G >> 1) * 4), s = lane % 16
  const int vs = lane & 15, vG = lane >> 4;
  const int v_base = DM_TILE_B + (((vG >> 1) * 4 + (vs >> 2)) * 256) + ((vs >> 2) << 6) +
                     ((((vG & 1) << 1) + ((vs & 3) >> 1)) << 4) + ((vs & 1) << 3);
  int v_rd[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) v_rd[db] = v_base ^ (db << 6);

  auto compute_tile = [&](int tile, int stage) {
    const int base = tile * KT;
    if (base > wave_last_slot) return;
    const unsigned char* sb = ring + stage * DM_STAGE_B;
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) sacc[kb] = negm;   // the S chain starts from -(running max)
    {
      bf16x8 kf[NKS][2];
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) kf[ks][kb] = *(const bf16x8*)(sb + k_rd[ks] + kb * 32 * 256);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
          sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks][kb], qf[ks], sacc[kb], 0, 0, 0);
      constexpr int AHEAD = 6;
      __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
      for (int i = 0; i < 2 * NKS - AHEAD; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
    }
    if (base + KT - 1 > n_c + tw0) {           // wave-uniform: tile crosses the diagonal
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int slot = base + kb * 32 + (r >> 2) * 8 + hi * 4 + (r & 3);
          if (slot > limit) sacc[kb][r] = -INFINITY;
        }
    }
    uint4 pb[4];
    {
      // The accumulator holds (logit - running max) in log2 units: exponentiate, pack to bf16, and sum.
      float ps;
      auto exp_pack_sum = [&]() {
        float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          uint32_t w[8];
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            const float e0 = __builtin_amdgcn_exp2f(sacc[kb][r]), e1 = __builtin_amdgcn_exp2f(sacc[kb][r + 1]);
            w[r >> 1] = pack_bf16(e0, e1);
            ps0 += e0;
            ps1 += e1;
          }
          pb[kb * 2 + 0] = make_uint4(w[0], w[1], w[2], w[3]);
          pb[kb * 2 + 1] = make_uint4(w[4], w[5], w[6], w[7]);
        }
        ps = ps0 + ps1;
      };
      exp_pack_sum();
      // The running max is only moved when it has to be: on the first tile, and when some lane's sum
      // over its 32 keys reaches 2^RESCALE_LOG2 (any probability that large, an overflow included,
      // shows there).  No row max is formed on the common path.  Rare path: take the row max, raise
      // the running max by it, scale sum and accumulator, refresh negm, correct this tile's logits
      // (formed against the old max) and redo its probabilities.
      if (fresh || __any(!(ps < 256.f))) {
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
        mx = max_across_halves(mx);
        const float delta = fresh ? mx : fmaxf(mx, 0.f);
        const float alpha = fresh ? 0.f : __builtin_amdgcn_exp2f(-delta);   // nothing accumulated yet when fresh
        m_run += delta;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
#pragma unroll
        for (int r = 0; r < 16; ++r) negm[r] = -m_run;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[kb][r] -= delta;
        fresh = false;
        exp_pack_sum();
      }
      l_run += ps;
    }
    {
      // V^T fragments: two transposing 8-byte reads each (keys +0..3 and +8..11 of the 16-key chunk)
      bf16x8 vf[4][NDB];
#pragma unroll
      for (int kc = 0; kc < 4; ++kc)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(sb + v_rd[db] + kc * 4096));
          s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(sb + v_rd[db] + kc * 4096 + 2048));
          typedef short s16x8 __attribute__((ext_vector_type(8)));
          s16x8 both = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
          vf[kc][db] = __builtin_bit_cast(bf16x8, both);
        }
#pragma unroll
      for (int kc = 0; kc < 4; ++kc)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kc][db], *(const bf16x8*)&pb[kc], oacc[db], 0, 0, 0);
      constexpr int AHEAD = 6;                  // fragments (two reads each) in flight
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * AHEAD, 1);
#pragma unroll
      for (int i = 0; i < 4 * NDB - AHEAD; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 1);
    }
  };

  // ---- ring ---------------------------------------------------------------------------------------
  if constexpr (NSTAGE == 4) {
    // Two tiles per barrier: tiles 2p, 2p+1 are computed while 2p+2, 2p+3 are in flight.  At the top
    // of a pair all of this wavefront's loads (issued one pair earlier) must have landed; after the
    // barrier the two stages read during the previous pair are free for the pair after next.
    issue(0, 0);
    issue(1, 1);
    for (int t = 0; t < n_tiles; t += 4) {
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
      issue(t + 2, 2);
      issue(t + 3, 3);
      compute_tile(t, 0);
      if (t + 1 < n_tiles) compute_tile(t + 1, 1);
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
      issue(t + 4, 0);
      issue(t + 5, 1);
      if (t + 2 < n_tiles) compute_tile(t + 2, 2);
      if (t + 3 < n_tiles) compute_tile(t + 3, 3);
    }
  } else {
    static_assert(NSTAGE == 2, "ring depths: 2 (one tile per barrier) or 4 (two tiles per barrier)");
    issue(0, 0);
    for (int t = 0; t < n_tiles; t += 2) {
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
      issue(t + 1, 1);
      compute_tile(t, 0);
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
      issue(t + 2, 0);
      if (t + 1 < n_tiles) compute_tile(t + 1, 1);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // trailing empty loads

  // ---- epilogue ---------------------------------------------------------------------------------
  {
    const int t = tw0 + n32;
    float l = l_run + __shfl_xor(l_run, 32, 64);
    if (t < Tn) {
      const float inv = 1.f / l;
      bf16_t* op = out + ((int64_t)t * h + j) * D;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          uint2 w;
          w.x = pack_bf16(oacc[db][rq * 4 + 0] * inv, oacc[db][rq * 4 + 1] * inv);
          w.y = pack_bf16(oacc[db][rq * 4 + 2] * inv, oacc[db][rq * 4 + 3] * inv);
          *(uint2*)(op + db * 32 + rq * 8 + hi * 4) = w;
        }
    }
  }
}

template <int NW, int NSTAGE>
static void dma_launch(const Dims& Dm, LaunchTimer tm, const void* q, const float2* tab, const void* Kx, const void* V, void* out, int T, int n_c,
                       float scale, hipStream_t st, const HeadLens& hl) {
  const int g = Dm.g;
  const int hpw = (NW == 8 && g % 8 == 0) ? 8 : (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
  const int wph = NW / hpw;
  const int TW = wph * 32;
  const int n_hgroups = Dm.h / hpw;
  const int n_ttiles = (T + TW - 1) / TW;
  const float c_log2 = scale * 1.4426950408889634f;
  hipExtLaunchKernelGGL((attn_dma_kernel<NW, NSTAGE>), dim3(n_hgroups * n_ttiles), dim3(NW * 64), 0, st, tm.start, tm.stop, 0,
                     (const bf16_t*)q, tab, (const bf16_t*)Kx, (const bf16_t*)V, (bf16_t*)out, T, Dm.h, g, Dm.cap, n_c,
                     c_log2, hpw, n_hgroups, n_ttiles, hl);
}

// `tab` non-null: q holds un-rotated queries and the kernel rotates them (table row n_c + t).
// variant 0: 8 wavefronts, 4-stage ring (one workgroup per CU); 1: 4 wavefronts, 2-stage ring (two per CU)
bool launch_attention_bf16_dma(const Dims& Dm, int variant, LaunchTimer tm, const void* q, const float2* tab, const void* Kx, const void* V, void* out,
                               int T, int n_c, float scale, hipStream_t st, const HeadLens* n_c_h) {
  const HeadLens hl = head_lens_or_common(n_c_h);
  if (Dm.d != DM_D) return false;
  if ((int64_t)Dm.cap * Dm.d * 2 >= (1ll << 31)) return false;   // 32-bit byte offsets inside one head
  if (variant == 1) dma_launch<4, 2>(Dm, tm, q, tab, Kx, V, out, T, n_c, scale, st, hl);
  else dma_launch<8, 4>(Dm, tm, q, tab, Kx, V, out, T, n_c, scale, st, hl);
  return true;
}

}  // namespace locret
