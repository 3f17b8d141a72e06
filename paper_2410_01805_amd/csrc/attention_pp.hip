// Chunk attention (Eq. 1) on the bf16 matrix cores of gfx950, head_dim 128 (and 96): K and V tiles go
// global -> LDS directly (buffer_load ... lds), and the two wavefronts of every SIMD are held in anti-phase.
//
// Products are formed transposed with v_mfma_f32_32x32x16_bf16: S^T = K Q^T (A = 32 key rows from LDS, B = the
// wavefront's 32 queries, held in registers for the whole kernel, pre-scaled by scale * log2 e and rotated),
// O^T += V^T P^T (A = V^T from LDS through the transposing read ds_read_b64_tr_b16, B = P^T straight from the S
// accumulator registers: a lane holds 16 keys of ONE query there, so row sums are per-lane scalars and P needs
// no shuffle).  A tile is 64 keys x 128 dims of K and of V, rows of 256 bytes.  A direct load writes lane L's
// 16 bytes at base + 16 L, so rows cannot be padded; bank conflicts are avoided by choosing WHICH 16-byte
// chunk a lane fetches: position c' of K row r holds chunk c' ^ (r & 15), of V row r chunk c' ^ ((r & 3) << 2).
// Tiles past the end are fetched through a zero-length buffer descriptor (they arrive as zeros).
// Softmax: every S chain starts from an accumulator holding -(running max), so the MFMA result is the exponent;
// the running max is set by the first tile and raised only when a lane's probability sum over its 32 keys
// reaches 2^30 (which also catches any overflow).
//
// A wavefront's tile is a chain S (16 MFMAs) -> softmax (32 exp2 on the transcendental unit, ~640
// cycles) -> PV (16 MFMAs).  Left alone, the two wavefronts of a SIMD drift into the same phase:
// the older one wins every arbitration, runs its chain at full speed, and the younger one finishes
// a pair of tiles ~30 % later, mostly alone on the SIMD with the matrix pipe idle during its softmax.
// Here wavefronts 0..3 (group A, one per SIMD) and 4..7 (group B, their SIMD mates) are
// offset by one S block with two workgroup barriers per tile:
//
//      barrier X(t) | A: S(t)                    | barrier Y(t) | A: softmax, PV, prefetch K frags of t+1
//                   | B: loads of t+3, K frags t |              | B: S(t), softmax, PV
//
// so the matrix pipe sees S_A, S_B, PV_A, PV_B back to back while each softmax runs beside the
// other group's MFMAs.  Group B issues all direct loads (8 per wavefront per tile) in the slot in
// which it waits for A's S block; group A uses its slot at the end of the tile to fetch the first K
// fragments of the next one.  A passes Y four MFMAs before the end of its S block (all its fragment reads
// are out by then), so B's first MFMAs queue behind A's last ones instead of meeting an idle pipe.
//
// The first workgroups of the launch can carry the step's selection (and the sum of the retaining head's
// partial scores before it): see the kernel body and select_body.h.
//
// Ring of 4 stages, one tile per step.  Invariant at X(t): tiles t and t+1 have landed in LDS (B waits
// for its own loads of tile t+2 before it arrives at X(t+1): s_waitcnt vmcnt(8) leaves only the 8 loads
// of tile t+3 in flight) and every wavefront has finished tile t-1, whose stage the loads of tile t+3
// overwrite.
//
// The V^T fragments are read with ds_read_b64_tr_b16 from inline assembly, with hand-counted
// s_waitcnt lgkmcnt: the compiler puts an s_waitcnt vmcnt(0) in front of the intrinsic form (it
// cannot tell that those reads never touch a stage with a load in flight), which would stall every
// PV block on the loads just issued.  LDS operations return in order, so a count of the asm reads
// issued after the wanted one is always sufficient, whatever else the compiler has in flight.
#include <hip/hip_ext.h>

#include "attn_common.h"
#include "kernels.h"
#include "select_body.h"

namespace locret {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(3))) unsigned char* lds_u8_ptr;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int PP_ROWB = 256;                   // bytes of a key's row in LDS: 128 bf16; head_dim 96 leaves the last quarter unused
constexpr int PP_TILE_B = KT * PP_ROWB;        // 16 KB per operand tile
constexpr int PP_STAGE_B = 2 * PP_TILE_B;      // K then V
constexpr int PP_NW = 8;
constexpr int PP_KPRE = 4;                     // K fragments fetched ahead of the S block
constexpr int PP_VPRE = 4;                     // V^T fragments in flight ahead of their MFMA
constexpr int PP_YTAIL = 4;                    // MFMAs of group A's S block issued behind barrier Y
constexpr int PP_SEL_MAXR = 48;                // keys per thread of a selection workgroup (512 threads)
constexpr int PP_MAX_SPLIT = 8;                // key ranges per (head group, token tile) item at most
constexpr int PP_SPLIT_TOKENS = 2048;          // token rows (times splits) the partial-result buffer holds at most

#define LOCRET_TR_READ(dst, addr, off) \
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(off) : "memory")
#define LOCRET_LGKM_WAIT(a, b, n) asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "i"(n))

// GENERAL = false is the common case: every KV head holds n_c_common units, one KV head per XCD, the whole key
// range per workgroup (n_c_h, spread_arg, order, n_split_arg and part_arg are ignored, so nothing of head-wise
// lengths, the spread launch order or the key split remains in its code).
// D = 128 or 96.  The tile layout in LDS is that of 128 dims for both (rows of 256 bytes): with 96 dims the lanes
// of a direct load that would fetch the last four 16-byte chunks of a row point outside the buffer instead and
// bring zeros, which nothing reads; every fragment address stays as it is, S takes 6 contraction steps and O^T
// has 3 blocks of 32 dims.
template <int D, bool GENERAL>
__global__ __launch_bounds__(PP_NW * 64, 2) void attn_pp_kernel(const bf16_t* __restrict__ q, const float2* __restrict__ tab, const bf16_t* __restrict__ Kx,
                                                             const bf16_t* __restrict__ V, bf16_t* __restrict__ out,
                                                             int Tn, int h, int g, int cap, int n_c_common, float c_log2,
                                                             int hpw, int n_hgroups, int n_ttiles, SelectArgs sel, int n_sel,
                                                             HeadLens n_c_h, int spread_arg, HeadOrder order,
                                                             int n_split_arg, float* __restrict__ part_arg) {
  const int n_split = GENERAL ? n_split_arg : 1;
  float* const part = GENERAL ? part_arg : nullptr;
  const int spread = GENERAL ? spread_arg : 0;
  constexpr int NW = PP_NW;
  static_assert(D == 128 || D == 96, "head dims of this kernel");
  constexpr int NKS = D / 16;
  constexpr int NDB = D / 32;
  __shared__ __attribute__((aligned(1024))) unsigned char ring[4 * PP_STAGE_B];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31;
  const int hi = lane >> 5;

  // The first n_sel workgroups of the launch do not attend: each runs the top-k selection of one KV head
  // (it depends on the scores only, which are complete before the launch) and retires after a few tens
  // of microseconds, long before the attention workgroups that follow it on the same CU would have started
  // their second round; the selection's latency disappears from the step.
  if ((int)blockIdx.x < n_sel) {
    select_reg_body<PP_SEL_MAXR, PP_NW * 64, 4>(sel, blockIdx.x, (uint32_t*)ring);
    static_assert(select_body_smem_words(PP_NW * 64, 4) * 4 <= (int)sizeof(ring), "the selection's scratch fits the ring");
    return;
  }
  const int bid = blockIdx.x - n_sel;
  int hgroup, tt;
  if (spread) {
    // Head-wise budgets: with one KV head per XCD the XCD of the longest head would set the launch's time.
    // Instead every XCD takes every eighth token tile of every head, the heads from the longest cache to
    // the shortest, so that all XCDs hold the same work and each hands out its long items first.
    // (Measured on 8 heads of 28672 ... 4096 units, mean 16384: 1.61 ms per step with one head per XCD,
    // 1.39 ms with the heads interleaved item by item, 1.14 ms in this order; equal heads 1.07 ms.)
    const int i = bid >> 3, per_head = (n_ttiles + 7) >> 3;
    const int r = i / per_head;                            // rank of the head group, longest first
    const int gph = g / hpw;                               // head groups per KV head
    hgroup = order.v[r / gph] * gph + r % gph;
    tt = (i % per_head) * 8 + (bid & 7);
    if (tt >= n_ttiles) return;                            // the launch is padded to whole rounds of the 8 XCDs
  } else if ((n_hgroups & 7) == 0) {                  // one KV head per XCD (workgroup ids go round the XCDs)
    const int g8 = n_hgroups >> 3;
    hgroup = (blockIdx.x & 7) * g8 + (bid >> 3) % g8;
    tt = bid / n_hgroups;
  } else {
    hgroup = bid % n_hgroups;
    tt = bid / n_hgroups;
  }
  // n_split > 1: n_ttiles counts (token tile, key split) pairs, the split being the fast index
  const int split = tt % n_split;
  tt = n_ttiles / n_split - 1 - tt / n_split;  // longest key ranges first
  const int wph = NW / hpw;
  const int TW = wph * 32;
  const int t0 = tt * TW;
  const int j = hgroup * hpw + wave / wph;
  const int m = (hgroup * hpw) / g;
  const int n_c = GENERAL ? __builtin_amdgcn_readfirstlane(head_len(n_c_h, m, n_c_common)) : n_c_common;   // this KV head's cache length
  const int tw0 = t0 + (wave % wph) * 32;
  const int t_last_wg = min(Tn, t0 + TW) - 1;
  const int n_keys = n_c + t_last_wg + 1;
  const int n_tiles_all = (n_keys + KT - 1) / KT;
  // Key split (short chunks leave most CUs without a workgroup otherwise): this workgroup takes the key tiles
  // [t_lo, t_lo + n_tiles) of its queries' range and leaves un-normalised partial results for the merge kernel.
  const int per_split = (n_tiles_all + n_split - 1) / n_split;
  const int t_lo = split * per_split;
  const int n_tiles = max(0, min(n_tiles_all, t_lo + per_split) - t_lo);
  const int n_keys_s = min(n_keys, (t_lo + n_tiles) * KT);
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

  const bool isB = wave >= NW / 2;             // wave-uniform; wavefronts w and w + 4 share a SIMD

  // ---- direct loads (group B): instruction i of a tile covers rows 4i .. 4i+3; wavefront w issues
  // ---- instructions w%4 + 4u, so (i & 3) is the same for all of them ----------------------------------
  const int w4 = wave & 3;
  const int l_row = lane >> 4, l_pos = lane & 15;
  // the lane's LDS slot is row 4 i + l_row, position l_pos; the row's swizzle decides which chunk of the row in
  // memory belongs there.  Memory rows are D * 2 bytes; instruction i = w4 + 4 u starts at row 16 u + 4 w4.
  constexpr int NCH = D / 8;                     // 16-byte chunks of a row in memory
  constexpr int OUTSIDE = 0x7ffff000;            // an offset no buffer reaches: the load brings zeros
  const int k_ch = l_pos ^ l_row ^ (w4 << 2), v_ch = l_pos ^ (l_row << 2);
  const int k_vo = k_ch < NCH ? (w4 * 4 + l_row) * (D * 2) + k_ch * 16 : OUTSIDE;   // + u * 16 rows (scalar offset)
  const int v_vo = v_ch < NCH ? (w4 * 4 + l_row) * (D * 2) + v_ch * 16 : OUTSIDE;
  auto issue = [&](int tile, int stage) __attribute__((always_inline)) {
    const int tile_u = __builtin_amdgcn_readfirstlane(tile);
    const int left = __builtin_amdgcn_readfirstlane(max(n_keys_s - tile_u * KT, 0) * (D * 2));   // 0 past the end
    __amdgpu_buffer_rsrc_t kr =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Kb + (int64_t)tile_u * (KT * D)), 0, left, 0x00020000);
    __amdgpu_buffer_rsrc_t vr =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Vb + (int64_t)tile_u * (KT * D)), 0, left, 0x00020000);
    unsigned char* sb = ring + stage * PP_STAGE_B;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = w4 + u * 4;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, (lds_ptr_t)(sb + i * 1024), 16, k_vo, u * (16 * D * 2), 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = w4 + u * 4;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(vr, (lds_ptr_t)(sb + PP_TILE_B + i * 1024), 16, v_vo, u * (16 * D * 2), 0, 0);
    }
  };

  // ---- fragment addresses (bytes inside a stage) ---------------------------------------------------
  const int kx = n32 & 15;
  const int k_base = n32 * 256 + ((kx >> 1) << 5) + ((hi ^ (kx & 1)) << 4);
  int k_rd[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) k_rd[ks] = k_base ^ (ks << 5);
  const int vs = lane & 15, vG = lane >> 4;
  const int v_base = PP_TILE_B + (((vG >> 1) * 4 + (vs >> 2)) * 256) + ((vs >> 2) << 6) +
                     ((((vG & 1) << 1) + ((vs & 3) >> 1)) << 4) + ((vs & 1) << 3);
  // LDS byte addresses of stage 0 for the asm reads
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(lds_u8_ptr)ring;
  uint32_t v_ad[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) v_ad[db] = ring_lds + (uint32_t)(v_base ^ (db << 6));

  bf16x8 kpre[PP_KPRE];                          // fragment f = ks * 2 + kb of the tile whose S block comes next
  auto prefetch_k = [&](int sb_off) __attribute__((always_inline)) {
    const unsigned char* sb = ring + sb_off;
#pragma unroll
    for (int f = 0; f < PP_KPRE; ++f) kpre[f] = *(const bf16x8*)(sb + k_rd[f >> 1] + (f & 1) * 32 * 256);
  };

  // `mid` runs before the last `tail` MFMAs are issued (all fragment reads are out by then)
  auto s_block = [&](f32x16 (&sacc)[2], int sb_off, auto mid, auto tail_c) __attribute__((always_inline)) {
    constexpr int TAIL = decltype(tail_c)::value;    // 0: no split
    const unsigned char* sb = ring + sb_off;
    bf16x8 kf[NKS][2];
#pragma unroll
    for (int f = 0; f < 2 * NKS; ++f)
      kf[f >> 1][f & 1] = f < PP_KPRE ? kpre[f] : *(const bf16x8*)(sb + k_rd[f >> 1] + (f & 1) * 32 * 256);
#pragma unroll
    for (int f = 0; f < 2 * NKS - TAIL; ++f)
      sacc[f & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[f >> 1][f & 1], qf[f >> 1], f < 2 ? negm : sacc[f & 1], 0, 0, 0);   // the S chain starts from -(running max)
#pragma unroll
    for (int i = 0; i < 2 * NKS - PP_KPRE; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    if (TAIL < PP_KPRE) __builtin_amdgcn_sched_group_barrier(0x008, PP_KPRE - TAIL, 0);
    if (TAIL > 0) {
      mid();
#pragma unroll
      for (int f = 2 * NKS - TAIL; f < 2 * NKS; ++f)
        sacc[f & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[f >> 1][f & 1], qf[f >> 1], sacc[f & 1], 0, 0, 0);
    }
  };

  // softmax and PV of one tile; the S accumulators are in sacc
  auto softmax_pv = [&](f32x16 (&sacc)[2], int tile, int sb_off) __attribute__((always_inline)) {
    const int base = tile * KT;
    uint32_t va[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db) va[db] = v_ad[db] + (uint32_t)sb_off;
    // V^T fragment f = kc * NDB + db: two transposing 8-byte reads (keys +0..3 and +8..11 of the 16-key chunk)
    s16x4 vlo[4 * NDB], vhi[4 * NDB];
#pragma unroll
    for (int f = 0; f < PP_VPRE; ++f) {
      LOCRET_TR_READ(vlo[f], va[f % NDB], (f / NDB) * 4096);
      LOCRET_TR_READ(vhi[f], va[f % NDB], (f / NDB) * 4096 + 2048);
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
      float ps;
      auto exp_pack_sum = [&]() __attribute__((always_inline)) {
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
      if (fresh || __any(!(ps < RESCALE_SUM))) {     // rare: set or raise the running max
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
        mx = max_across_halves(mx);
        // Key-split launches only: in the split that holds the diagonal a query may see none of the split's keys
        // (its row of the first tile is wholly masked, and every later tile lies further right).  Such a lane keeps
        // max 0 and sum 0, and the merge kernel drops partials whose sum is 0; without the test it would form
        // -inf - (-inf).  In unsplit launches every query sees key 0, which lies in the first tile.
        const float delta = fresh ? ((GENERAL && mx == -INFINITY) ? 0.f : mx) : fmaxf(mx, 0.f);
        const float alpha = fresh ? 0.f : __builtin_amdgcn_exp2f(-delta);
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
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int f = 0; f < 4 * NDB; ++f) {
      constexpr int LASTF = 4 * NDB - 1;
      const int newest = f + PP_VPRE - 1 < LASTF ? f + PP_VPRE - 1 : LASTF;   // newest fragment already requested
      // reads issued after fragment f's: two per fragment
      static_assert(PP_VPRE <= 6, "lgkmcnt cases");
      switch (2 * (newest - f)) {
        case 10: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 10); break;
        case 8: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 8); break;
        case 6: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 6); break;
        case 4: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 4); break;
        case 2: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 2); break;
        default: LOCRET_LGKM_WAIT(vlo[f], vhi[f], 0); break;
      }
      const s16x8 both = __builtin_shufflevector(vlo[f], vhi[f], 0, 1, 2, 3, 4, 5, 6, 7);
      oacc[f % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), *(const bf16x8*)&pb[f / NDB],
                                                              oacc[f % NDB], 0, 0, 0);
      if (f + PP_VPRE < 4 * NDB) {
        const int fn = f + PP_VPRE;
        LOCRET_TR_READ(vlo[fn], va[fn % NDB], (fn / NDB) * 4096);
        LOCRET_TR_READ(vhi[fn], va[fn % NDB], (fn / NDB) * 4096 + 2048);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  auto wg_barrier = []() __attribute__((always_inline)) {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };

  // tiles this wavefront's queries can see (wave-uniform, <= n_tiles): later tiles only keep the barriers
  const int n_active = max(0, min(n_tiles, wave_last_slot / KT + 1 - t_lo));
  if (isB) {
    issue(t_lo, 0);
    issue(t_lo + 1, 1);
    issue(t_lo + 2, 2);
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");            // tiles 0 and 1 have landed
    wg_barrier();
    for (int t = 0; t < n_active; ++t) {
      const int sb_off = (t & 3) * PP_STAGE_B;
      wg_barrier();                                              // X(t)
      issue(t_lo + t + 3, (t + 3) & 3);
      prefetch_k(sb_off);
      wg_barrier();                                              // Y(t)
      f32x16 sacc[2];
      s_block(sacc, sb_off, []() {}, IntC<0>());
      softmax_pv(sacc, t_lo + t, sb_off);
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");          // own loads of tile t+2 have landed
    }
    for (int t = n_active; t < n_tiles; ++t) {
      wg_barrier();
      issue(t_lo + t + 3, (t + 3) & 3);
      wg_barrier();
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    }
  } else {
    wg_barrier();
    prefetch_k(0);
    for (int t = 0; t < n_active; ++t) {
      const int sb_off = (t & 3) * PP_STAGE_B;
      wg_barrier();                                              // X(t)
      f32x16 sacc[2];
      s_block(sacc, sb_off, wg_barrier, IntC<PP_YTAIL>());        // Y(t), passed PP_YTAIL MFMAs before the end of the block
      softmax_pv(sacc, t_lo + t, sb_off);
      prefetch_k(((t + 1) & 3) * PP_STAGE_B);
    }
    for (int t = n_active; t < n_tiles; ++t) {
      wg_barrier();
      wg_barrier();
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // trailing empty loads

  // ---- epilogue ---------------------------------------------------------------------------------
  {
    const int t = tw0 + n32;
    float l = l_run + __shfl_xor(l_run, 32, 64);
    if (part != nullptr) {
      // partial result of this key split: O un-normalised, running max (log2 units) and sum; a wavefront that saw
      // no key leaves sum 0
      if (t < Tn) {
        const int64_t row = ((int64_t)split * Tn + t) * h + j;
        float* op = part + row * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq)
            *(float4*)(op + db * 32 + rq * 8 + hi * 4) =
                make_float4(oacc[db][rq * 4 + 0], oacc[db][rq * 4 + 1], oacc[db][rq * 4 + 2], oacc[db][rq * 4 + 3]);
        if (hi == 0) {
          float* ml = part + (int64_t)n_split * Tn * h * D + row * 2;
          *(float2*)ml = make_float2(m_run, l);
        }
      }
    } else if (t < Tn) {
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

// out[t][j][:] = sum_s w_s O_s / sum_s w_s l_s with w_s = 2^(m_s - max m) over the key splits of a row (t, j);
// a split whose sum is 0 saw no key of that row.  A thread owns 4 elements of a row.
__global__ __launch_bounds__(256) void attn_pp_merge_kernel(const float* __restrict__ part, bf16_t* __restrict__ out,
                                                            int rows, int n_split, int D) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = gid / (D / 4);
  const int e = (int)(gid % (D / 4)) * 4;
  if (row >= rows) return;
  const float* ml = part + (int64_t)n_split * rows * D;
  float M = -INFINITY;
  for (int s = 0; s < n_split; ++s) {
    const float2 x = *(const float2*)(ml + ((int64_t)s * rows + row) * 2);
    if (x.y > 0.f) M = fmaxf(M, x.x);
  }
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f, den = 0.f;
  for (int s = 0; s < n_split; ++s) {
    const float2 x = *(const float2*)(ml + ((int64_t)s * rows + row) * 2);
    if (!(x.y > 0.f)) continue;
    const float w = __builtin_amdgcn_exp2f(x.x - M);
    const float4 o = *(const float4*)(part + ((int64_t)s * rows + row) * D + e);
    den = fmaf(w, x.y, den);
    a0 = fmaf(w, o.x, a0);
    a1 = fmaf(w, o.y, a1);
    a2 = fmaf(w, o.z, a2);
    a3 = fmaf(w, o.w, a3);
  }
  const float inv = 1.f / den;      // every query sees at least its own key
  uint2 wd;
  wd.x = pack_bf16(a0 * inv, a1 * inv);
  wd.y = pack_bf16(a2 * inv, a3 * inv);
  *(uint2*)(out + row * D + e) = wd;
}

static bool pp_head_dim(int d) { return d == 128 || d == 96; }

// Floats of workspace for the partial results of key-split launches (0: this shape never splits).
size_t attention_pp_split_floats(const Dims& Dm, int chunk_max) {
  if (!pp_head_dim(Dm.d) || !Dm.bf16) return 0;
  const int tokens = chunk_max < PP_SPLIT_TOKENS / 2 ? 2 * chunk_max : PP_SPLIT_TOKENS;
  return (size_t)tokens * Dm.h * (Dm.d + 2);
}

// `tab` non-null: q holds un-rotated queries and the kernel rotates them (table row n_c + t).
bool attention_pp_fuses_select(const Dims& Dm, int n_cand) {
  if (!pp_head_dim(Dm.d) || (int64_t)Dm.cap * Dm.d * 2 >= (1ll << 31)) return false;
  const int wseg = ((n_cand + PP_NW - 1) / PP_NW + 63) & ~63;
  return wseg <= PP_SEL_MAXR * 64;
}

// `sel` non-null (and attention_pp_fuses_select true): the launch also performs that selection.
bool launch_attention_bf16_pp(const Dims& Dm, LaunchTimer tm, const void* q, const float2* tab, const void* Kx, const void* V, void* out,
                              int T, int n_c, float scale, hipStream_t st, const SelectArgs* sel,
                              const HeadLens* n_c_h, float* split_part, size_t split_floats) {
  if (!pp_head_dim(Dm.d)) return false;
  if ((int64_t)Dm.cap * Dm.d * 2 >= (1ll << 31)) return false;   // 32-bit byte offsets inside one head
  constexpr int NW = PP_NW;
  const int g = Dm.g;
  const int hpw = (g % 8 == 0) ? 8 : (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
  const int wph = NW / hpw;
  const int TW = wph * 32;
  const int n_hgroups = Dm.h / hpw;
  const int n_ttiles = (T + TW - 1) / TW;
  const float c_log2 = scale * 1.4426950408889634f;
  const int n_sel = sel ? Dm.h_kv : 0;
  const HeadLens hl = head_lens_or_common(n_c_h);
  const SelectArgs sa = sel ? *sel : SelectArgs{};
  // Key split: a short chunk has too few (head group, token tile) items for the 256 CUs (chunks of 1024 tokens of
  // a 32-head layer: 128), so each item is cut into n_split key ranges, as many as bring the launch to about one
  // workgroup per CU, and a second kernel merges the partial results.  Only while every split still has a
  // few key tiles in every head and the partials fit their buffer.  Tuning::pp_split: 0 = never,
  // k = always k ranges (bounded by the buffer only).
  int n_split = 1;
  if (split_part != nullptr) {
    const int forced = Dm.tune.pp_split;
    int min_nc = n_c;
    if (hl.ragged) for (int m = 0; m < Dm.h_kv; ++m) min_nc = hl.v[m] < min_nc ? hl.v[m] : min_nc;
    const int items = n_hgroups * n_ttiles;
    int want = forced >= 0 ? forced : 256 / items;
    want = want > PP_MAX_SPLIT ? PP_MAX_SPLIT : want;
    const int min_tiles = (min_nc + 1 + KT - 1) / KT;
    while (want > 1 && ((size_t)want * T * Dm.h * (Dm.d + 2) > split_floats || (forced < 0 && min_tiles / want < 8))) --want;
    n_split = want < 1 ? 1 : want;
  }
  const int n_tt_eff = n_ttiles * n_split;
  const int spread = (hl.ragged && Dm.tune.pp_spread != 0) || Dm.tune.pp_spread == 1;
  const int n_wg = spread ? n_hgroups * ((n_tt_eff + 7) / 8) * 8 : n_hgroups * n_tt_eff;
  float* part = n_split > 1 ? split_part : nullptr;
#define LOCRET_PP_LAUNCH(SP)                                                                                          \
  do { if (Dm.d == 96) LOCRET_PP_LAUNCH_D(96, SP); else LOCRET_PP_LAUNCH_D(128, SP); } while (0)
#define LOCRET_PP_LAUNCH_D(DD, SP)                                                                                    \
  hipExtLaunchKernelGGL((attn_pp_kernel<DD, SP>), dim3(n_sel + n_wg), dim3(NW * 64), 0, st, tm.start,                   \
                        part ? nullptr : tm.stop, 0, (const bf16_t*)q, tab, (const bf16_t*)Kx, (const bf16_t*)V,        \
                        (bf16_t*)out, T, Dm.h, g, Dm.cap, n_c, c_log2, hpw, n_hgroups, n_tt_eff, sa, n_sel, hl, spread, \
                        longest_first(hl, Dm.h_kv), n_split, part)
  if (part || spread || hl.ragged) LOCRET_PP_LAUNCH(true); else LOCRET_PP_LAUNCH(false);
#undef LOCRET_PP_LAUNCH
#undef LOCRET_PP_LAUNCH_D
  if (part) {
    const int rows = T * Dm.h;
    const int64_t threads = (int64_t)rows * (Dm.d / 4);
    hipExtLaunchKernelGGL(attn_pp_merge_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, nullptr, tm.stop, 0,
                          (const float*)part, (bf16_t*)out, rows, n_split, Dm.d);
  }
  return true;
}

}  // namespace locret
