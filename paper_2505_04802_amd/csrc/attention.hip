// Tile-local multi-head self-attention (ORBIT-2 Sec. 4.2): for every sample, tile
// and head, O = softmax(Q K^T / sqrt(dh)) V over the tokens of that tile only.
// The paper relies on a cache-blocked ("Flash") attention library (Sec. 4.4); the
// kernel below is written for gfx950 from the arithmetic itself.
//
// bf16 kernel.  The unit of work is 128 queries of one (sample, tile, head); each of
// the four waves of a work-group owns 32 of them.  Keys/values are visited in blocks
// of BKV rows that go from global memory straight into LDS.  Scores are computed
// TRANSPOSED, S^T = K Q^T, with MFMA 32x32x16: a lane then owns one query column
// and the softmax row statistics are in-lane reductions plus one exchange between
// the two lane halves.  The rows of the K operand are read in a permuted order
// chosen so that the accumulator registers of S^T are, without any data movement,
// the B operand (P^T) of the second MFMA, O^T = V^T P^T.  Online softmax in fp32
// with base-2 exponentials; P is rounded to bf16 for PV.  Units are numbered so the
// query blocks that share one K/V set run on one XCD (one L2).
#include <type_traits>

#include "attention_common.h"

namespace reslim {

// ------------------------------------------------------------------ bf16 kernel
// Data movement.  K and V blocks are loaded with global_load_lds_dwordx4 (no
// register staging), two stages deep with one barrier per block, both ROW-MAJOR; a
// direct load cannot pad rows, so the 16-byte chunks of a row are XOR-swizzled on
// the global-address side.  K rows use swzK (conflict-free for the 16-byte
// fragment reads, 16 lanes = 256 B per LDS cycle).  The V^T operand is read with
// ds_read_b64_tr_b16: within 16 lanes, lane i receives element i of each of the
// four 16-element rows the lanes 4r..4r+3 point at, i.e. four consecutive keys of
// feature column i -- the transpose happens in the LDS read.  Per 32 lanes that
// read touches 4 chunks of 4 consecutive rows; rows r and r+2 (dh = 64; all four
// rows at dh = 128) would hit the same banks, so V rows use their own swizzle swzV
// that moves the chunk group by row.  The address of a direct load is one uniform
// base per block plus a per-lane 32-bit offset.  Keys past the end of a ragged tile
// re-read the last valid row (finite data; their probabilities are exactly zero).
//
// Softmax bookkeeping with few vector instructions per score (at dh = 64 the fp32
// vector pipe, not the matrix pipe, is the scarcer one):
//  * every S^T accumulator chain starts from `minit` = -(reference logit of this
//    lane's query), so the MFMA already delivers logit - reference;
//  * the reference is only moved (and O, L rescaled) when some query of the wave
//    meets a logit more than TAU above it -- rare after the first block -- so the
//    common block costs one max3 per three scores, one exp2 and half a convert
//    per score;
//  * the row sums L come from the bf16 probabilities the P V product uses, two per
//    v_dot2c_f32_bf16 into one register per lane (a block of ones through the matrix
//    pipe gives the same sums for a fifth of the matrix instructions at dh = 64).
// QS: the caller has already multiplied q by log2(e)/sqrt(dh) (the fused QKV
// epilogue does, before its single rounding to bf16), so the MFMA output is the
// base-2 logit itself.
//
// Scheduling.  Work-groups are PERSISTENT: the grid holds MINW work-groups per
// compute unit and each walks over its share of the units.  The K/V pipeline is
// flattened over units -- block 0 of the next unit (and its Q fragments) is in
// flight while the last block of the current one is computed.  O^T leaves the
// registers with 8-byte stores, one query row per lane (no staging, no extra
// barrier).  Measured on MI355X (c1, dh = 64): 64-key blocks with three waves per
// SIMD (156 VGPRs) beat 128-key blocks with two (0.097 vs 0.102 ms per launch).
// ST: stitched output -- a query that its tile owns writes its patch's row of a [batch, N, D]
// output, halo queries write nothing, and units or waves without an owned query are skipped (they
// still take part in the loads and barriers of their work-group).
template <int DH, int BKV, bool QS, int MINW = 2, bool ST = false, int PQK = 1, int PPV = 1>
__global__ __launch_bounds__(256, MINW) void tiles_attention_bf16_kernel(AttnArgs a) {
  constexpr int BQ = 128;
  constexpr int ROWB = DH * 2;            // bytes per K/V row in LDS
  constexpr int CPR = DH / 8;             // 16-byte chunks per row (8 or 16)
  constexpr int RPB = 64 / CPR;           // rows per 1 KiB load block
  constexpr int TILE_B = BKV * ROWB;
  constexpr int STAGE = 2 * TILE_B;       // K block then V block
  constexpr int LPW = TILE_B / 1024 / 4;  // direct loads per wave and operand
  constexpr int NKT = BKV / 32, NKS = DH / 16, NDT = DH / 32;
  constexpr bool PIPE = DH == 64 && NKT == 2;   // second key group's softmax woven into the first group's P V
  static_assert(TILE_B % 4096 == 0 && 2 * STAGE <= 65536, "LDS plan");
  __shared__ __align__(1024) unsigned char smem[2 * STAGE];

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // uniform: keeps LDS destinations in scalar registers
  const int l32 = lane & 31, hi = lane >> 5;
  const int ld = 3 * a.D;
  const int G = gridDim.x;
  auto swzK = [](int r) { return CPR == 8 ? ((r & 7) ^ ((r >> 3) & 1)) : (r & 15); };
  auto swzV = [](int r) {
    return CPR == 8 ? ((((r >> 1) & 1) << 2) | (((r >> 3) & 1) << 1)) : (((r & 3) << 2) | (((r >> 3) & 1) << 1));
  };

  // ---- work units (all of this is uniform over the work-group)
  struct Unit { int n_t, q0, nkb, tile; const bf16_t *base; bf16_t *out; float *lse; };
  // stitched output: first and last query of a tile that the tile owns (its tokens are row-major
  // over the haloed box)
  auto owned_range = [&](int tile, int &lo, int &up) {
    const tile_desc &td = a.tiles[tile];
    const int bw = td.X1 - td.X0;
    lo = (td.y0 - td.Y0) * bw + (td.x0 - td.X0);
    up = (td.y1 - 1 - td.Y0) * bw + (td.x1 - 1 - td.X0);
  };
  auto decode = [&](int vb, Unit &u) -> int {      // first non-empty unit at or after vb (stride G), or >= total
    while (vb < a.total) {
      const int logical = xcd_remap_attn(vb, a.total);
      const int qb = logical % a.QB;
      int rest = logical / a.QB;
      const int head = rest % a.heads;
      rest /= a.heads;
      const int tile = rest % a.T;
      const int b = rest / a.T;
      const int n_t = a.tiles[tile].n_tok;
      bool wanted = qb * BQ < n_t;
      if constexpr (ST) {
        int lo, up;
        owned_range(tile, lo, up);
        wanted = wanted && qb * BQ <= up && qb * BQ + BQ - 1 >= lo;
      }
      if (wanted) {
        const size_t row0 = static_cast<size_t>(b) * a.n_h + a.tiles[tile].tok_off;
        u.n_t = n_t;
        u.tile = tile;
        u.q0 = qb * BQ;
        u.nkb = (n_t + BKV - 1) / BKV;
        u.base = static_cast<const bf16_t *>(a.qkv) + row0 * ld + head * DH;
        u.out = static_cast<bf16_t *>(a.out) + (ST ? static_cast<size_t>(b) * a.N : row0) * a.D + head * DH;
        u.lse = (ST || !a.lse) ? nullptr : a.lse + (static_cast<size_t>(b) * a.heads + head) * a.n_h + a.tiles[tile].tok_off;
        return vb;
      }
      vb += G;
    }
    return vb;
  };
  Unit cur, nxt;
  int vb = decode(blockIdx.x, cur);
  if (vb >= a.total) return;
  // stitched output: a wave whose 32 queries are all halo copies does no arithmetic
  bool wave_owns = true;
  auto set_wave_owns = [&]() {
    if constexpr (ST) {
      int lo, up;
      owned_range(cur.tile, lo, up);
      const int wq0 = cur.q0 + wave * 32;
      wave_owns = wq0 <= up && wq0 + 31 >= lo;
    }
  };
  set_wave_owns();
  vb = decode(vb + G, nxt);
  bool has_next = vb < a.total;

  // ---- load side: lane -> (row of the block, 16-byte chunk), per-lane byte offsets
  int ld_row[LPW], offK[LPW], offV[LPW];
  const int ld2 = ld * 2;
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    ld_row[i] = (wave + 4 * i) * RPB + lane / CPR;
    offK[i] = ld_row[i] * ld2 + ((lane % CPR) ^ swzK(ld_row[i])) * 16;
    offV[i] = ld_row[i] * ld2 + ((lane % CPR) ^ swzV(ld_row[i])) * 16 + a.D * 2;
  }
  auto issue = [&](const Unit &u, int kv0, int buf) {
    unsigned char *sk = smem + buf * STAGE;
    const unsigned char *gk = reinterpret_cast<const unsigned char *>(u.base + a.D + static_cast<size_t>(kv0) * ld);
    const int lim = u.n_t - 1 - kv0;
    if (lim >= BKV - 1) {                // whole block inside the tile (uniform): offsets need no arithmetic
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        attn_dl_load16(reinterpret_cast<const bf16_t *>(gk + static_cast<uint32_t>(offK[i])), sk + (wave + 4 * i) * 1024);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(gk + static_cast<uint32_t>(offV[i])),
                       sk + TILE_B + (wave + 4 * i) * 1024);
      }
    } else {                             // rows past the tile end re-read its last row (finite, masked later)
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const int back = max(ld_row[i] - lim, 0) * ld2;
        attn_dl_load16(reinterpret_cast<const bf16_t *>(gk + static_cast<uint32_t>(offK[i] - back)), sk + (wave + 4 * i) * 1024);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(gk + static_cast<uint32_t>(offV[i] - back)),
                       sk + TILE_B + (wave + 4 * i) * 1024);
      }
    }
  };
  bf16x8 qf[NKS];
  auto load_q = [&](const Unit &u) {
    const int qrow = min(u.q0 + wave * 32 + l32, u.n_t - 1);
    const bf16_t *qp = u.base + static_cast<size_t>(qrow) * ld + hi * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
  };

  // ---- read side
  // K fragment: A-operand row l32 carries key key_perm(l32) of its 32-key group.
  // V^T fragment through the transposing read: this lane points at key row
  // 8*hi + 4*e + (lane%16)/4 of a 16-key step and at the 4 features
  // 32*dt + 16*((lane/16)&1) + 4*(lane%4) .. +3
  const int kr = key_perm(l32);
  const int k_row = kr * ROWB, k_swz = swzK(kr);
  const int L16 = lane & 15;
  int v_addr[2][NDT];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int vr = 8 * hi + 4 * e + (L16 >> 2);
#pragma unroll
    for (int d = 0; d < NDT; ++d) {
      const int o = 32 * d + 16 * ((lane >> 4) & 1) + 4 * (L16 & 3);
      v_addr[e][d] = TILE_B + vr * ROWB + (((o >> 3) ^ swzV(vr)) << 4) + ((o >> 2) & 1) * 8;
    }
  }

  f32x16 o[NDT], minit;
  // Sum of this lane's probabilities (its query, its half of the keys), taken from the same bf16
  // values the P V product uses, two per instruction (v_dot2c_f32_bf16 against a pair of ones).
  // A block of ones through the matrix unit gives the same sums but costs a fifth of the matrix
  // instructions at head dimension 64 and sixteen registers; the two key halves meet at the end.
  float lsum;
  auto rowsum = [](const bf16x8 &p, float acc) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 one2 = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bf16x2 pr = {p[2 * i], p[2 * i + 1]};
      acc = __builtin_amdgcn_fdot2_f32_bf16(pr, one2, acc, false);
    }
    return acc;
  };
  const float c = QS ? 1.0f : a.scale_log2;     // MFMA output -> base-2 logit
  const float TAU = 10.0f / c;                    // in units of the MFMA output
  bool have_ref = false;
  auto reset = [&]() {
#pragma unroll
    for (int d = 0; d < NDT; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) minit[r] = 0.f;
    lsum = 0.f;
    have_ref = false;
  };
  reset();
  load_q(cur);
  issue(cur, 0, 0);

  int kb = 0;
  for (int g = 0;; ++g) {
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's loads of block g (and earlier stores) are done
    __syncthreads();                        // ... and everybody's; the other buffer is free
    const bool last = kb + 1 == cur.nkb;
    if (!last) issue(cur, (kb + 1) * BKV, (g + 1) & 1);
    else if (has_next) issue(nxt, 0, (g + 1) & 1);
    const unsigned char *st = smem + (g & 1) * STAGE;
    const int kv0 = kb * BKV;
    const bool active = cur.q0 + wave * 32 < cur.n_t && wave_owns;   // wave-uniform

    f32x16 s[NKT];
    if (active) {
      // The MFMA phases run at raised wave priority, the softmax arithmetic at the default one: a
      // wave whose operands are ready gets the matrix pipe ahead of the vector work of the other
      // waves on its SIMD (c1, same box: 0.0882 -> 0.0862 ms; no effect on the gradient kernels or
      // the GEMMs, where it was tried too).  At dh = 64 the two phases get DIFFERENT levels (scores
      // 2, P V 1; c3 shapes, same box: 3.47-3.51 ms with 1 / 1, 3.43-3.44 with 2 / 1, 1 / 2 or
      // 3 / 1, 3.50 with 2 / 2, 3.62 with the P V phase at the default level, 3.76 with none).
      __builtin_amdgcn_s_setprio(PQK);
      // feature step outermost: consecutive MFMAs belong to different accumulator chains
      if constexpr (DH <= 128) {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
          for (int kt = 0; kt < NKT; ++kt) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(st + kt * 32 * ROWB + k_row + (((2 * ks + hi) ^ k_swz) << 4));
            s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? minit : s[kt], 0, 0, 0);
          }
        }
      } else {
        // dh = 256 runs one wave per SIMD: the fragment reads go PF steps ahead of the MFMAs that
        // use them (ring of PF + 1 register sets; a scheduling barrier per step keeps that order),
        // so a wave hides its own LDS latency (1.87 -> 1.75 ms for the 10B model's block; with the
        // two waves per SIMD of dh = 128 the same ring gains nothing)
        constexpr int PF = 2, NSTEP = NKS * NKT;
        bf16x8 kf[PF + 1];
        auto fetch = [&](int i) {
          const int ks = i / NKT, kt = i % NKT;
          kf[i % (PF + 1)] = *reinterpret_cast<const bf16x8 *>(st + kt * 32 * ROWB + k_row + (((2 * ks + hi) ^ k_swz) << 4));
        };
#pragma unroll
        for (int i = 0; i < PF; ++i) fetch(i);
#pragma unroll
        for (int i = 0; i < NSTEP; ++i) {
          if (i + PF < NSTEP) fetch(i + PF);
          const int ks = i / NKT, kt = i % NKT;
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % (PF + 1)], qf[ks], ks == 0 ? minit : s[kt], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    __builtin_amdgcn_s_setprio(0);
    // the query fragments are dead after the last block of a unit: fetch the next unit's
    if (last && has_next) load_q(nxt);
    if (active) {
      if (kv0 + BKV > cur.n_t) {           // ragged last block: keys past the tile end get -inf
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kv0 + kt * 32 + 16 * (r / 8) + 8 * hi + (r % 8);
            if (key >= cur.n_t) s[kt][r] = -INFINITY;
          }
      }
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
      {
        // Exchange between the two lane halves with v_permlane32_swap, not through LDS:
        // an LDS lane permute makes the wave wait on the LDS counter, and that wait
        // also covers the direct-to-LDS loads of the next block just issued (measured:
        // the prefetch stops being asynchronous).
        unsigned m_lo, m_up;
        lane_pair_exchange(__builtin_bit_cast(unsigned, mx), m_lo, m_up);
        mx = fmaxf(__builtin_bit_cast(float, m_lo), __builtin_bit_cast(float, m_up));   // finite: every block holds a valid key
      }
      if (!have_ref || __any(mx > TAU)) {
        // move this lane's reference up by d (first block: to the block maximum)
        const float d = have_ref ? fmaxf(mx, 0.f) : mx;
        const float alpha = have_ref ? __builtin_amdgcn_exp2f(-d * c) : 0.f;
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[kt][r] -= d;
#pragma unroll
        for (int dd = 0; dd < NDT; ++dd)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dd][r] *= alpha;
        const float ninit = minit[0] - d;
#pragma unroll
        for (int r = 0; r < 16; ++r) minit[r] = ninit;
        lsum *= alpha;
        have_ref = true;
      }
      if constexpr (!PIPE) {
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            s[kt][r] = __builtin_amdgcn_exp2f(QS ? s[kt][r] : s[kt][r] * c);
      }

      __builtin_amdgcn_s_setprio(PPV);
      if constexpr (PIPE) {
        // The exponentials and conversions of the second 32-key group are placed between the
        // matrix instructions of the first group's P V product: a wave issues in order, so its own
        // vector work only overlaps its matrix work when the two are interleaved in the stream.
        const unsigned st_off = static_cast<unsigned>(reinterpret_cast<uintptr_t>(
            (__attribute__((address_space(3))) const unsigned char *)st));
        unsigned va[2][2];
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
          for (int d = 0; d < 2; ++d) va[e][d] = st_off + static_cast<unsigned>(v_addr[e][d]);
        typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
        // the first group's V reads are issued ahead of its exponentials, which cover their latency
        VFrag64 vf0, vf1;
        v_frag_issue<0>(vf0, va);
#pragma unroll
        for (int r = 0; r < 16; ++r) s[0][r] = __builtin_amdgcn_exp2f(QS ? s[0][r] : s[0][r] * c);
        bf16x8 pf0[2], pf1[2];
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
          for (int e = 0; e < 8; ++e) pf0[h2][e] = static_cast<__bf16>(s[0][8 * h2 + e]);
        v_frag_wait(vf0);
        v_frag_issue<32 * ROWB>(vf1, va);     // in flight under the whole first group
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          lsum = rowsum(pf0[h2], lsum);
#pragma unroll
          for (int d = 0; d < 2; ++d) {
            const u64x2 both = {vf0.r[h2][d][0], vf0.r[h2][d][1]};
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf0[h2], o[d], 0, 0, 0);
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) s[1][r] = __builtin_amdgcn_exp2f(QS ? s[1][r] : s[1][r] * c);
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
          for (int e = 0; e < 8; ++e) pf1[h2][e] = static_cast<__bf16>(s[1][8 * h2 + e]);
        // one matrix instruction, then six vector instructions, four times (16 exponentials + 8 conversions)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        v_frag_wait(vf1);
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          lsum = rowsum(pf1[h2], lsum);
#pragma unroll
          for (int d = 0; d < 2; ++d) {
            const u64x2 both = {vf1.r[h2][d][0], vf1.r[h2][d][1]};
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf1[h2], o[d], 0, 0, 0);
          }
        }
      } else if constexpr (DH == 64) {
        // LDS byte addresses of this lane's four fragment pointers in the current stage
        const unsigned st_off = static_cast<unsigned>(reinterpret_cast<uintptr_t>(
            (__attribute__((address_space(3))) const unsigned char *)st));
        unsigned va[2][2];
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
          for (int d = 0; d < 2; ++d) va[e][d] = st_off + static_cast<unsigned>(v_addr[e][d]);
        auto group = [&](auto kt_c) {
          constexpr int kt = decltype(kt_c)::value;
          VFrag64 vf;
          v_frag_issue<kt * 32 * ROWB>(vf, va);
          bf16x8 pf[2];
#pragma unroll
          for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[h2][e] = static_cast<__bf16>(s[kt][8 * h2 + e]);
          v_frag_wait(vf);
#pragma unroll
          for (int h2 = 0; h2 < 2; ++h2) {
            lsum = rowsum(pf[h2], lsum);
#pragma unroll
            for (int d = 0; d < 2; ++d) {
              typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
              const u64x2 both = {vf.r[h2][d][0], vf.r[h2][d][1]};
              o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[h2], o[d], 0, 0, 0);
            }
          }
        };
        group(std::integral_constant<int, 0>{});
        group(std::integral_constant<int, 1>{});
        if constexpr (NKT == 4) {
          group(std::integral_constant<int, 2>{});
          group(std::integral_constant<int, 3>{});
        }
      } else if constexpr (DH <= 128) {
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
#pragma unroll
          for (int h2 = 0; h2 < 2; ++h2) {
            bf16x8 pf;
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[e] = static_cast<__bf16>(s[kt][8 * h2 + e]);
            lsum = rowsum(pf, lsum);
#pragma unroll
            for (int d = 0; d < NDT; ++d) {
              const unsigned char *vp = st + (kt * 32 + h2 * 16) * ROWB;
              const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (s16x4 __attribute__((address_space(3))) *)(vp + v_addr[0][d]));
              const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (s16x4 __attribute__((address_space(3))) *)(vp + v_addr[1][d]));
              typedef __attribute__((ext_vector_type(8))) short s16x8;
              const s16x8 both = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
              const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
              o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[d], 0, 0, 0);
            }
          }
        }
      } else {
        // the same ring for the transposed V fragments of P V: step = (key group, half, feature block)
        constexpr int PF = 2, NSTEP = NKT * 2 * NDT;
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        s16x4 vlo[PF + 1], vhi[PF + 1];
        auto fetch = [&](int i) {
          const int d = i % NDT, h2 = (i / NDT) % 2, kt = i / (2 * NDT);
          const unsigned char *vp = st + (kt * 32 + h2 * 16) * ROWB;
          vlo[i % (PF + 1)] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(vp + v_addr[0][d]));
          vhi[i % (PF + 1)] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(vp + v_addr[1][d]));
        };
#pragma unroll
        for (int i = 0; i < PF; ++i) fetch(i);
        bf16x8 pf;
#pragma unroll
        for (int i = 0; i < NSTEP; ++i) {
          if (i + PF < NSTEP) fetch(i + PF);
          const int d = i % NDT, h2 = (i / NDT) % 2, kt = i / (2 * NDT);
          if (d == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[e] = static_cast<__bf16>(s[kt][8 * h2 + e]);
            lsum = rowsum(pf, lsum);
          }
          const s16x8 both = __builtin_shufflevector(vlo[i % (PF + 1)], vhi[i % (PF + 1)], 0, 1, 2, 3, 4, 5, 6, 7);
          o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf, o[d], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    __builtin_amdgcn_s_setprio(0);
    if (!last) { ++kb; continue; }

    // ---- end of a unit: normalise and store this lane's query row, then move on
    const int qrow = cur.q0 + wave * 32 + l32;
    int orow = qrow;
    bool keep = true;
    if constexpr (ST) {                    // the query's patch, if this tile owns it
      const tile_desc &td = a.tiles[cur.tile];
      const int bw = td.X1 - td.X0;
      const int yy = td.Y0 + qrow / bw, xx = td.X0 + qrow % bw;
      keep = yy >= td.y0 && yy < td.y1 && xx >= td.x0 && xx < td.x1;
      orow = yy * a.Wp + xx;
    }
    if (active && qrow < cur.n_t) {
      // lanes l and l + 32 hold the two key halves of query l: full sum = own + partner
      unsigned l_lo, l_up;
      lane_pair_exchange(__builtin_bit_cast(unsigned, lsum), l_lo, l_up);
      const float ltot = __builtin_bit_cast(float, l_lo) + __builtin_bit_cast(float, l_up);
      const float inv = 1.0f / ltot;
      // log-sum-exp of the logits (kept for the gradient): reference + log of the sum
      if (!ST && cur.lse && hi == 0) cur.lse[qrow] = (__builtin_amdgcn_logf(ltot) - minit[0] * c) * 0.69314718055994531f;
      bf16_t *op = cur.out + static_cast<size_t>(orow) * a.D + hi * 4;
      if (keep) {
#pragma unroll
        for (int d = 0; d < NDT; ++d)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            // registers 4*r4 .. 4*r4+3 hold features 32d + 8*r4 + 4*hi + (0..3) of query l32
            bf16x4 tmp;
#pragma unroll
            for (int e = 0; e < 4; ++e) tmp[e] = static_cast<__bf16>(o[d][4 * r4 + e] * inv);
            *reinterpret_cast<u32x2 *>(op + d * 32 + r4 * 8) = __builtin_bit_cast(u32x2, tmp);
          }
      }
    }
    if (!has_next) break;
    cur = nxt;
    set_wave_owns();
    vb = decode(vb + G, nxt);
    has_next = vb < a.total;
    kb = 0;
    reset();
  }
}

// ------------------------------------------------------------------ fp32 debug path
// One work-group per (sample, tile-major token, head): scores for all keys of the
// tile in LDS, two block reductions, then one thread per feature accumulates P V.
__global__ __launch_bounds__(128) void tiles_attention_f32_kernel(AttnArgs a, int dh, const int32_t *tile_of_tok) {
  extern __shared__ float sm[];
  float *sc = sm;              // [max_n_tok]
  float *qv = sm + a.QB;       // [dh]   (QB carries max_n_tok here)
  __shared__ float red[128];
  const int64_t tok = blockIdx.x;
  const int head = blockIdx.y, b = blockIdx.z;
  const int tile = tile_of_tok[tok];
  const int n_t = a.tiles[tile].n_tok;
  const int64_t tok_off = a.tiles[tile].tok_off;
  const int ld = 3 * a.D;
  const float *base = static_cast<const float *>(a.qkv) + (static_cast<size_t>(b) * a.n_h + tok_off) * ld + head * dh;
  const float *qrow = static_cast<const float *>(a.qkv) + (static_cast<size_t>(b) * a.n_h + tok) * ld + head * dh;
  const int t = threadIdx.x;
  for (int d = t; d < dh; d += 128) qv[d] = qrow[d];
  __syncthreads();
  const float scale = rsqrtf(static_cast<float>(dh));
  float mx = -INFINITY;
  for (int j = t; j < n_t; j += 128) {
    const float *kr = base + a.D + static_cast<size_t>(j) * ld;
    float s = 0.f;
    for (int d = 0; d < dh; ++d) s = fmaf(qv[d], kr[d], s);
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  red[t] = mx;
  __syncthreads();
  for (int w = 64; w > 0; w >>= 1) {
    if (t < w) red[t] = fmaxf(red[t], red[t + w]);
    __syncthreads();
  }
  mx = red[0];
  __syncthreads();
  float sum = 0.f;
  for (int j = t; j < n_t; j += 128) {
    const float p = expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  red[t] = sum;
  __syncthreads();
  for (int w = 64; w > 0; w >>= 1) {
    if (t < w) red[t] += red[t + w];
    __syncthreads();
  }
  const float inv = 1.0f / red[0];
  if (a.lse && t == 0) a.lse[(static_cast<size_t>(b) * a.heads + head) * a.n_h + tok] = mx + logf(red[0]);
  float *orow = static_cast<float *>(a.out) + (static_cast<size_t>(b) * a.n_h + tok) * a.D + head * dh;
  for (int d = t; d < dh; d += 128) {
    const float *vc = base + 2 * a.D + d;
    float acc = 0.f;
    for (int j = 0; j < n_t; ++j) acc = fmaf(sc[j], vc[static_cast<size_t>(j) * ld], acc);
    orow[d] = acc * inv;
  }
}

// 0: 64-key blocks, three work-groups per CU at dh = 64 (default); 1: 128-key blocks, two per CU
static int g_attn_variant = 0;
static int g_attn_cus = 0;

hipError_t attention_init() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  return hipDeviceGetAttribute(&g_attn_cus, hipDeviceAttributeMultiprocessorCount, dev);
}
bool attention_accepts_prescaled_q() { return true; }

SeqGeom ctx_geom(const reslim_ctx *c) {
  SeqGeom g;
  g.d_tiles = c->d_tiles;
  g.d_tile_of_tok = c->d_tile_of_tok;
  g.T = c->T;
  g.n_h = c->n_h;
  g.max_n_tok = c->max_n_tok;
  g.pairs = 0;
  g.pairs_owned = 0;
  for (const tile_desc &t : c->tiles) {
    g.pairs += static_cast<double>(t.n_tok) * t.n_tok;
    g.pairs_owned += static_cast<double>(t.y1 - t.y0) * (t.x1 - t.x0) * t.n_tok;
  }
  return g;
}

// PQK, PPV: wave priority during the score and the P V matrix instructions
template <int DH, int BKV, int MINW, int PQK = 1, int PPV = 1>
static void launch_bf16_variant(const AttnArgs &a, bool q_prescaled, bool stitched, int grid, hipStream_t st) {
  if (stitched) {
    if (q_prescaled) tiles_attention_bf16_kernel<DH, BKV, true, MINW, true, PQK, PPV><<<dim3(grid), dim3(256), 0, st>>>(a);
    else tiles_attention_bf16_kernel<DH, BKV, false, MINW, true, PQK, PPV><<<dim3(grid), dim3(256), 0, st>>>(a);
  } else {
    if (q_prescaled) tiles_attention_bf16_kernel<DH, BKV, true, MINW, false, PQK, PPV><<<dim3(grid), dim3(256), 0, st>>>(a);
    else tiles_attention_bf16_kernel<DH, BKV, false, MINW, false, PQK, PPV><<<dim3(grid), dim3(256), 0, st>>>(a);
  }
}

hipError_t launch_tiles_attention(const reslim_ctx *c, const void *qkv, void *out, int batch, bool q_prescaled,
                                  hipStream_t st, float *lse, const SeqGeom *geom, bool stitched) {
  const SeqGeom own = geom ? *geom : ctx_geom(c);
  const SeqGeom &sg = own;
  AttnArgs a;
  a.qkv = qkv;
  a.out = out;
  a.lse = lse;
  a.tiles = sg.d_tiles;
  a.T = sg.T;
  a.heads = c->cfg.heads;
  a.D = c->cfg.embed_dim;
  a.n_h = sg.n_h;
  a.scale_log2 = 1.4426950408889634f / sqrtf(static_cast<float>(c->dh));
  a.Wp = 0;
  a.N = 0;
  if (stitched) {                          // the context's own tiling, bf16 kernel, no log-sum-exp rows
    if (geom || lse || c->cfg.dtype != RESLIM_BF16) return hipErrorInvalidValue;
    a.Wp = c->Wp;
    a.N = c->N;
  }
  if (c->cfg.dtype == RESLIM_BF16) {
    a.QB = (sg.max_n_tok + 127) / 128;
    const int64_t total = static_cast<int64_t>(batch) * sg.T * a.heads * a.QB;
    if (total > INT32_MAX) return hipErrorInvalidValue;
    a.total = static_cast<int>(total);
    if (a.total == 0) return hipSuccess;
    if (g_attn_cus <= 0) return hipErrorInvalidValue;
    const int pg2 = a.total < 2 * g_attn_cus ? a.total : 2 * g_attn_cus;   // persistent grids
    const int pg3 = a.total < 3 * g_attn_cus ? a.total : 3 * g_attn_cus;
    if (c->dh == 64 && g_attn_variant == 0) launch_bf16_variant<64, 64, 3, 2, 1>(a, q_prescaled, stitched, pg3, st);
    else if (c->dh == 64) launch_bf16_variant<64, 128, 2>(a, q_prescaled, stitched, pg2, st);
    else if (c->dh == 128) launch_bf16_variant<128, 64, 2>(a, q_prescaled, stitched, pg2, st);
    else if (c->dh == 256) {
      // 128 output-accumulator and 64 query-fragment registers per lane: one work-group per CU
      const int pg1 = a.total < g_attn_cus ? a.total : g_attn_cus;
      launch_bf16_variant<256, 32, 1>(a, q_prescaled, stitched, pg1, st);
    } else {
      return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  a.QB = sg.max_n_tok;
  a.total = 0;
  const size_t lds = (static_cast<size_t>(sg.max_n_tok) + c->dh) * sizeof(float);
  if (lds > 60 * 1024 || sg.n_h > INT32_MAX) return hipErrorInvalidValue;
  tiles_attention_f32_kernel<<<dim3(static_cast<unsigned>(sg.n_h), a.heads, batch), dim3(128), lds, st>>>(
      a, c->dh, sg.d_tile_of_tok);
  return hipGetLastError();
}

}  // namespace reslim

// tuning hook for dh = 64: 0 = 64-key blocks, three work-groups per CU (default), 1 = 128-key blocks, two per CU
extern "C" void reslim_debug_set_attention_variant(int v) { reslim::g_attn_variant = v; }
